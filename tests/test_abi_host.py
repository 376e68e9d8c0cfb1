"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, sizes workspaces, and rejects bad arguments before any device call."""
import ctypes as C
import os
import re

import pytest

import paper_1312_5766_amd as pk
from paper_1312_5766_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "strads_lasso.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(strads_lasso_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = pk.load()
    names = _declared_functions()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(pk.EXPORTS) == names


def test_ctypes_structs_match_the_header_layout(tmp_path):
    # the header, compiled by the host C compiler, reports size and field offsets of its three
    # structs; the binding's ctypes mirrors must agree field by field
    pairs = [("strads_lasso_config_t", b.Config), ("strads_round_info_t", b.RoundInfo), ("strads_run_info_t", b.RunInfo)]
    lines = ['#include <stdio.h>', '#include "strads_lasso.h"', 'int main(void) {']
    for cname, ct in pairs:
        lines.append(f'  printf("{cname} %zu\\n", sizeof({cname}));')
        for fname, _ in ct._fields_:
            cfield = {"lam": "lambda"}.get(fname, fname)
            lines.append(f'  printf("{cname}.{fname} %zu\\n", offsetof({cname}, {cfield}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    import subprocess
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)], check=True)
    out = dict(l.split() for l in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for cname, ct in pairs:
        assert int(out[cname]) == C.sizeof(ct), cname
        for fname, _ in ct._fields_:
            assert int(out[f"{cname}.{fname}"]) == getattr(ct, fname).offset, f"{cname}.{fname}"
        # and no field of the header is missing from the mirror
        text = open(os.path.join(ROOT, "include", "strads_lasso.h")).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        end = text.index("} " + cname + ";")
        body = text[text.rindex("typedef struct {", 0, end) + len("typedef struct {"):end]
        n_decl = sum(len(d.split(",")) for d in body.split(";") if d.strip())
        assert n_decl == len(ct._fields_), cname


def test_workspace_bytes_scales_and_rejects():
    small = pk.strads_lasso_workspace_bytes(1000, 5000, 200)
    big = pk.strads_lasso_workspace_bytes(10000, 100000, 1000)
    assert 0 < small < big < 1 << 30
    assert pk.strads_lasso_workspace_bytes(1000, 5000, 200, keep_gram=True) > small
    assert pk.strads_lasso_workspace_bytes(0, 5000, 200) == 0
    assert pk.strads_lasso_workspace_bytes(1000, 0, 200) == 0
    assert pk.strads_lasso_workspace_bytes(1000, 5000, 0) == 0
    assert pk.strads_lasso_workspace_bytes(1000, 5000, pk.MAX_L_PRIME + 1) == 0
    assert pk.strads_lasso_workspace_bytes(1000, 1 << 31, 200) == 0
    assert pk.load().strads_lasso_workspace_bytes(None) == 0
    # l_prime larger than j is clamped, not rejected
    assert pk.strads_lasso_workspace_bytes(100, 50, 200) == pk.strads_lasso_workspace_bytes(100, 50, 50)


def _cfg(**kw):
    base = dict(n=100, j=50, layout=0, x=256, y=256, lam=0.1, rho=0.1, eta=1e-6, c_init=1e6, l_prime=10,
                p_max=0, seed=0, keep_gram=0, workspace=256, workspace_bytes=1 << 40, stream=None)
    base.update(kw)
    return b.Config(**base)


@pytest.mark.parametrize("bad", [
    dict(n=0), dict(j=0), dict(layout=7), dict(x=None), dict(y=None), dict(workspace=None),
    dict(lam=-1.0), dict(lam=float("nan")), dict(lam=float("inf")), dict(rho=0.0), dict(rho=-0.1),
    dict(rho=float("nan")), dict(eta=0.0), dict(eta=float("nan")), dict(c_init=0.0), dict(c_init=float("inf")),
    dict(l_prime=0), dict(l_prime=pk.MAX_L_PRIME + 1), dict(p_max=-1), dict(workspace=257), dict(x=258),
    dict(layout=1, row_idx=None, col_ptr=None),
    dict(layout=2, col_mean=None, col_scale=256), dict(layout=2, col_mean=256, col_scale=None),
    dict(layout=2, col_mean=256, col_scale=256, x=264),          # packed columns start on 16-byte boundaries
    dict(deps=3), dict(priority=3), dict(loss=2), dict(loss=-1), dict(n_shards=-1), dict(n_shards=9), dict(n_shards=8, j=5),
])
def test_create_rejects_invalid_arguments_without_touching_the_device(bad):
    lib = pk.load()
    h = C.c_void_p(0x1234)
    rc = lib.strads_lasso_create(C.byref(_cfg(**bad)), C.byref(h))
    assert rc == b.E_INVALID_ARG
    assert h.value == 0x1234                    # outputs untouched on error


def test_create_reports_small_workspace_and_null_handles():
    lib = pk.load()
    h = C.c_void_p()
    assert lib.strads_lasso_create(C.byref(_cfg(workspace_bytes=1024)), C.byref(h)) == b.E_WORKSPACE_TOO_SMALL
    assert lib.strads_lasso_create(None, C.byref(h)) == b.E_INVALID_ARG
    assert lib.strads_lasso_create(C.byref(_cfg()), None) == b.E_INVALID_ARG
    assert lib.strads_lasso_round(None, None) == b.E_INVALID_ARG
    assert lib.strads_lasso_run(None, 1, 0.0, 0, None) == b.E_INVALID_ARG
    assert lib.strads_lasso_objective(None, None) == b.E_INVALID_ARG
    assert lib.strads_lasso_kkt(None, None, None) == b.E_INVALID_ARG
    assert lib.strads_lasso_set_tuning(None, b"gram_split_k", 1) == b.E_INVALID_ARG
    lib.strads_lasso_destroy(None)              # a no-op
    assert lib.strads_lasso_strerror(0) == b"ok"
    assert b"workspace" in lib.strads_lasso_strerror(b.E_WORKSPACE_TOO_SMALL)


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        b.load()


def test_debug_build_exports_the_same_symbols_and_says_what_it_is():
    path = os.path.join(ROOT, "paper_1312_5766_amd", "libstrads_lasso_debug.so")
    assert os.path.exists(path), "build it with `python -m paper_1312_5766_amd.build --debug`"
    dbg = C.CDLL(path)
    for n in _declared_functions():
        assert hasattr(dbg, n), n
    assert dbg.strads_lasso_debug_build() == 1
    assert pk.load().strads_lasso_debug_build() == (1 if os.environ.get("STRADS_LASSO_DEBUG") == "1" else 0)


def test_static_filter_rejects_bad_arguments_before_any_device_call():
    lib = pk.load()
    f = lib.strads_lasso_filter_static
    assert f(None, 2, 0.1, 0, 1, 1, None) == b.E_INVALID_ARG
    assert f(1, 0, 0.1, 0, 1, 1, None) == b.E_INVALID_ARG
    assert f(1, 2, float("nan"), 0, 1, 1, None) == b.E_INVALID_ARG
    assert f(1, 2, 0.1, -1, 1, 1, None) == b.E_INVALID_ARG
    assert f(1, b.FILTER_STATIC_MAX_L + 1, 0.1, 0, 1, 1, None) == b.E_TOO_LARGE
    assert b"maximum" in lib.strads_lasso_strerror(b.E_TOO_LARGE)


# ---------------------------------------------------------------------------------------------
# host logic of the tile kernel for long candidate lists: the queue of (tile, stage range) items
# ---------------------------------------------------------------------------------------------
def _weight(ta, tb, t, half_last):
    return 10 if ta == tb else (8 if half_last and tb == t - 1 else 16)


@pytest.mark.parametrize("n,l", [(50000, 8000), (50000, 8192), (4096, 4300), (1000, 700), (5000, 513), (4096, 128),
                                 (260, 1100), (8, 257), (33, 300), (100000, 6000)])
def test_gram256_queue_covers_every_tile_stage_once_in_shrinking_items(n, l):
    import numpy as np
    items, first, count = pk.strads_lasso_gram256_plan(n, l)
    stages, t = (n + 31) // 32, (l + 255) // 256
    half_last = t * 256 > (l + 127) // 128 * 128        # the last tile column holds 128 columns of the padded list
    cover = np.zeros((t, t, stages), np.int32)
    assert np.array_equal(items[:, 4], np.arange(len(items)))          # slots are numbered in queue order
    total = sum(_weight(a, b_, t, half_last) * stages for a in range(t) for b_ in range(a, t))
    left, prev_tile, prev_end, limit = total, None, 0, 0
    for ta, tb, s0, s1, slot in (tuple(int(v) for v in row) for row in items):
        assert 0 <= ta <= tb < t and 0 <= s0 < s1 <= stages
        cover[ta, tb, s0:s1] += 1
        w = _weight(ta, tb, t, half_last)
        # a tile's items are consecutive in the queue and in row order, so its slots are too
        if (ta, tb) != prev_tile:
            assert s0 == 0 and first[ta, tb] == slot and (prev_tile is None or prev_end == stages)
            left -= w * stages
            # guided sizes: no item is worth more than a 256th of the work queued behind its tile (32 stages
            # at least), so that the queue ends in short items whatever the workgroups' speeds
            limit = max(left // 256 // w, 32)
        else:
            assert s0 == prev_end
        prev_tile, prev_end = (ta, tb), s1
        assert first[ta, tb] <= slot < first[ta, tb] + count[ta, tb]
        assert s1 - s0 <= limit and (s1 - s0 >= limit // 2 or s1 - s0 == stages or limit == 32)
    assert left == 0 and prev_end == stages
    for a in range(t):
        for b_ in range(t):
            if a <= b_:
                assert (cover[a, b_] == 1).all(), (a, b_)
                assert count[a, b_] >= 1
            else:
                assert cover[a, b_].sum() == 0 and count[a, b_] == 0 and first[a, b_] == 0
    assert int(count.sum()) == len(items)


def test_gram256_queue_at_the_bench_shape():
    items, first, count = pk.strads_lasso_gram256_plan(50000, 8000)
    lens = items[:, 3] - items[:, 2]
    assert len(count) == 32 and count.max() <= 1563 // 32 + 1
    assert (lens[:240] == 1563).all()               # the queue starts with whole tiles, about one per workgroup
    assert lens[-200:].max() <= 32                  # the queue ends in short items
    assert 900 <= len(items) <= 2000                # tile slots: 256 KB each
    assert lens.min() >= 31


def test_gram256_plan_rejects_bad_arguments():
    n_items = C.c_int32(7)
    buf = (C.c_int32 * 5)()
    tt = (C.c_int32 * 1024)()
    lib = pk.load()
    assert lib.strads_lasso_gram256_plan(0, 100, 0, C.byref(n_items), None, tt, tt) == pk.E_INVALID_ARG
    assert lib.strads_lasso_gram256_plan(100, 0, 0, C.byref(n_items), None, tt, tt) == pk.E_INVALID_ARG
    assert lib.strads_lasso_gram256_plan(100, pk.MAX_L_PRIME + 1, 0, C.byref(n_items), None, tt, tt) == pk.E_INVALID_ARG
    assert lib.strads_lasso_gram256_plan(100, 100, -1, C.byref(n_items), buf, tt, tt) == pk.E_INVALID_ARG
    assert lib.strads_lasso_gram256_plan(100, 100, 1, C.byref(n_items), None, tt, tt) == pk.E_INVALID_ARG
    assert lib.strads_lasso_gram256_plan(100, 100, 0, None, None, tt, tt) == pk.E_INVALID_ARG
    assert lib.strads_lasso_gram256_plan(100, 100, 0, C.byref(n_items), None, None, tt) == pk.E_INVALID_ARG
    assert n_items.value == 7
    assert lib.strads_lasso_gram256_plan(100, 100, 1, C.byref(n_items), buf, tt, tt) == pk.STRADS_OK
    assert n_items.value == 1 and list(buf) == [0, 0, 0, 4, 0]


def test_default_tile_kernel_by_shape():
    """Which tile kernel forms Step 2's Gram by default (host-side rule, no GPU): the five configurations, the
    borders of the rules, and the layouts and dependency rules that have no choice."""
    edge = pk.strads_lasso_gram_default_tile_edge
    assert edge(50000, 8000) == 256                  # long list over long columns: 256-wide tiles from a queue
    assert edge(10000, 1000) == 128 and edge(1000, 200) == 128
    assert edge(500, 2000) == 64                     # short columns under a long list: 64-wide tiles, no K-slices
    assert edge(500, 2000, pk.LAYOUT_GENO2) == 64
    assert edge(4096, 4097) == 256 and edge(4096, 4096) == 128 and edge(4092, 8000) == 128
    assert edge(4094, 8000) == 128                   # columns of a length that is no multiple of 4 floats
    assert edge(50000, 2048) == 256 and edge(50000, 1024) == 128     # enough stages of work per compute unit or not
    assert edge(1024, 1024) == 64 and edge(1024, 896) == 128 and edge(1025, 1024) == 128
    assert edge(2048, 3072) == 64 and edge(2048, 2944) == 128 and edge(2049, 3072) == 128
    assert edge(500, 2000, pk.LAYOUT_DENSE, pk.DEPS_DYNAMIC) == 128  # the movers' Gram is tiled on the device
    assert edge(500, 2000, pk.LAYOUT_CSC) == 0 and edge(500, 2000, pk.LAYOUT_DENSE, pk.DEPS_NONE) == 0
    assert edge(50000, 8000, pk.LAYOUT_GENO2) == 128
    lib, out = pk.load(), C.c_int32(7)
    for bad in ((0, 10, 0, 0), (10, 0, 0, 0), (10, pk.MAX_L_PRIME + 1, 0, 0), (10, 10, 3, 0), (10, 10, -1, 0),
                (10, 10, 0, 3), (10, 10, 0, -1)):
        assert lib.strads_lasso_gram_default_tile_edge(*bad, C.byref(out)) == pk.E_INVALID_ARG
    assert lib.strads_lasso_gram_default_tile_edge(10, 10, 0, 0, None) == pk.E_INVALID_ARG
    assert out.value == 7


def test_gram_tile_edge_rejects_null_arguments():
    edge = C.c_int32(5)
    assert pk.load().strads_lasso_gram_tile_edge(None, C.byref(edge)) == pk.E_INVALID_ARG
    assert edge.value == 5
