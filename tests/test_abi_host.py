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
# host logic of the tile kernel for long candidate lists: the stream of (tile, stage) pairs cut into runs
# ---------------------------------------------------------------------------------------------
def _plan_facts(n, l, cap):
    import numpy as np
    wgs, pieces, planes = pk.strads_lasso_gram256_plan(n, l, cap)
    stages, t = (n + 31) // 32, (l + 255) // 256
    cover = np.zeros((t, t, stages), np.int32)
    seen, load = set(), np.zeros(256)
    for w in range(256):
        ended = False
        for i in range(pk.GRAM256_MAX_PIECES):
            ta, tb, s0, s1, plane = (int(v) for v in pieces[w, i])
            if s1 <= s0:
                ended = True
                continue
            assert not ended, "pieces of a workgroup are listed without gaps"
            assert w < wgs and 0 <= ta <= tb < t and 0 <= s0 < s1 <= stages
            cover[ta, tb, s0:s1] += 1
            assert (ta, tb, plane) not in seen, "two pieces of a tile share a plane"
            seen.add((ta, tb, plane))
            load[w] += (s1 - s0) * (10 if ta == tb else 16)
    return wgs, planes, cover, seen, load[:wgs], t


@pytest.mark.parametrize("n,l,cap", [(50000, 8000, 2), (50000, 8192, 2), (4096, 4300, 4), (1000, 700, 16),
                                     (5000, 513, 30), (4096, 128, 64), (260, 1100, 4), (8, 257, 1),
                                     (33, 300, 2)])
def test_gram256_plan_covers_every_tile_stage_once(n, l, cap):
    import numpy as np
    wgs, planes, cover, seen, load, t = _plan_facts(n, l, cap)
    assert 8 <= wgs <= 256 and wgs % 8 == 0
    for a in range(t):
        for b_ in range(t):
            if a <= b_:
                assert (cover[a, b_] == 1).all(), (a, b_)
                assert planes[a, b_] == sum(1 for (x, y, _) in seen if (x, y) == (a, b_))
                # a tile's planes are numbered 0 .. count-1 without gaps
                assert {p for (x, y, p) in seen if (x, y) == (a, b_)} == set(range(int(planes[a, b_])))
            else:
                assert cover[a, b_].sum() == 0 and planes[a, b_] == 0
    assert planes.max() <= cap
    # equal runs: no workgroup's share (in MFMA blocks on the busiest SIMD) differs from another's by more
    # than one stage of the heavier kind of tile
    assert load.max() - load.min() <= 16 + 10


def test_gram256_plan_at_the_bench_shape_needs_two_planes_and_all_compute_units():
    wgs, planes, cover, seen, load, t = _plan_facts(50000, 8000, 2)
    assert wgs == 256 and t == 32 and planes.max() == 2
    assert len(seen) <= 528 + 256           # every cut adds at most one piece


def test_gram256_plan_rejects_bad_arguments_and_impossible_caps():
    wgs = C.c_int32(7)
    buf = (C.c_int32 * (256 * 8 * 5))()
    pl = (C.c_int32 * 1024)()
    lib = pk.load()
    assert lib.strads_lasso_gram256_plan(0, 100, 1, C.byref(wgs), buf, pl) == pk.E_INVALID_ARG
    assert lib.strads_lasso_gram256_plan(100, 0, 1, C.byref(wgs), buf, pl) == pk.E_INVALID_ARG
    assert lib.strads_lasso_gram256_plan(100, pk.MAX_L_PRIME + 1, 1, C.byref(wgs), buf, pl) == pk.E_INVALID_ARG
    assert lib.strads_lasso_gram256_plan(100, 100, 0, C.byref(wgs), buf, pl) == pk.E_INVALID_ARG
    assert lib.strads_lasso_gram256_plan(100, 100, 1, None, buf, pl) == pk.E_INVALID_ARG
    # 15 tiles of 9 stages cannot be dealt to 8 or more workgroups in whole tiles
    assert lib.strads_lasso_gram256_plan(260, 1100, 1, C.byref(wgs), buf, pl) == pk.E_UNSUPPORTED
    assert wgs.value == 0
