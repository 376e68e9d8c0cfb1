"""Thin Python binding of libstrads_lasso.so (include/strads_lasso.h).

Argument marshalling only: every step of a round runs in the library's HIP
kernels.  PyTorch supplies device memory (the workspace and output tensors)
and the stream.  There is no CPU fallback: if the library is missing, import
of this module's entry points fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# STRADS_LASSO_DEBUG=1 selects the debug build (waits and checks after every launch; checks unit norms at create)
# STRADS_LASSO_LIB=<path> loads another build of the same library (measurements of kernel variants)
LIB_PATH = os.environ.get("STRADS_LASSO_LIB") or os.path.join(
    _HERE, "libstrads_lasso_debug.so" if os.environ.get("STRADS_LASSO_DEBUG") == "1" else "libstrads_lasso.so")

STRADS_OK = 0
E_INVALID_ARG, E_WORKSPACE_TOO_SMALL, E_HIP, E_DIVERGED, E_UNSUPPORTED, E_TOO_LARGE = -1, -2, -3, -4, -5, -6
FILTER_STATIC_MAX_L = 8192
LAYOUT_DENSE, LAYOUT_CSC, LAYOUT_GENO2 = 0, 1, 2
LOSS = {"squared": 0, "logistic": 1}
MAX_L_PRIME = 8192
N_STAGES = 7
STAGE_NAMES = ["sampler", "cand_dots", "gram_tiles", "gram_mask", "filter", "update", "residual"]
DEPS_STATIC, DEPS_DYNAMIC, DEPS_NONE = 0, 1, 2
PRIORITY = {"squared": 0, "linear": 1, "uniform": 2}

EXPORTS = [
    "strads_lasso_workspace_bytes", "strads_lasso_create", "strads_lasso_round", "strads_lasso_run",
    "strads_lasso_objective", "strads_lasso_kkt", "strads_lasso_get_state", "strads_lasso_set_state",
    "strads_lasso_last_round", "strads_lasso_last_candidates", "strads_lasso_stage_keys", "strads_lasso_stage_filter",
    "strads_lasso_set_tuning", "strads_lasso_stage_times", "strads_lasso_last_kkt_ms", "strads_lasso_destroy",
    "strads_lasso_strerror", "strads_lasso_filter_static", "strads_lasso_debug_build", "strads_lasso_gram256_plan",
    "strads_lasso_gram_tile_edge", "strads_lasso_gram_default_tile_edge",
]


class Config(C.Structure):
    _fields_ = [("n", C.c_int64), ("j", C.c_int64), ("layout", C.c_int32), ("x", C.c_void_p),
                ("row_idx", C.c_void_p), ("col_ptr", C.c_void_p), ("col_mean", C.c_void_p), ("col_scale", C.c_void_p),
                ("y", C.c_void_p),
                ("lam", C.c_float), ("rho", C.c_float), ("eta", C.c_float), ("c_init", C.c_float),
                ("l_prime", C.c_int32), ("p_max", C.c_int32), ("seed", C.c_uint64), ("keep_gram", C.c_int32),
                ("max_col_nnz", C.c_int32), ("deps", C.c_int32), ("priority", C.c_int32), ("n_shards", C.c_int32),
                ("loss", C.c_int32), ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("stream", C.c_void_p)]


class RoundInfo(C.Structure):
    _fields_ = [("round", C.c_int64), ("n_cand", C.c_int32), ("n_kept", C.c_int32), ("n_moved", C.c_int32),
                ("near_rho_pairs", C.c_int32), ("max_abs_delta", C.c_float)]


class RunInfo(C.Structure):
    _fields_ = [("rounds_done", C.c_int64), ("updates_done", C.c_int64), ("objective", C.c_double),
                ("kkt_violation", C.c_float), ("converged", C.c_int32), ("graph_replays", C.c_int32)]


_lib = None


def load():
    """dlopen the HIP library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1312_5766_amd.build` "
                           "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    L.strads_lasso_workspace_bytes.argtypes = [C.POINTER(Config)]
    L.strads_lasso_workspace_bytes.restype = C.c_size_t
    L.strads_lasso_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
    L.strads_lasso_round.argtypes = [vp, C.POINTER(RoundInfo)]
    L.strads_lasso_run.argtypes = [vp, C.c_int64, C.c_float, C.c_int32, C.POINTER(RunInfo)]
    L.strads_lasso_objective.argtypes = [vp, C.POINTER(C.c_double)]
    L.strads_lasso_kkt.argtypes = [vp, C.POINTER(C.c_float), vp]
    L.strads_lasso_get_state.argtypes = [vp, vp, vp, vp, C.POINTER(C.c_int64)]
    L.strads_lasso_set_state.argtypes = [vp, vp, vp, vp, C.c_int64]
    L.strads_lasso_last_round.argtypes = [vp, vp, vp, vp, vp, vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    L.strads_lasso_last_candidates.argtypes = [vp, vp, vp, C.POINTER(C.c_int32)]
    L.strads_lasso_stage_keys.argtypes = [vp, C.c_int64, vp]
    L.strads_lasso_stage_filter.argtypes = [vp, vp, C.c_int32, vp, C.POINTER(C.c_int32)]
    L.strads_lasso_set_tuning.argtypes = [vp, C.c_char_p, C.c_int64]
    L.strads_lasso_stage_times.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
    L.strads_lasso_filter_static.argtypes = [vp, C.c_int32, C.c_float, C.c_int32, vp, vp, vp]
    L.strads_lasso_debug_build.argtypes = []
    L.strads_lasso_gram_tile_edge.argtypes = [vp, C.POINTER(C.c_int32)]
    L.strads_lasso_gram_default_tile_edge.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
    L.strads_lasso_gram256_plan.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.POINTER(C.c_int32), vp, vp, vp]
    L.strads_lasso_destroy.argtypes = [vp]
    L.strads_lasso_destroy.restype = None
    L.strads_lasso_strerror.argtypes = [C.c_int]
    L.strads_lasso_strerror.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("strads_lasso_workspace_bytes", "strads_lasso_destroy", "strads_lasso_strerror"):
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


class StradsError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {load().strads_lasso_strerror(code).decode()} ({code})")


def _check(code: int, what: str):
    if code != STRADS_OK:
        raise StradsError(code, what)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def strads_lasso_workspace_bytes(n, j, l_prime, layout=LAYOUT_DENSE, keep_gram=False, max_col_nnz=0,
                                 dynamic=False, n_shards=0) -> int:
    cfg = Config(n=n, j=j, layout=layout, l_prime=l_prime, keep_gram=int(keep_gram), max_col_nnz=int(max_col_nnz),
                 deps=DEPS_DYNAMIC if dynamic else DEPS_STATIC, n_shards=int(n_shards))
    return int(load().strads_lasso_workspace_bytes(C.byref(cfg)))


def strads_lasso_gram_default_tile_edge(n: int, l: int, layout: int = LAYOUT_DENSE, deps: int = DEPS_STATIC) -> int:
    """Host only.  Edge of the tiles Step 2's Gram of l candidates over n rows takes by default (256, 128, 64, or 0)."""
    edge = C.c_int32(-1)
    _check(load().strads_lasso_gram_default_tile_edge(int(n), int(l), int(layout), int(deps), C.byref(edge)),
           "strads_lasso_gram_default_tile_edge")
    return int(edge.value)


def strads_lasso_gram256_plan(n: int, l: int):
    """Host only.  (items, first_slot, n_slots): items is an int32 array [n_items][5] of (tile row, tile column,
    first stage, end stage, slot) in queue order; first_slot and n_slots are int32 arrays [T][T], T = ceil(l / 256)."""
    import numpy as np
    t = (l + 255) // 256
    first, count = np.zeros((t, t), np.int32), np.zeros((t, t), np.int32)
    n_items = C.c_int32(0)
    _check(load().strads_lasso_gram256_plan(int(n), int(l), 0, C.byref(n_items), None, first.ctypes.data,
                                            count.ctypes.data), "strads_lasso_gram256_plan")
    items = np.zeros((max(1, n_items.value), 5), np.int32)
    _check(load().strads_lasso_gram256_plan(int(n), int(l), n_items.value, C.byref(n_items), items.ctypes.data,
                                            first.ctypes.data, count.ctypes.data), "strads_lasso_gram256_plan")
    return items[:n_items.value], first, count


def strads_lasso_filter_static(gram: torch.Tensor, rho: float, p_max: int, kept_pos: torch.Tensor,
                               n_kept: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """The dependency filter on a caller-supplied Gram without handle or workspace.  Every tensor is the
    caller's (gram: l x l fp32; kept_pos: >= l int32; n_kept: >= 1 int32, all on the GPU); nothing is
    allocated and nothing is waited for."""
    assert gram.is_cuda and gram.dtype == torch.float32 and gram.is_contiguous() and gram.dim() == 2
    l = gram.shape[0]
    assert gram.shape[1] == l and kept_pos.dtype == torch.int32 and n_kept.dtype == torch.int32
    assert kept_pos.is_cuda and n_kept.is_cuda and kept_pos.numel() >= l and n_kept.numel() >= 1
    s = stream if stream is not None else torch.cuda.current_stream(gram.device)
    with torch.cuda.device(gram.device):
        _check(load().strads_lasso_filter_static(_ptr(gram), l, float(rho), int(p_max), _ptr(kept_pos), _ptr(n_kept),
                                                 s.cuda_stream), "strads_lasso_filter_static")


class StradsLasso:
    """One solver handle.  Methods carry the C entry points' names without the prefix."""

    def __init__(self, y: torch.Tensor, lam: float, rho: float, eta: float, l_prime: int, seed: int = 0,
                 p_max: int = 0, c_init: float = 1e6, keep_gram: bool = False,
                 x: Optional[torch.Tensor] = None, values: Optional[torch.Tensor] = None,
                 row_idx: Optional[torch.Tensor] = None, col_ptr: Optional[torch.Tensor] = None,
                 codes: Optional[torch.Tensor] = None, col_mean: Optional[torch.Tensor] = None,
                 col_scale: Optional[torch.Tensor] = None,
                 n: Optional[int] = None, max_col_nnz: Optional[int] = None,
                 stream: Optional[torch.cuda.Stream] = None, dynamic: bool = False, priority: str = "squared",
                 no_deps: bool = False, n_shards: int = 1, loss: str = "squared"):
        lib = load()
        self._h = None
        dev = y.device
        if dev.type != "cuda":
            raise ValueError("tensors must live on the GPU")
        self.device = dev
        if x is not None:
            assert x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 2
            self.J, self.N = x.shape                      # row j of the tensor = column x_j (ld = N)
            layout = LAYOUT_DENSE
            self._keep = (x, y)
        elif codes is not None:
            # packed genotype counts: (J, 4*ceil(N/64)) int32 words plus a mean and a scale per column
            assert codes.dtype == torch.int32 and codes.is_contiguous() and codes.dim() == 2
            assert col_mean.dtype == torch.float32 and col_scale.dtype == torch.float32
            self.J, self.N = codes.shape[0], int(n)
            assert codes.shape[1] == (self.N + 63) // 64 * 4 and col_mean.numel() == self.J == col_scale.numel()
            layout = LAYOUT_GENO2
            self._keep = (codes, col_mean, col_scale, y)
        else:
            assert values.dtype == torch.float32 and row_idx.dtype == torch.int32 and col_ptr.dtype == torch.int64
            self.J, self.N = col_ptr.numel() - 1, int(n)
            layout = LAYOUT_CSC
            self._keep = (values, row_idx, col_ptr, y)
            if max_col_nnz is None:
                max_col_nnz = int((col_ptr[1:] - col_ptr[:-1]).max().item())
        assert y.dtype == torch.float32 and y.is_contiguous() and y.numel() == self.N
        self.L = min(int(l_prime), self.J // max(1, int(n_shards)))
        self.stream = stream if stream is not None else torch.cuda.current_stream(dev)
        data = x if x is not None else (codes if codes is not None else values)
        cfg = Config(n=self.N, j=self.J, layout=layout, x=_ptr(data),
                     row_idx=_ptr(row_idx), col_ptr=_ptr(col_ptr), col_mean=_ptr(col_mean),
                     col_scale=_ptr(col_scale), y=_ptr(y), lam=lam, rho=rho, eta=eta,
                     c_init=c_init, l_prime=int(l_prime), p_max=int(p_max), seed=int(seed),
                     keep_gram=int(keep_gram), max_col_nnz=int(max_col_nnz or 0),
                     deps=DEPS_NONE if no_deps else (DEPS_DYNAMIC if dynamic else DEPS_STATIC),
                     priority=PRIORITY[priority], n_shards=int(n_shards), loss=LOSS[loss],
                     stream=self.stream.cuda_stream)
        nbytes = int(lib.strads_lasso_workspace_bytes(C.byref(cfg)))
        if nbytes == 0:
            raise StradsError(E_INVALID_ARG, "strads_lasso_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        assert self.workspace.data_ptr() % 256 == 0
        cfg.workspace, cfg.workspace_bytes = self.workspace.data_ptr(), nbytes
        self.keep_gram = bool(keep_gram)
        h = C.c_void_p()
        with torch.cuda.device(dev):
            _check(lib.strads_lasso_create(C.byref(cfg), C.byref(h)), "strads_lasso_create")
        self._h = h
        self._cfg = cfg

    def close(self):
        if self._h is not None:
            torch.cuda.synchronize(self.device)
            load().strads_lasso_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the four calls of the boundary ---------------------------------------------------------
    def round(self, want_info: bool = False) -> Optional[RoundInfo]:
        info = RoundInfo() if want_info else None
        _check(load().strads_lasso_round(self._h, C.byref(info) if want_info else None), "strads_lasso_round")
        return info

    def run(self, max_rounds: int, kkt_tol: float = 0.0, check_every: int = 0) -> RunInfo:
        out = RunInfo()
        _check(load().strads_lasso_run(self._h, int(max_rounds), float(kkt_tol), int(check_every), C.byref(out)),
               "strads_lasso_run")
        return out

    def objective(self) -> float:
        v = C.c_double()
        _check(load().strads_lasso_objective(self._h, C.byref(v)), "strads_lasso_objective")
        return v.value

    # -- support --------------------------------------------------------------------------------
    def kkt(self, want_g: bool = False):
        v = C.c_float()
        g = torch.empty(self.J, dtype=torch.float32, device=self.device) if want_g else None
        _check(load().strads_lasso_kkt(self._h, C.byref(v), _ptr(g)), "strads_lasso_kkt")
        return (v.value, g) if want_g else v.value

    def get_state(self):
        beta = torch.empty(self.J, dtype=torch.float32, device=self.device)
        dbeta = torch.empty_like(beta)
        r = torch.empty(self.N, dtype=torch.float32, device=self.device)
        t = C.c_int64()
        _check(load().strads_lasso_get_state(self._h, _ptr(beta), _ptr(dbeta), _ptr(r), C.byref(t)),
               "strads_lasso_get_state")
        return beta, dbeta, r, t.value

    def set_state(self, beta, dbeta, r, t: int):
        def dev(a, n):
            if a is None:
                return None
            a = torch.as_tensor(a, dtype=torch.float32).to(self.device).contiguous()
            assert a.numel() == n
            return a
        b, d, rr = dev(beta, self.J), dev(dbeta, self.J), dev(r, self.N)
        _check(load().strads_lasso_set_state(self._h, _ptr(b), _ptr(d), _ptr(rr), int(t)), "strads_lasso_set_state")

    def last_round(self, want_gram: bool = False) -> dict:
        L = self.L
        cand = torch.empty(L, dtype=torch.int32, device=self.device)
        kept_pos = torch.empty(L, dtype=torch.int32, device=self.device)
        z = torch.empty(L, dtype=torch.float32, device=self.device)
        delta = torch.empty(L, dtype=torch.float32, device=self.device)
        G = torch.empty((L, L), dtype=torch.float32, device=self.device) if want_gram else None
        nc, nk = C.c_int32(), C.c_int32()
        _check(load().strads_lasso_last_round(self._h, _ptr(cand), _ptr(kept_pos), _ptr(z), _ptr(delta), _ptr(G),
                                              C.byref(nc), C.byref(nk)), "strads_lasso_last_round")
        k = nk.value
        out = {"cand": cand[:nc.value], "kept_pos": kept_pos[:k], "z": z[:k], "delta": delta[:k]}
        out["kept"] = out["cand"][out["kept_pos"].long()]
        if want_gram:
            out["G"] = G
        return out

    def last_candidates(self) -> dict:
        z = torch.empty(self.L, dtype=torch.float32, device=self.device)
        d = torch.empty(self.L, dtype=torch.float32, device=self.device)
        nm = C.c_int32()
        _check(load().strads_lasso_last_candidates(self._h, _ptr(z), _ptr(d), C.byref(nm)),
               "strads_lasso_last_candidates")
        return {"z_cand": z, "delta_cand": d, "n_movers": nm.value}

    def stage_keys(self, t: int) -> torch.Tensor:
        keys = torch.empty(self.J, dtype=torch.float32, device=self.device)
        _check(load().strads_lasso_stage_keys(self._h, int(t), _ptr(keys)), "strads_lasso_stage_keys")
        return keys

    def stage_filter(self, G: torch.Tensor) -> torch.Tensor:
        G = G.to(self.device, torch.float32).contiguous()
        l = G.shape[0]
        kept = torch.empty(max(l, 1), dtype=torch.int32, device=self.device)
        nk = C.c_int32()
        _check(load().strads_lasso_stage_filter(self._h, _ptr(G), l, _ptr(kept), C.byref(nk)),
               "strads_lasso_stage_filter")
        return kept[:nk.value]

    def stage_times(self) -> dict:
        ms = (C.c_float * N_STAGES)()
        n = C.c_int32()
        _check(load().strads_lasso_stage_times(self._h, ms, C.byref(n)), "strads_lasso_stage_times")
        return {"rounds": n.value, **{name: float(ms[i]) for i, name in enumerate(STAGE_NAMES)}}

    def last_kkt_ms(self) -> float:
        ms = C.c_float()
        _check(load().strads_lasso_last_kkt_ms(self._h, C.byref(ms)), "strads_lasso_last_kkt_ms")
        return float(ms.value)

    def gram_tile_edge(self) -> int:
        edge = C.c_int32(-1)
        _check(load().strads_lasso_gram_tile_edge(self._h, C.byref(edge)), "strads_lasso_gram_tile_edge")
        return edge.value

    def set_tuning(self, name: str, value: int):
        _check(load().strads_lasso_set_tuning(self._h, name.encode(), int(value)), "strads_lasso_set_tuning")
