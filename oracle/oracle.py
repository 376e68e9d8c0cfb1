"""ctypes front end of the plain-C oracle (oracle/strads_oracle.c).

Test infrastructure: only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this.  Nothing here touches the HIP library.
All arithmetic lives in the C file; this module marshals numpy arrays and
keeps the solver state (beta, dbeta, r, round counter) between rounds.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "strads_oracle.c")
_LIB = os.path.join(_HERE, "libstrads_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps every fp32
    operation of the specified key arithmetic separately rounded."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Problem(C.Structure):
    _fields_ = [("N", C.c_int64), ("J", C.c_int64), ("X", C.c_void_p), ("row_idx", C.c_void_p),
                ("col_ptr", C.c_void_p), ("lam", C.c_float), ("rho", C.c_float), ("eta", C.c_float),
                ("l_prime", C.c_int32), ("p_max", C.c_int32), ("seed", C.c_uint64),
                ("priority", C.c_int32), ("deps", C.c_int32), ("n_shards", C.c_int32), ("loss", C.c_int32),
                ("y", C.c_void_p)]


PRIORITY = {"squared": 0, "linear": 1, "uniform": 2}
LOSS = {"squared": 0, "logistic": 1}


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        vp, i32, i64, u64, f32, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_double
        L.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.oracle_philox4x32_10.restype = None
        L.oracle_uniform.argtypes = [u64, u64, u64]
        L.oracle_uniform.restype = f32
        L.oracle_log2_spec.argtypes = [f32]
        L.oracle_log2_spec.restype = f32
        L.oracle_priority_key.argtypes = [f32, f32, u64, u64, u64]
        L.oracle_priority_key.restype = f32
        L.oracle_priority_keys.argtypes = [i64, vp, f32, u64, u64, vp]
        L.oracle_priority_keys.restype = None
        L.oracle_priority_keys_mode.argtypes = [i64, vp, f32, u64, u64, i32, vp]
        L.oracle_priority_keys_mode.restype = None
        L.oracle_priority_weight.argtypes = [f32, f32, i32]
        L.oracle_priority_weight.restype = f32
        L.oracle_draw.argtypes = [i64, vp, i32, vp]
        L.oracle_draw.restype = i32
        L.oracle_gram_dense.argtypes = [i64, vp, vp, i32, vp]
        L.oracle_gram_dense.restype = None
        L.oracle_gram_rows_dense.argtypes = [i64, vp, vp, i32, vp, i32, vp]
        L.oracle_gram_rows_dense.restype = None
        L.oracle_gram_pairs_dense.argtypes = [i64, vp, vp, vp, vp, i64, vp]
        L.oracle_gram_pairs_dense.restype = None
        L.oracle_gram_csc.argtypes = [vp, vp, vp, vp, i32, vp]
        L.oracle_gram_csc.restype = None
        L.oracle_filter.argtypes = [i32, vp, f32, i32, vp]
        L.oracle_filter.restype = i32
        L.oracle_dots_dense.argtypes = [i64, vp, vp, i32, vp, vp]
        L.oracle_dots_dense.restype = None
        L.oracle_dots_csc.argtypes = [vp, vp, vp, vp, i32, vp, vp]
        L.oracle_dots_csc.restype = None
        L.oracle_soft_threshold.argtypes = [f64, f64]
        L.oracle_soft_threshold.restype = f64
        L.oracle_update.argtypes = [i32, vp, vp, f32, f64, vp, vp, vp]
        L.oracle_update.restype = None
        L.oracle_residual_dense.argtypes = [i64, vp, vp, i32, vp, vp]
        L.oracle_residual_dense.restype = None
        L.oracle_residual_csc.argtypes = [i64, vp, vp, vp, vp, i32, vp, vp]
        L.oracle_residual_csc.restype = None
        L.oracle_objective.argtypes = [i64, vp, i64, vp, f32]
        L.oracle_objective.restype = f64
        L.oracle_logistic_weights.argtypes = [i64, vp, vp, vp]
        L.oracle_logistic_weights.restype = None
        L.oracle_objective_logistic.argtypes = [i64, vp, vp, i64, vp, f32]
        L.oracle_objective_logistic.restype = f64
        L.oracle_kkt_dense.argtypes = [i64, i64, vp, vp, vp, f32, vp]
        L.oracle_kkt_dense.restype = f64
        L.oracle_kkt_csc.argtypes = [i64, vp, vp, vp, vp, vp, f32, vp]
        L.oracle_kkt_csc.restype = f64
        L.oracle_round.argtypes = [C.POINTER(_Problem), u64, vp, vp, vp, vp, i32, vp, i32,
                                   vp, C.POINTER(i32), vp, vp, vp, vp, vp]
        L.oracle_round.restype = i32
        L.oracle_round_dynamic.argtypes = [C.POINTER(_Problem), u64, vp, vp, vp, vp, i32, vp, vp, i32,
                                           vp, C.POINTER(i32), vp, vp, vp, vp, vp, vp, vp, vp]
        L.oracle_round_dynamic.restype = i32
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _arr(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# -- thin stage-level wrappers (used by the pin tests and stage-isolated parity) --------------

def philox4x32_10(ctr, key) -> np.ndarray:
    c, k = _arr(ctr, np.uint32), _arr(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().oracle_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def uniform(seed: int, t: int, j: int) -> float:
    return float(lib().oracle_uniform(seed, t, j))


def log2_spec(x: float) -> float:
    return float(lib().oracle_log2_spec(np.float32(x)))


def priority_keys(dbeta, eta, seed, t, priority="squared") -> np.ndarray:
    d = _arr(dbeta, np.float32)
    keys = np.empty(d.shape[0], np.float32)
    lib().oracle_priority_keys_mode(d.shape[0], _p(d), np.float32(eta), seed, t, PRIORITY[priority], _p(keys))
    return keys


def draw(keys, l_prime) -> np.ndarray:
    k = _arr(keys, np.float32)
    cand = np.empty(max(1, min(int(l_prime), k.shape[0])), np.int32)
    n = lib().oracle_draw(k.shape[0], _p(k), int(l_prime), _p(cand))
    if n < 0:
        raise MemoryError
    return cand[:n].copy()


def gram_dense(x_cols, cand) -> np.ndarray:
    """x_cols: (J, N) fp32, row j = covariate x_j."""
    x, c = _arr(x_cols, np.float32), _arr(cand, np.int32)
    L = c.shape[0]
    G = np.empty((L, L), np.float32)
    lib().oracle_gram_dense(x.shape[1], _p(x), _p(c), L, _p(G))
    return G


def gram_rows_dense(x_cols, cand, rows) -> np.ndarray:
    """Rows `rows` (positions into cand) of the candidate Gram: (len(rows), len(cand)) fp32."""
    x, c, rw = _arr(x_cols, np.float32), _arr(cand, np.int32), _arr(rows, np.int32)
    out = np.empty((rw.shape[0], c.shape[0]), np.float32)
    lib().oracle_gram_rows_dense(x.shape[1], _p(x), _p(c), c.shape[0], _p(rw), rw.shape[0], _p(out))
    return out


def gram_pairs_dense(x_cols, cand, pa, pb) -> np.ndarray:
    """Entries (pa[t], pb[t]) (positions into cand) of the candidate Gram."""
    x, c = _arr(x_cols, np.float32), _arr(cand, np.int32)
    a, b = _arr(pa, np.int32), _arr(pb, np.int32)
    assert a.shape == b.shape
    out = np.empty(a.shape[0], np.float32)
    lib().oracle_gram_pairs_dense(x.shape[1], _p(x), _p(c), _p(a), _p(b), a.shape[0], _p(out))
    return out


def gram_csc(values, row_idx, col_ptr, cand) -> np.ndarray:
    v, ri, cp, c = _arr(values, np.float32), _arr(row_idx, np.int32), _arr(col_ptr, np.int64), _arr(cand, np.int32)
    L = c.shape[0]
    G = np.empty((L, L), np.float32)
    lib().oracle_gram_csc(_p(v), _p(ri), _p(cp), _p(c), L, _p(G))
    return G


def greedy_filter(G, rho, p_max=0) -> np.ndarray:
    g = _arr(G, np.float32)
    L = g.shape[0]
    kept = np.empty(max(L, 1), np.int32)
    k = lib().oracle_filter(L, _p(g), np.float32(rho), int(p_max), _p(kept))
    return kept[:k].copy()


def dots_dense(x_cols, cols, r) -> np.ndarray:
    """x_j^T r (fp64) for the listed columns of a dense design; x_cols: (J, N) fp32, row j = covariate x_j."""
    x, c, rr = _arr(x_cols, np.float32), _arr(cols, np.int32), _arr(r, np.float32)
    z = np.empty(c.shape[0], np.float64)
    lib().oracle_dots_dense(x.shape[1], _p(x), _p(c), c.shape[0], _p(rr), _p(z))
    return z


def dots_csc(values, row_idx, col_ptr, cols, r) -> np.ndarray:
    v, ri, cp = _arr(values, np.float32), _arr(row_idx, np.int32), _arr(col_ptr, np.int64)
    c, rr = _arr(cols, np.int32), _arr(r, np.float32)
    z = np.empty(c.shape[0], np.float64)
    lib().oracle_dots_csc(_p(v), _p(ri), _p(cp), _p(c), c.shape[0], _p(rr), _p(z))
    return z


def update(cols, z, lam, beta, dbeta, inv_kappa: float = 1.0) -> np.ndarray:
    """eq. (2) and Step 4 for the listed coordinates, in place on beta and dbeta (fp32 arrays that must be
    C-contiguous); returns the changes (fp64).  inv_kappa: 1 for the squared loss, 4 for the logistic loss."""
    c, zz = _arr(cols, np.int32), _arr(z, np.float64)
    assert beta.dtype == np.float32 and dbeta.dtype == np.float32 and beta.flags.c_contiguous and dbeta.flags.c_contiguous
    delta = np.empty(c.shape[0], np.float64)
    lib().oracle_update(c.shape[0], _p(c), _p(zz), np.float32(lam), float(inv_kappa), _p(beta), _p(dbeta), _p(delta))
    return delta


def residual_dense(x_cols, cols, delta, r) -> None:
    """r <- r - sum_c x_{cols[c]} delta[c], in place on r (fp32, C-contiguous)."""
    x, c, d = _arr(x_cols, np.float32), _arr(cols, np.int32), _arr(delta, np.float64)
    assert r.dtype == np.float32 and r.flags.c_contiguous and r.shape[0] == x.shape[1]
    lib().oracle_residual_dense(x.shape[1], _p(x), _p(c), c.shape[0], _p(d), _p(r))


def residual_csc(values, row_idx, col_ptr, cols, delta, r) -> None:
    v, ri, cp = _arr(values, np.float32), _arr(row_idx, np.int32), _arr(col_ptr, np.int64)
    c, d = _arr(cols, np.int32), _arr(delta, np.float64)
    assert r.dtype == np.float32 and r.flags.c_contiguous
    lib().oracle_residual_csc(r.shape[0], _p(v), _p(ri), _p(cp), _p(c), c.shape[0], _p(d), _p(r))


def logistic_weights(y, v) -> np.ndarray:
    """w_i = y_i / (1 + exp(-y_i v_i)) from the state vector v = -X beta."""
    yy, vv = _arr(y, np.float32), _arr(v, np.float32)
    w = np.empty(yy.shape[0], np.float32)
    lib().oracle_logistic_weights(yy.shape[0], _p(yy), _p(vv), _p(w))
    return w


def objective_logistic(y, v, beta, lam) -> float:
    yy, vv, b = _arr(y, np.float32), _arr(v, np.float32), _arr(beta, np.float32)
    return float(lib().oracle_objective_logistic(yy.shape[0], _p(yy), _p(vv), b.shape[0], _p(b), np.float32(lam)))


def soft_threshold(a: float, lam: float) -> float:
    return float(lib().oracle_soft_threshold(float(a), float(lam)))


def objective(r, beta, lam) -> float:
    rr, b = _arr(r, np.float32), _arr(beta, np.float32)
    return float(lib().oracle_objective(rr.shape[0], _p(rr), b.shape[0], _p(b), np.float32(lam)))


class OracleLasso:
    """State + rounds of Algorithm 1 on the CPU.  Dense: pass x of shape (J, N)
    (row j = covariate j).  CSC: pass values,row_idx,col_ptr and n."""

    def __init__(self, y, lam, rho, eta, l_prime, seed=0, p_max=0, c_init=1e6, x=None,
                 values=None, row_idx=None, col_ptr=None, n=None, dynamic=False, priority="squared",
                 no_deps=False, n_shards=1, loss="squared"):
        self.dynamic = bool(dynamic)          # update-aware dependencies (oracle_round_dynamic)
        self.priority = priority              # "squared" | "linear" | "uniform"
        self.no_deps = bool(no_deps)          # skip Step 2 (Shotgun)
        self.n_shards = max(1, int(n_shards)) # scheduler shards taking turns; coordinate j is in shard j % S
        assert not (self.dynamic and self.no_deps)
        self.loss = loss                      # "squared" | "logistic" (labels y in {-1, +1}; state vector -X beta)
        self.y = _arr(y, np.float32)
        if x is not None:
            self.x = _arr(x, np.float32)
            self.J, self.N = self.x.shape
            self.csc = False
            self.row_idx = self.col_ptr = None
        else:
            self.x = _arr(values, np.float32)
            self.row_idx = _arr(row_idx, np.int32)
            self.col_ptr = _arr(col_ptr, np.int64)
            self.J, self.N = self.col_ptr.shape[0] - 1, int(n)
            self.csc = True
        assert self.y.shape[0] == self.N
        self.lam, self.rho, self.eta = np.float32(lam), np.float32(rho), np.float32(eta)
        self.l_prime, self.p_max, self.seed = min(int(l_prime), self.J // max(1, int(n_shards))), int(p_max), int(seed)
        # Algorithm 1 initialisation: beta^(t-1) = 0, beta^(t-2) = C  =>  delta beta_j = C for all j
        self.beta = np.zeros(self.J, np.float32)
        self.dbeta = np.full(self.J, c_init, np.float32)
        self.r = self.y.copy() if loss == "squared" else np.zeros(self.N, np.float32)
        self.t = 0
        self._prob = _Problem(self.N, self.J, _p(self.x), _p(self.row_idx), _p(self.col_ptr),
                              self.lam, self.rho, self.eta, self.l_prime, self.p_max, self.seed,
                              PRIORITY[priority], 2 if self.no_deps else (1 if self.dynamic else 0),
                              self.n_shards, LOSS[loss], _p(self.y))

    def set_state(self, beta, dbeta, r, t):
        self.beta[:] = beta
        self.dbeta[:] = dbeta
        self.r[:] = r
        self.t = int(t)

    def round(self, want_gram=False, forced_cand=None, forced_kept_pos=None, forced_mover=None) -> dict:
        if self.dynamic:
            return self._round_dynamic(want_gram, forced_cand, forced_mover, forced_kept_pos)
        assert forced_mover is None
        Lmax = max(self.l_prime if forced_cand is None else len(forced_cand), 1)
        cand = np.empty(Lmax, np.int32)
        kept_pos = np.empty(Lmax, np.int32)
        kept = np.empty(Lmax, np.int32)
        z = np.empty(Lmax, np.float64)
        delta = np.empty(Lmax, np.float64)
        G = np.empty((Lmax, Lmax), np.float32) if want_gram else None
        fc = None if forced_cand is None else _arr(forced_cand, np.int32)
        fk = None if forced_kept_pos is None else _arr(forced_kept_pos, np.int32)
        ncand = C.c_int32(0)
        k = lib().oracle_round(C.byref(self._prob), self.t, _p(self.beta), _p(self.dbeta), _p(self.r),
                               _p(fc), 0 if fc is None else fc.shape[0],
                               _p(fk), 0 if fk is None else fk.shape[0],
                               _p(cand), C.byref(ncand), _p(kept_pos), _p(kept), _p(G), _p(z), _p(delta))
        if k < 0:
            raise MemoryError("oracle_round allocation failed")
        L = ncand.value
        self.t += 1
        out = {"cand": cand[:L].copy(), "kept_pos": kept_pos[:k].copy(), "kept": kept[:k].copy(),
               "z": z[:k].copy(), "delta": delta[:k].copy()}
        if want_gram:
            out["G"] = G[:L, :L] if L == Lmax else G.reshape(-1)[:L * L].reshape(L, L).copy()
        return out

    def _round_dynamic(self, want_gram, forced_cand, forced_mover, forced_kept_pos) -> dict:
        Lmax = max(self.l_prime if forced_cand is None else len(forced_cand), 1)
        cand = np.empty(Lmax, np.int32)
        kept_pos = np.empty(Lmax, np.int32)
        kept = np.empty(Lmax, np.int32)
        mover = np.zeros(Lmax, np.uint8)
        z_cand = np.empty(Lmax, np.float64)
        d_cand = np.empty(Lmax, np.float64)
        z = np.empty(Lmax, np.float64)
        delta = np.empty(Lmax, np.float64)
        G = np.empty((Lmax, Lmax), np.float32) if want_gram else None
        fc = None if forced_cand is None else _arr(forced_cand, np.int32)
        fm = None if forced_mover is None else _arr(forced_mover, np.uint8)
        fk = None if forced_kept_pos is None else _arr(forced_kept_pos, np.int32)
        ncand = C.c_int32(0)
        k = lib().oracle_round_dynamic(C.byref(self._prob), self.t, _p(self.beta), _p(self.dbeta), _p(self.r),
                                       _p(fc), 0 if fc is None else fc.shape[0], _p(fm),
                                       _p(fk), 0 if fk is None else fk.shape[0],
                                       _p(cand), C.byref(ncand), _p(mover), _p(z_cand), _p(d_cand),
                                       _p(kept_pos), _p(kept), _p(G), _p(z), _p(delta))
        if k < 0:
            raise MemoryError("oracle_round_dynamic allocation failed")
        L = ncand.value
        self.t += 1
        out = {"cand": cand[:L].copy(), "kept_pos": kept_pos[:k].copy(), "kept": kept[:k].copy(),
               "z": z[:k].copy(), "delta": delta[:k].copy(), "mover": mover[:L].astype(bool),
               "z_cand": z_cand[:L].copy(), "delta_cand": d_cand[:L].copy()}
        if want_gram:
            out["G"] = G[:L, :L] if L == Lmax else G.reshape(-1)[:L * L].reshape(L, L).copy()
        return out

    def objective(self) -> float:
        if self.loss == "logistic":
            return float(lib().oracle_objective_logistic(self.N, _p(self.y), _p(self.r), self.J, _p(self.beta),
                                                         self.lam))
        return objective(self.r, self.beta, self.lam)

    def dots_vector(self) -> np.ndarray:
        """What eq. (2) and the optimality test take dot products with: r, or the logistic weights."""
        if self.loss != "logistic":
            return self.r
        w = np.empty(self.N, np.float32)
        lib().oracle_logistic_weights(self.N, _p(self.y), _p(self.r), _p(w))
        return w

    def kkt(self, want_g=False):
        g = np.empty(self.J, np.float64) if want_g else None
        dv = self.dots_vector()
        if self.csc:
            v = lib().oracle_kkt_csc(self.J, _p(self.x), _p(self.row_idx), _p(self.col_ptr), _p(dv),
                                     _p(self.beta), self.lam, _p(g))
        else:
            v = lib().oracle_kkt_dense(self.N, self.J, _p(self.x), _p(dv), _p(self.beta), self.lam, _p(g))
        return (float(v), g) if want_g else float(v)
