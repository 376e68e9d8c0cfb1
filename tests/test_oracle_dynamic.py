"""Pins for the oracle's round with update-aware ("dynamic") dependencies (CPU only).

Section 1 ("Dynamic Block Structures") and Step 4 of Section 2: a coefficient that does not change
in a round has no dependency with any other; only pairs of coefficients that both move are
checked against rho.  Each test here fixes the result by something other than the oracle's own
code: the baseline round in the limits where both must coincide, a brute-force enumeration written
in numpy, hand-built three-column designs, and the fixed point of eq. (1).
"""
import itertools

import numpy as np
import pytest

from oracle.oracle import OracleLasso
from synth import lasso_inputs as si


def _small(n=120, j=60, seed=0, **kw):
    kw.setdefault("nnz", 6)
    kw.setdefault("l_prime", 20)
    return si.make("c1_dense_iid", n=n, j=j, seed=seed, **kw)


def _solver(p, **kw):
    args = dict(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
    args.update(kw)
    return OracleLasso(**args)


def _same_state(a, b):
    return np.array_equal(a.beta, b.beta) and np.array_equal(a.dbeta, b.dbeta) and np.array_equal(a.r, b.r)


def test_without_conflicts_dynamic_equals_baseline():
    # rho above every correlation: no pair conflicts in either variant, so the rounds coincide bit for bit
    p = _small(seed=1)
    a, b = _solver(p, rho=10.0), _solver(p, rho=10.0, dynamic=True)
    for _ in range(12):
        oa, ob = a.round(), b.round()
        assert np.array_equal(oa["cand"], ob["cand"]) and np.array_equal(oa["kept"], ob["kept"])
        assert np.array_equal(oa["delta"], ob["delta"])
        assert _same_state(a, b)


def test_when_every_candidate_moves_dynamic_equals_baseline():
    # lambda = 0: S(a, 0) = a, so every candidate's change is x^T r, nonzero for generic data;
    # then d_t is the full dependency and the two variants are the same algorithm
    p = _small(seed=2)
    a, b = _solver(p, lam=0.0, rho=0.15), _solver(p, lam=0.0, rho=0.15, dynamic=True)
    for _ in range(8):
        oa, ob = a.round(), b.round()
        assert ob["mover"].all()
        assert np.array_equal(oa["kept"], ob["kept"])
        assert _same_state(a, b)


def test_kept_set_equals_brute_force_on_tiny_candidate_sets():
    # independent statement: among all subsets S of the candidates in which no two *moving*
    # members have |x_a^T x_b| >= rho, B_1 is the one whose indicator vector is lexicographically
    # largest (take the first candidate if at all possible, then the second, ...)
    rng = np.random.default_rng(5)
    for trial in range(30):
        n, j, L = 40, 12, int(rng.integers(2, 9))
        f = rng.normal(size=(n, 3))
        x = (f @ rng.normal(size=(3, j)) + 0.7 * rng.normal(size=(n, j)))
        x -= x.mean(0)
        x /= np.linalg.norm(x, axis=0)
        x = np.ascontiguousarray(x.T, dtype=np.float32)
        y = rng.normal(size=n).astype(np.float32)
        lam = float(np.quantile(np.abs(x.astype(np.float64) @ y), 0.5))     # about half the candidates move
        rho = float(rng.uniform(0.1, 0.5))
        s = OracleLasso(x=x, y=y, lam=lam, rho=rho, eta=1e-6, l_prime=L, seed=trial, dynamic=True)
        beta0, r0 = s.beta.copy(), s.r.copy()
        out = s.round(want_gram=True)
        cand = out["cand"]
        X64 = x.astype(np.float64)
        z = X64[cand] @ r0.astype(np.float64)
        a_ = z + beta0[cand]
        newb = (np.sign(a_) * np.maximum(np.abs(a_) - np.float32(lam), 0)).astype(np.float32)
        mover = (newb.astype(np.float64) - beta0[cand]) != 0
        assert np.array_equal(mover, out["mover"])
        G = (X64[cand] @ X64[cand].T).astype(np.float32)
        best = None
        for bits in itertools.product((1, 0), repeat=L):                    # lexicographically decreasing
            S = [i for i in range(L) if bits[i]]
            ok = all(not (mover[u] and mover[v] and not (abs(G[u, v]) < np.float32(rho)))
                     for u, v in itertools.combinations(S, 2))
            if ok:
                best = S
                break
        assert out["kept_pos"].tolist() == best
        # the dependency matrix the oracle reports is d_t: zero wherever a non-mover is involved
        assert np.all(out["G"][~mover, :] == 0) and np.all(out["G"][:, ~mover] == 0)
        mm = np.ix_(mover, mover)
        assert np.allclose(out["G"][mm], G[mm], atol=1e-6)


def _three_columns(c_ab, c_bc):
    """Unit-norm a, b, c with a.b = c_ab, b.c = c_bc and a orthogonal to c."""
    e = np.eye(8)
    a = e[0]
    b = c_ab * e[0] + c_bc * e[2] + np.sqrt(1 - c_ab ** 2 - c_bc ** 2) * e[1]
    c = e[2]
    return np.ascontiguousarray(np.stack([a, b, c]), dtype=np.float32)


def test_a_coefficient_that_stays_put_blocks_nobody():
    # b correlates strongly with a and with c, but its own update is zero (|x_b^T y| <= lambda)
    # while a and c move.  Baseline: b drawn first blocks both a and c, otherwise b is rejected.
    # Dynamic: all three are kept and the result is the exact joint update of the two orthogonal
    # movers.
    x = _three_columns(0.6, 0.6)
    y = np.zeros(8, np.float32)
    y[0], y[2] = 2.0, -3.0                                  # x_a^T y = 2, x_c^T y = -3, x_b^T y = -0.6
    lam = 1.0
    for seed in range(6):
        dyn = OracleLasso(x=x, y=y, lam=lam, rho=0.1, eta=1e-6, l_prime=3, seed=seed, dynamic=True)
        out = dyn.round()
        order = out["cand"].tolist()
        assert sorted(out["kept"].tolist()) == [0, 1, 2]
        assert out["mover"].tolist() == [j != 1 for j in order]
        assert dyn.beta.tolist() == [1.0, 0.0, -2.0]
        assert dyn.dbeta.tolist() == [1.0, 0.0, 2.0]
        assert np.allclose(dyn.r, y - x.T @ dyn.beta, atol=1e-7)
        base = OracleLasso(x=x, y=y, lam=lam, rho=0.1, eta=1e-6, l_prime=3, seed=seed)
        ob = base.round()
        assert order == ob["cand"].tolist()                                  # same draw
        assert ob["kept"].tolist() == ([1] if order[0] == 1 else [j for j in order if j != 1])


def test_two_moving_correlated_coefficients_still_conflict():
    x = _three_columns(0.6, 0.0)                            # a and b correlated, c orthogonal to both
    y = (3.0 * x[0] + 3.0 * x[1]).astype(np.float32)
    dyn = OracleLasso(x=x, y=y, lam=0.5, rho=0.1, eta=1e-6, l_prime=3, seed=0, dynamic=True)
    out = dyn.round()
    order = out["cand"].tolist()
    first_ab = [j for j in order if j in (0, 1)][0]
    second_ab = 1 - first_ab
    assert first_ab in out["kept"] and second_ab not in out["kept"] and 2 in out["kept"]
    assert dyn.dbeta[second_ab] == np.float32(1e6)          # a rejected candidate keeps its priority
    assert dyn.dbeta[2] == 0.0                              # kept, did not move


def test_cap_counts_kept_coordinates_in_draw_order():
    p = _small(seed=3, l_prime=20)
    full = _solver(p, dynamic=True)
    capped = _solver(p, dynamic=True, p_max=7)
    of, oc = full.round(), capped.round()
    assert np.array_equal(oc["kept_pos"], of["kept_pos"][:7])


def test_residual_invariant_and_bookkeeping_along_a_trajectory():
    p = _small(n=150, j=90, seed=6, l_prime=25, rho=0.15)
    s = _solver(p, dynamic=True)
    X = p.x.numpy().astype(np.float64)
    y = p.y.numpy().astype(np.float64)
    for _ in range(60):
        before = s.beta.copy(), s.dbeta.copy()
        out = s.round(want_gram=True)
        kept, cand = out["kept"], out["cand"]
        rejected = np.setdiff1d(cand, kept)
        untouched = np.setdiff1d(np.arange(p.j), kept)
        assert np.array_equal(s.beta[untouched], before[0][untouched])
        assert np.array_equal(s.dbeta[untouched], before[1][untouched])
        assert np.all(out["mover"][np.isin(cand, rejected)])            # only movers are ever rejected
        assert np.allclose(s.dbeta[kept], np.abs(s.beta[kept].astype(np.float64) - before[0][kept]), atol=1e-7)
        km = out["kept_pos"][out["mover"][out["kept_pos"]]]
        Gk = np.abs(out["G"][np.ix_(km, km)])
        np.fill_diagonal(Gk, 0)
        assert np.all(Gk < s.rho)                                        # kept movers are pairwise admissible
        assert np.abs(s.r - (y - X.T @ s.beta.astype(np.float64))).max() < 5e-6


def test_converges_to_the_lasso_solution():
    from sklearn.linear_model import Lasso
    p = _small(n=150, j=80, seed=4, l_prime=16)
    s = _solver(p, dynamic=True)
    for _ in range(1500):
        s.round()
    assert s.kkt() < 2e-5
    ref = Lasso(alpha=float(s.lam) / p.n, fit_intercept=False, tol=1e-14, max_iter=200000)
    ref.fit(p.x.numpy().T.astype(np.float64), p.y.numpy().astype(np.float64))
    assert np.abs(s.beta - ref.coef_).max() < 5e-5


def test_the_sweep_is_faster_than_with_static_dependencies():
    # non-movers are never rejected, so untouched coordinates (delta beta = C) run out sooner
    p = si.make("c2_dense_block_corr", n=200, j=600, nnz=6, l_prime=60)
    a, b = _solver(p), _solver(p, dynamic=True)
    ra = rb = None
    for t in range(60):
        a.round(); b.round()
        if ra is None and not np.any(a.dbeta == np.float32(1e6)): ra = t
        if rb is None and not np.any(b.dbeta == np.float32(1e6)): rb = t
    assert rb is not None and (ra is None or rb <= ra)


def test_forced_decisions_are_followed():
    p = _small(seed=9)
    s = _solver(p, dynamic=True)
    out = s.round(forced_cand=np.array([5, 3, 9], np.int32), forced_mover=np.array([1, 0, 1], np.uint8),
                  forced_kept_pos=np.array([0, 1], np.int32))
    assert out["cand"].tolist() == [5, 3, 9] and out["kept"].tolist() == [5, 3]
    assert s.dbeta[3] == 0.0 and s.beta[3] == 0.0 and s.dbeta[9] == np.float32(1e6)


def test_csc_round_equals_dense_round():
    p = si.make("c4_sparse_csc", n=200, j=300, nnz_per_col=10, nnz=8, l_prime=30, rho=0.2)
    xd = si.csc_to_dense(p).numpy()
    kw = dict(y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=3, dynamic=True)
    a = OracleLasso(values=p.values.numpy(), row_idx=p.row_idx.numpy(), col_ptr=p.col_ptr.numpy(), n=p.n, **kw)
    b = OracleLasso(x=xd, **kw)
    for _ in range(20):
        oa, ob = a.round(), b.round()
        assert np.array_equal(oa["cand"], ob["cand"]) and np.array_equal(oa["kept"], ob["kept"])
    assert np.allclose(a.beta, b.beta, atol=1e-7) and np.allclose(a.r, b.r, atol=1e-6)
