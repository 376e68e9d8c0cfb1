"""Pins for the oracle's update steps and for whole rounds of Algorithm 1 (CPU only)."""
import math

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle.oracle import OracleLasso
from synth import lasso_inputs as si


# ---- soft-threshold closed form ---------------------------------------------------------------
@settings(max_examples=300, deadline=None)
@given(st.floats(-50, 50), st.floats(0, 10), st.floats(-50, 50))
def test_soft_threshold_properties(a, lam, b):
    from oracle import oracle as o
    s = o.soft_threshold(a, lam)
    if abs(a) <= lam:
        assert s == 0.0
    elif a > 0:
        assert s == a - lam
    else:
        assert s == a + lam
    assert o.soft_threshold(-a, lam) == -s                       # odd
    assert abs(s - o.soft_threshold(b, lam)) <= abs(a - b) + 1e-12   # 1-Lipschitz
    # it is the minimiser of 1/2 (v - a)^2 + lam |v|
    f = lambda v: 0.5 * (v - a) ** 2 + lam * abs(v)
    for dv in (-1e-3, 1e-3, -0.1, 0.1):
        assert f(s) <= f(s + dv) + 1e-12


def _small(n=120, j=60, seed=0, **kw):
    kw.setdefault("nnz", 6)
    kw.setdefault("l_prime", 20)
    return si.make("c1_dense_iid", n=n, j=j, seed=seed, **kw)


def _solver(p, **kw):
    args = dict(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
    args.update(kw)
    return OracleLasso(**args)


# ---- closed-form whole-solver cases -----------------------------------------------------------
def test_orthonormal_design_is_solved_in_one_round():
    rng = np.random.default_rng(0)
    q, _ = np.linalg.qr(rng.normal(size=(64, 24)))
    x = np.ascontiguousarray(q.T, dtype=np.float32)             # (J, N), orthonormal columns
    y = rng.normal(size=64).astype(np.float32)
    lam = 0.3
    s = OracleLasso(x=x, y=y, lam=lam, rho=0.05, eta=1e-6, l_prime=24, seed=1)
    out = s.round(want_gram=True)
    assert len(out["kept"]) == 24                               # nothing conflicts
    xty = x.astype(np.float64) @ y.astype(np.float64)
    exact = np.sign(xty) * np.maximum(np.abs(xty) - lam, 0)
    assert np.abs(s.beta - exact).max() < 1e-6
    assert s.kkt() < 1e-6
    # a second round changes nothing
    b = s.beta.copy()
    s.round()
    assert np.abs(s.beta - b).max() < 1e-6


def test_large_lambda_keeps_beta_zero():
    p = _small()
    xty = np.abs(p.x.numpy().astype(np.float64) @ p.y.numpy().astype(np.float64)).max()
    s = _solver(p, lam=float(xty) * 1.0001)
    for _ in range(5):
        s.round()
    assert not s.beta.any() and np.array_equal(s.r, p.y.numpy())
    assert s.objective() == pytest.approx(0.5 * float((p.y.double() ** 2).sum()), rel=1e-12)


def test_single_column_and_two_columns_closed_form():
    rng = np.random.default_rng(3)
    x1 = rng.normal(size=50); x1 /= np.linalg.norm(x1)
    y = (2.0 * x1 + 0.1 * rng.normal(size=50)).astype(np.float32)
    s = OracleLasso(x=x1[None, :].astype(np.float32), y=y, lam=0.5, rho=0.1, eta=1e-6, l_prime=1)
    s.round()
    a = float(x1.astype(np.float32).astype(np.float64) @ y.astype(np.float64))
    assert s.beta[0] == pytest.approx(math.copysign(max(abs(a) - 0.5, 0), a), abs=1e-6)
    # two unit columns with correlation c, both active with positive sign:
    # beta = (X^T X)^-1 (X^T y - lam * 1)
    c = 0.6
    u = rng.normal(size=50); u -= (u @ x1) * x1; u /= np.linalg.norm(u)
    x2 = c * x1 + math.sqrt(1 - c * c) * u
    X = np.stack([x1, x2]).astype(np.float32)
    y = (3.0 * x1 + 2.0 * x2).astype(np.float32)
    lam = 0.2
    s = OracleLasso(x=X, y=y, lam=lam, rho=0.1, eta=1e-6, l_prime=2)     # rho < c: one at a time
    for _ in range(400):
        out = s.round()
        assert len(out["kept"]) == 1
    X64 = X.astype(np.float64)
    exact = np.linalg.solve(X64 @ X64.T, X64 @ y.astype(np.float64) - lam)
    assert np.all(exact > 0)
    assert np.abs(s.beta - exact).max() < 1e-5


# ---- fixed point: KKT and an independent library solver ------------------------------------------
def test_converged_solution_satisfies_kkt_and_matches_sklearn():
    from sklearn.linear_model import Lasso
    p = _small(n=150, j=80, seed=4, l_prime=16)
    s = _solver(p)
    for _ in range(1500):
        s.round()
    viol, g = s.kkt(want_g=True)
    lam = float(s.lam)
    zero = s.beta == 0
    assert np.all(np.abs(g[zero]) <= lam + 2e-5)
    assert np.abs(g[~zero] - lam * np.sign(s.beta[~zero])).max() < 2e-5
    assert viol < 2e-5
    ref = Lasso(alpha=lam / p.n, fit_intercept=False, tol=1e-14, max_iter=200000)
    ref.fit(p.x.numpy().T.astype(np.float64), p.y.numpy().astype(np.float64))
    assert np.abs(s.beta - ref.coef_).max() < 5e-5
    assert (s.beta != 0).sum() > 0


def test_converged_solution_matches_plain_cyclic_cd():
    p = _small(n=100, j=40, seed=5, l_prime=10)
    s = _solver(p)
    for _ in range(1200):
        s.round()
    X = p.x.numpy().astype(np.float64).T
    y = p.y.numpy().astype(np.float64)
    b = np.zeros(p.j)
    for _ in range(3000):
        for j in range(p.j):
            a = X[:, j] @ (y - X @ b) + b[j] * (X[:, j] @ X[:, j])
            b[j] = np.sign(a) * max(abs(a) - p.lam, 0) / (X[:, j] @ X[:, j])
    assert np.abs(s.beta - b).max() < 5e-5


# ---- invariants along the trajectory ----------------------------------------------------------
def test_sequential_updates_never_increase_the_objective():
    p = _small(n=100, j=50, seed=6, l_prime=10)
    s = _solver(p, p_max=1)
    f = s.objective()
    for _ in range(300):
        out = s.round()
        assert len(out["kept"]) == 1
        g = s.objective()
        assert g <= f + 1e-9 * max(1.0, abs(f))
        f = g


def test_residual_invariant_and_bookkeeping():
    p = si.make("c2_dense_block_corr", n=200, j=300, nnz=12, l_prime=40)
    s = _solver(p)
    X = p.x.numpy().astype(np.float64)
    seen = np.zeros(p.j, bool)
    for t in range(30):
        before_beta, before_db, before_r = s.beta.copy(), s.dbeta.copy(), s.r.copy()
        out = s.round(want_gram=True)
        kept, cand = out["kept"], out["cand"]
        # candidate set: distinct; kept set: pairwise below rho, drawn from the candidates in order
        assert len(set(cand.tolist())) == len(cand) == 40
        assert np.array_equal(kept, cand[out["kept_pos"]]) and np.all(np.diff(out["kept_pos"]) > 0)
        G = out["G"]
        sub = np.abs(G[np.ix_(out["kept_pos"], out["kept_pos"])]) - np.eye(len(kept))
        assert sub.max() < p.rho
        for a in set(range(40)) - set(out["kept_pos"].tolist()):       # maximal w.r.t. earlier kept
            earlier = [b for b in out["kept_pos"] if b < a]
            assert any(abs(G[a, b]) >= p.rho for b in earlier)
        # all dots use the residual from the start of the round (eq. 2 with beta^(t-1))
        z_ref = X[kept] @ before_r.astype(np.float64)
        assert np.abs(out["z"] - z_ref).max() < 1e-9
        # coordinates outside B_1 keep beta and delta-beta; inside: dbeta = |change|
        mask = np.ones(p.j, bool); mask[kept] = False
        assert np.array_equal(s.beta[mask], before_beta[mask]) and np.array_equal(s.dbeta[mask], before_db[mask])
        assert np.allclose(s.dbeta[kept], np.abs(s.beta[kept].astype(np.float64) - before_beta[kept]), atol=1e-7)
        assert np.allclose(out["delta"], s.beta[kept].astype(np.float64) - before_beta[kept], atol=0)
        # r == y - X beta, recomputed from scratch
        r_ref = p.y.numpy().astype(np.float64) - s.beta.astype(np.float64) @ X
        assert np.abs(s.r - r_ref).max() < 5e-6
        assert s.objective() == pytest.approx(0.5 * (r_ref ** 2).sum() + float(s.lam) * np.abs(s.beta).sum(), rel=1e-5)
        seen[kept] = True
    assert s.t == 30


def test_first_rounds_sweep_unvisited_coordinates_first():
    # the paper's remark on the early sharp drop: once every coordinate has been visited the
    # priorities are informed.  With delta beta = C initially, a round draws only coordinates that
    # were never updated (rejected candidates keep C and come back) while P' of them remain.
    p = _small(n=80, j=100, seed=8, l_prime=25)
    s = _solver(p)
    C = np.float32(1e6)
    rounds = 0
    while (s.dbeta == C).any():
        unvisited = s.dbeta == C
        out = s.round()
        if unvisited.sum() >= 25:
            assert unvisited[out["cand"]].all()
        else:
            assert unvisited[out["cand"]].sum() == unvisited.sum()
        assert not (s.dbeta[out["kept"]] == C).any()
        rounds += 1
        assert rounds < 60
    assert rounds >= 4


def test_csc_round_equals_dense_round():
    p = si.make("c4_sparse_csc", n=200, j=300, nnz_per_col=10, nnz=8, l_prime=30, rho=0.2)
    xd = si.csc_to_dense(p).numpy()
    a = OracleLasso(values=p.values.numpy(), row_idx=p.row_idx.numpy(), col_ptr=p.col_ptr.numpy(), n=p.n,
                    y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=3)
    b = OracleLasso(x=xd, y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=3)
    for _ in range(25):
        oa, ob = a.round(), b.round()
        assert np.array_equal(oa["cand"], ob["cand"]) and np.array_equal(oa["kept"], ob["kept"])
        assert np.allclose(oa["z"], ob["z"], atol=1e-12)
    assert np.allclose(a.beta, b.beta, atol=1e-7) and np.allclose(a.r, b.r, atol=1e-6)
    assert a.kkt() == pytest.approx(b.kkt(), abs=1e-9)


def test_forced_decisions_are_followed():
    p = _small(seed=9)
    s = _solver(p)
    out = s.round(forced_cand=np.array([5, 3, 9], np.int32), forced_kept_pos=np.array([0, 2], np.int32))
    assert out["cand"].tolist() == [5, 3, 9] and out["kept"].tolist() == [5, 9]
    assert s.dbeta[3] == np.float32(1e6)


# ---- the stage functions called one by one (as the full-size GPU parity tests call them) --------
def test_stage_functions_one_by_one_equal_the_whole_round_and_the_closed_forms():
    from oracle import oracle as o
    p = si.make("c5_dense_duplicates", n=150, j=240, nnz=8, l_prime=60, lam_frac=0.02)
    x, y = p.x.numpy(), p.y.numpy()
    s = _solver(p)
    for _ in range(3):
        beta0, dbeta0, r0 = s.beta.copy(), s.dbeta.copy(), s.r.copy()
        out = s.round()
        kept = out["kept"]
        # dots: against an fp64 matmul with the columns as rows (a transposed or shifted operand fails it)
        z = o.dots_dense(x, kept, r0)
        assert np.array_equal(z, out["z"])
        assert np.abs(z - x[kept].astype(np.float64) @ r0.astype(np.float64)).max() < 1e-12
        # update: closed form of the soft-threshold per coordinate, nothing else touched
        b, d = beta0.copy(), dbeta0.copy()
        delta = o.update(kept, z, p.lam, b, d)
        assert np.array_equal(delta, out["delta"]) and np.array_equal(b, s.beta) and np.array_equal(d, s.dbeta)
        for c, j in enumerate(kept):
            a = z[c] + float(beta0[j])
            want = np.float32(math.copysign(max(abs(a) - float(np.float32(p.lam)), 0.0), a))
            assert b[j] == want and d[j] == np.float32(abs(float(want) - float(beta0[j])))
        untouched = np.ones(p.j, bool)
        untouched[kept] = False
        assert np.array_equal(b[untouched], beta0[untouched]) and np.array_equal(d[untouched], dbeta0[untouched])
        # residual: r - X_B delta, and the invariant r = y - X beta
        r = r0.copy()
        o.residual_dense(x, kept, delta, r)
        assert np.array_equal(r, s.r)
        assert np.abs(r - (r0.astype(np.float64) - delta @ x[kept].astype(np.float64))).max() < 1e-6
        assert np.abs(r - (y.astype(np.float64) - b.astype(np.float64) @ x.astype(np.float64))).max() < 1e-5
    assert np.count_nonzero(s.beta) > 0


def test_stage_functions_csc_equal_dense_and_logistic_wrappers():
    from oracle import oracle as o
    p = si.make("c4_sparse_csc", n=200, j=300, nnz_per_col=9, nnz=6, l_prime=40)
    xd = si.csc_to_dense(p).numpy()
    v, ri, cp = p.values.numpy(), p.row_idx.numpy(), p.col_ptr.numpy()
    rng = np.random.default_rng(1)
    cols = rng.permutation(p.j)[:37].astype(np.int32)
    r = rng.normal(size=p.n).astype(np.float32)
    z_s, z_d = o.dots_csc(v, ri, cp, cols, r), o.dots_dense(xd, cols, r)
    assert np.abs(z_s - z_d).max() < 1e-12
    delta = rng.normal(size=37)
    r1, r2 = r.copy(), r.copy()
    o.residual_csc(v, ri, cp, cols, delta, r1)
    o.residual_dense(xd, cols, delta, r2)
    assert np.abs(r1.astype(np.float64) - r2).max() < 1e-6
    # logistic weights and objective: the textbook expressions in fp64
    yl = np.where(rng.random(p.n) < 0.5, -1.0, 1.0).astype(np.float32)
    w = o.logistic_weights(yl, r)
    assert np.abs(w - yl / (1.0 + np.exp(-yl.astype(np.float64) * r))).max() < 1e-7
    beta = rng.normal(size=p.j).astype(np.float32)
    f = o.objective_logistic(yl, r, beta, 0.3)
    assert f == pytest.approx(float(np.logaddexp(0.0, yl.astype(np.float64) * r).sum())
                              + float(np.float32(0.3)) * float(np.abs(beta.astype(np.float64)).sum()), rel=1e-12)
    # update with the logistic step (1 / curvature = 4): S(beta + 4 z, 4 lambda)
    b, d = beta.copy(), np.zeros_like(beta)
    zz = rng.normal(size=37) * 0.2
    dl = o.update(cols, zz, 0.3, b, d, inv_kappa=4.0)
    for c, j in enumerate(cols):
        a = 4.0 * zz[c] + float(beta[j])
        want = np.float32(math.copysign(max(abs(a) - 4.0 * float(np.float32(0.3)), 0.0), a))
        assert b[j] == want and dl[c] == float(want) - float(beta[j])


def test_unchecked_updates_of_copies_of_one_column_diverge():
    # Section 2's remark: updating correlated variables in parallel can diverge.  64 copies of one unit
    # column updated together overshoot 63-fold per round; the dependency check (rho = 0.1) lets one copy
    # through per round and the objective falls.
    rng = np.random.default_rng(0)
    col = rng.normal(size=256)
    col -= col.mean()
    col /= np.linalg.norm(col)
    x = np.tile(col.astype(np.float32), (64, 1))
    y = (3.0 * col + 0.01 * rng.normal(size=256)).astype(np.float32)
    wild = OracleLasso(x=x, y=y, lam=0.01, rho=0.1, eta=1e-6, l_prime=64, no_deps=True, priority="uniform")
    f0 = wild.objective()
    for _ in range(6):
        out = wild.round()
        assert len(out["kept"]) == 64
    assert wild.objective() > 1e15 * f0
    with np.errstate(all="ignore"):
        for _ in range(40):
            wild.round()
    assert not np.isfinite(wild.objective())
    tame = OracleLasso(x=x, y=y, lam=0.01, rho=0.1, eta=1e-6, l_prime=64)
    for _ in range(5):
        assert len(tame.round()["kept"]) == 1
    assert tame.objective() < 0.01 * f0
