"""Pins for the oracle's logistic-loss round (CPU only).  Section 2.1 allows the logistic loss in
eq. (1) and gives no formula; the oracle's reading is: labels in {-1, +1}, coordinate update =
minimiser of the quadratic upper bound with curvature 1/4 (unit-norm columns).

Pinned by: the closed-form zero-solution threshold lambda >= max |X^T y| / 2; finite differences of
the objective against the dot products the update uses (sign, index and formula of the weights);
the sufficient-decrease inequality of a majorisation step with exactly that curvature; the fixed
point against scikit-learn's l1-penalised logistic regression; the optimality conditions at
convergence; the state vector against -X beta recomputed from scratch.
"""
import numpy as np
import pytest

from oracle import oracle as orc
from oracle.oracle import OracleLasso
from synth import lasso_inputs as si


def _problem(n=120, j=60, nnz=6, l_prime=12, **kw):
    return si.with_labels(si.make("c1_dense_iid", n=n, j=j, nnz=nnz, l_prime=l_prime), **kw)


def _solver(p, **kw):
    args = dict(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=3,
                loss="logistic")
    args.update(kw)
    return OracleLasso(**args)


def _loss(X, y, beta):
    m = X.T @ beta
    return float(np.sum(np.logaddexp(0.0, -y * m)))


def test_labels_and_initial_state():
    p = _problem()
    y = p.y.numpy()
    assert set(np.unique(y)) == {-1.0, 1.0} and 0.2 < (y > 0).mean() < 0.8
    s = _solver(p)
    assert not s.r.any() and not s.beta.any()
    assert np.array_equal(s.dots_vector(), (y / 2).astype(np.float32))        # w = y / 2 at beta = 0
    assert s.objective() == pytest.approx(p.n * np.log(2.0), rel=1e-12)


def test_nothing_moves_from_half_the_largest_correlation_upwards():
    p = _problem()
    X, y = p.x.numpy().astype(np.float64), p.y.numpy().astype(np.float64)
    lam0 = np.abs(X @ y).max() / 2
    s = _solver(p, lam=float(np.float32(lam0 * 1.0001)), l_prime=p.j)
    for _ in range(3):
        out = s.round()
        assert not np.any(out["delta"]) and not s.beta.any() and not s.r.any()
    # just below the threshold the coordinate with the largest |x_j^T y| moves, and only it can
    jmax = int(np.abs(X @ y).argmax())
    s = _solver(p, lam=float(np.float32(lam0 * 0.98)), l_prime=p.j, rho=10.0)
    s.round()
    assert s.beta[jmax] != 0 and np.sign(s.beta[jmax]) == np.sign((X @ y)[jmax])
    assert np.all(np.abs(X @ y)[s.beta != 0] / 2 > lam0 * 0.98)


def test_dot_products_are_minus_the_gradient_of_the_loss():
    p = _problem(n=80, j=30, l_prime=30)
    X, y = p.x.numpy().astype(np.float64), p.y.numpy().astype(np.float64)
    rng = np.random.default_rng(0)
    beta = (rng.standard_normal(p.j) * 0.3).astype(np.float32)
    s = _solver(p, lam=0.0)
    v = (-(X.T @ beta.astype(np.float64))).astype(np.float32)
    s.set_state(beta, np.ones(p.j, np.float32), v, 0)
    assert s.objective() == pytest.approx(_loss(X, y, beta.astype(np.float64)), rel=1e-6)
    _, g = s.kkt(want_g=True)                                   # g_j = x_j^T w
    h = 1e-5
    for j in range(p.j):
        e = np.zeros(p.j)
        e[j] = h
        fd = (_loss(X, y, beta + e) - _loss(X, y, beta - e)) / (2 * h)
        assert g[j] == pytest.approx(-fd, abs=2e-5), j


def test_sequential_updates_decrease_the_objective_by_at_least_the_majoriser_bound():
    # one coordinate per round: F_old - F_new >= (kappa / 2) delta^2 with kappa = 1/4, and the bound is
    # what the step minimises: a step twice as long (curvature 1/8) breaks the inequality somewhere
    p = _problem(n=150, j=40, nnz=5, l_prime=8)
    s = _solver(p, p_max=1)
    f = s.objective()
    worst = np.inf
    for _ in range(400):
        out = s.round()
        f_new = s.objective()
        d = float(out["delta"][0]) if len(out["delta"]) else 0.0
        # (the state vector is fp32: the objective carries rounding noise of about 1e-7 of its value)
        assert f - f_new >= 0.125 * d * d - 2e-5
        if abs(d) > 0.03:
            worst = min(worst, (f - f_new) / (d * d))
        f = f_new
    assert worst < 0.5                                # the bound is not vacuous: some step comes close to it


def test_fixed_point_matches_scikit_learn_and_satisfies_the_optimality_conditions():
    from sklearn.linear_model import LogisticRegression
    p = _problem(n=200, j=50, nnz=6, l_prime=10, lam_frac=0.15)
    X, y = p.x.numpy().astype(np.float64), p.y.numpy().astype(np.float64)
    s = _solver(p)
    for _ in range(6000):
        s.round()
    v, g = s.kkt(want_g=True)
    assert v < 1e-5
    assert np.all(np.abs(g[s.beta == 0]) <= p.lam + 1e-5)
    nzb = s.beta != 0
    assert nzb.any() and np.allclose(g[nzb], p.lam * np.sign(s.beta[nzb]), atol=1e-5)
    # scikit-learn minimises ||w||_1 + C sum log(1 + exp(-y x.w)): C = 1 / lambda
    ref = LogisticRegression(penalty="l1", solver="liblinear", C=1.0 / p.lam, fit_intercept=False, tol=1e-10,
                             max_iter=100000)
    ref.fit(X.T, y)
    assert np.abs(s.beta - ref.coef_[0]).max() < 2e-3
    f_ref = _loss(X, y, ref.coef_[0]) + p.lam * np.abs(ref.coef_[0]).sum()
    assert s.objective() <= f_ref * (1 + 1e-7)        # at least as good a minimiser
    # the state vector is -X beta
    assert np.abs(s.r + X.T @ s.beta.astype(np.float64)).max() < 1e-5


def test_dynamic_dependencies_and_other_schedulers_reach_the_same_fixed_point():
    p = _problem(n=150, j=40, nnz=5, l_prime=8, lam_frac=0.2)
    ref = _solver(p)
    for _ in range(5000):
        ref.round()
    for kw in (dict(dynamic=True), dict(priority="uniform"), dict(n_shards=3)):
        s = _solver(p, **kw)
        for _ in range(5000):
            s.round()
        assert np.abs(s.beta - ref.beta).max() < 1e-4, kw
