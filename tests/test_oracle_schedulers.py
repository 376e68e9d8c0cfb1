"""Pins for the oracle's other schedulers (CPU only): the linear priority |delta beta| + eta of
Algorithm 1 as printed, and the two comparison schedulers of Section 5.1 -- uniform draw with the
same dependency check ("static correlation") and uniform draw with no check (Shotgun).

Pinned by: successive-sampling probabilities for the linear weight; uniformity over subsets and
independence of delta beta for the uniform draw; for the round without a dependency check, the
textbook Jacobi step (every coordinate updated from the same residual), the closed-form
overshoot on duplicated columns, and equality with Algorithm 1's round when nothing conflicts.
"""
import itertools

import numpy as np

from oracle.oracle import OracleLasso
from synth import lasso_inputs as si


def _draws(o, dbeta, eta, l_prime, rounds, priority, seed=7):
    out = np.empty((rounds, l_prime), np.int32)
    for t in range(rounds):
        out[t] = o.draw(o.priority_keys(dbeta, eta, seed, t, priority), l_prime)
    return out


def test_linear_weight_first_and_second_draw(oracle_mod):
    dbeta = np.array([0.5, 1.0, 0.25, 2.0, 0.1], np.float32)
    eta = 1e-2
    w = np.abs(dbeta.astype(np.float64)) + eta
    W = w.sum()
    R = 60000
    d = _draws(oracle_mod, dbeta, eta, 2, R, "linear")
    cnt = np.bincount(d[:, 0], minlength=5)
    exp = R * w / W
    assert ((cnt - exp) ** 2 / exp).sum() < 30.0
    chi2 = 0.0
    for a, b in itertools.permutations(range(5), 2):
        e = R * w[a] / W * w[b] / (W - w[a])
        c = int(((d[:, 0] == a) & (d[:, 1] == b)).sum())
        chi2 += (c - e) ** 2 / e
    assert chi2 < 60.0
    # and it is not the squared weight: with delta beta = (1, 3) coordinate 1 comes first 3/4 of the time
    d = _draws(oracle_mod, np.array([1.0, 3.0], np.float32), 1e-9, 1, 40000, "linear", seed=3)
    assert abs((d[:, 0] == 1).mean() - 0.75) < 0.01
    # negative delta beta cannot occur, but the weight is defined through |.|
    assert oracle_mod.lib().oracle_priority_weight(np.float32(-2.0), np.float32(0.5), 1) == 2.5
    assert oracle_mod.lib().oracle_priority_weight(np.float32(-2.0), np.float32(0.5), 0) == 4.5
    assert oracle_mod.lib().oracle_priority_weight(np.float32(-2.0), np.float32(0.5), 2) == 1.0


def test_uniform_draw_ignores_delta_beta_and_is_uniform_over_subsets(oracle_mod):
    J, L, R = 6, 3, 40000
    rng = np.random.default_rng(0)
    a = oracle_mod.priority_keys(rng.uniform(0, 5, J).astype(np.float32), 1e-6, 11, 4, "uniform")
    b = oracle_mod.priority_keys(np.full(J, 1e6, np.float32), 1e-3, 11, 4, "uniform")
    assert np.array_equal(a, b)
    d = _draws(oracle_mod, np.array([1e6, 0, 3.0, 0.1, 1e-3, 7.0], np.float32), 1e-6, L, R, "uniform", seed=1)
    subsets = {}
    for row in d:
        key = tuple(sorted(row))
        subsets[key] = subsets.get(key, 0) + 1
    assert len(subsets) == 20
    exp = R / 20
    assert sum((c - exp) ** 2 / exp for c in subsets.values()) < 60.0
    first = np.bincount(d[:, 0], minlength=J)
    assert ((first - R / J) ** 2 / (R / J)).sum() < 35.0


def test_round_without_dependency_check_is_a_jacobi_step():
    # all J coordinates drawn, none rejected, all updated from r = y: beta_j = S(x_j^T y, lambda)
    p = si.make("c1_dense_iid", n=200, j=50, nnz=5, l_prime=50)
    s = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=50, seed=2,
                    priority="uniform", no_deps=True)
    out = s.round()
    assert sorted(out["kept"].tolist()) == list(range(50)) and out["kept_pos"].tolist() == list(range(50))
    X = p.x.numpy().astype(np.float64)
    xty = X @ p.y.numpy().astype(np.float64)
    exact = np.sign(xty) * np.maximum(np.abs(xty) - p.lam, 0)
    assert np.abs(s.beta - exact).max() < 1e-6
    assert np.abs(s.r - (p.y.numpy() - X.T @ s.beta.astype(np.float64))).max() < 1e-5
    # the cap takes the first p_max of the draw
    c = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=50, seed=2,
                    priority="uniform", no_deps=True, p_max=9)
    oc = c.round()
    assert np.array_equal(oc["kept"], out["cand"][:9])


def test_duplicated_columns_overshoot_without_the_check_and_not_with_it():
    # two identical unit columns, y = 2x, lambda = 0.5.  Alone: beta = 1.5.  Both at once from r = y:
    # beta = (1.5, 1.5), r = y - 3x = -x: F = 1/2 + 0.5*3 = 2, no better than not moving at all
    # (F(0) = 2), while the single update gives F = 1/2 * 0.25 + 0.75 = 0.875.  The dependency
    # check rejects the second column.
    x = np.zeros((2, 4), np.float32)
    x[:, 0] = 1.0
    y = np.array([2.0, 0, 0, 0], np.float32)
    a = OracleLasso(x=x, y=y, lam=0.5, rho=0.1, eta=1e-6, l_prime=2, seed=0, priority="uniform", no_deps=True)
    a.round()
    assert a.beta.tolist() == [1.5, 1.5] and a.r.tolist() == [-1.0, 0, 0, 0]
    assert a.objective() == 2.0
    b = OracleLasso(x=x, y=y, lam=0.5, rho=0.1, eta=1e-6, l_prime=2, seed=0, priority="uniform")
    ob = b.round()
    assert len(ob["kept"]) == 1 and sorted(b.beta.tolist()) == [0.0, 1.5]
    assert b.objective() == 0.875


def test_uniform_with_check_equals_shotgun_when_nothing_conflicts():
    p = si.make("c1_dense_iid", n=150, j=80, nnz=6, l_prime=16)
    kw = dict(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, eta=p.eta, l_prime=16, seed=5, priority="uniform")
    a, b = OracleLasso(rho=10.0, **kw), OracleLasso(rho=10.0, no_deps=True, **kw)
    for _ in range(10):
        oa, ob = a.round(), b.round()
        assert np.array_equal(oa["kept"], ob["kept"])
    assert np.array_equal(a.beta, b.beta) and np.array_equal(a.r, b.r)


def test_all_schedulers_reach_the_same_optimum():
    from sklearn.linear_model import Lasso
    p = si.make("c1_dense_iid", n=150, j=80, nnz=6, l_prime=8)
    ref = Lasso(alpha=p.lam / p.n, fit_intercept=False, tol=1e-14, max_iter=200000)
    ref.fit(p.x.numpy().T.astype(np.float64), p.y.numpy().astype(np.float64))
    for kw in (dict(priority="linear"), dict(priority="uniform"), dict(priority="uniform", no_deps=True, p_max=2)):
        s = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=8, seed=1, **kw)
        for _ in range(4000):
            s.round()
        assert np.abs(s.beta - ref.coef_).max() < 1e-4, kw
