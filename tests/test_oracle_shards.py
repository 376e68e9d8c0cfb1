"""Pins for the oracle's sharded schedulers (Section 3: S scheduler threads, each owning a fixed
disjoint set of coordinates, taking turns): CPU only.

Pinned by: the degenerate sharding S = J with P' = 1, which is textbook cyclic coordinate descent;
the draw law restricted to the shard in turn; the full-order-restricted-to-the-shard identity of
the candidate list; the same fixed point as the unsharded solver."""
import numpy as np

from oracle import oracle as orc
from oracle.oracle import OracleLasso
from synth import lasso_inputs as si


def _small(n=120, j=60, seed=0, **kw):
    kw.setdefault("nnz", 6)
    kw.setdefault("l_prime", 20)
    return si.make("c1_dense_iid", n=n, j=j, seed=seed, **kw)


def test_one_coordinate_per_shard_is_cyclic_coordinate_descent():
    p = _small(n=80, j=12, seed=2, l_prime=1)
    s = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=1, seed=4, n_shards=12)
    X = p.x.numpy().astype(np.float64).T
    y = p.y.numpy().astype(np.float64)
    b = np.zeros(12)
    for sweep in range(6):
        for j in range(12):
            out = s.round()
            assert out["cand"].tolist() == [j] and out["kept"].tolist() == [j]
            a = X[:, j] @ (y - X @ b) + b[j]
            b[j] = np.sign(a) * max(abs(a) - p.lam, 0)
        assert np.abs(s.beta - b).max() < 2e-6


def test_a_round_touches_only_the_shard_in_turn():
    p = _small(seed=3, l_prime=10)
    S = 4
    s = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=10, seed=1, n_shards=S)
    for t in range(24):
        before = s.beta.copy(), s.dbeta.copy()
        out = s.round()
        assert np.all(out["cand"] % S == t % S) and len(set(out["cand"].tolist())) == len(out["cand"]) == 10
        others = np.arange(p.j) % S != t % S
        assert np.array_equal(s.beta[others], before[0][others]) and np.array_equal(s.dbeta[others], before[1][others])
    # the candidate count is clamped to the shard size: 60 coordinates in 4 shards of 15
    big = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=50, seed=1, n_shards=S)
    assert len(big.round()["cand"]) == 15


def test_candidates_are_the_full_order_restricted_to_the_shard():
    p = _small(n=50, j=200, seed=5, l_prime=17)
    S = 3
    s = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=17, seed=9, n_shards=S)
    rng = np.random.default_rng(0)
    for t in range(9):
        s.dbeta[:] = np.abs(rng.normal(size=p.j)).astype(np.float32)
        keys = orc.priority_keys(s.dbeta, s.eta, s.seed, t)
        full = orc.draw(keys, p.j)
        want = [j for j in full.tolist() if j % S == t % S][:17]
        assert s.round()["cand"].tolist() == want


def test_first_draw_follows_the_priority_within_the_shard():
    dbeta = np.array([0.5, 9.0, 1.0, 9.0, 0.25, 9.0], np.float32)     # shard 0 of 2 = coordinates 0, 2, 4
    w = dbeta[[0, 2, 4]].astype(np.float64) ** 2 + 1e-2
    x = np.eye(6, 8, dtype=np.float32)
    y = np.zeros(8, np.float32)
    s = OracleLasso(x=x, y=y, lam=1.0, rho=0.5, eta=1e-2, l_prime=1, seed=3, n_shards=2)
    cnt = np.zeros(6)
    R = 30000
    for i in range(R):
        s.set_state(np.zeros(6, np.float32), dbeta, y, 2 * i)        # even rounds: shard 0
        cnt[s.round()["cand"][0]] += 1
    assert cnt[[1, 3, 5]].sum() == 0
    exp = R * w / w.sum()
    assert ((cnt[[0, 2, 4]] - exp) ** 2 / exp).sum() < 25.0


def test_sharded_solver_reaches_the_same_optimum():
    from sklearn.linear_model import Lasso
    p = _small(n=150, j=80, seed=4, l_prime=8)
    ref = Lasso(alpha=p.lam / p.n, fit_intercept=False, tol=1e-14, max_iter=200000)
    ref.fit(p.x.numpy().T.astype(np.float64), p.y.numpy().astype(np.float64))
    for kw in (dict(n_shards=2), dict(n_shards=5, dynamic=True)):
        s = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=8, seed=1, **kw)
        for _ in range(4000):
            s.round()
        assert np.abs(s.beta - ref.coef_).max() < 1e-4, kw
