"""GPU parity of sharded scheduling (Section 3: S scheduler shards taking turns) against the oracle.

The shards' scheduling work runs on separate streams and overlaps; the updates are applied in round
order.  Besides the usual per-round parity this checks that the overlap changes nothing: a run
enqueued in one call is bit-identical to the same rounds enqueued one call at a time (which
serialises the shards), and two runs are bit-identical to each other."""
import numpy as np
import pytest
import torch

from oracle.oracle import OracleLasso
from synth import lasso_inputs as si
from test_gpu_parity import _check_round, _gpu, _np, _pair

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kw", [dict(n_shards=2), dict(n_shards=3), dict(n_shards=8, priority="uniform"),
                                dict(n_shards=2, no_deps=True, p_max=150)])
def test_teacher_forced_rounds(kw):
    p = si.make("c2_dense_block_corr", n=2000, j=8001, nnz=40, l_prime=400)
    g, o = _pair(p, **kw)
    log = []
    for _ in range(3 * kw["n_shards"] + 2):
        assert _check_round(g, o, log, teacher_forced=True)
    print(kw, log)


def test_dynamic_dependencies_with_shards():
    from test_gpu_dynamic import _check_round as check, _pair as pair
    p = si.make("c2_dense_block_corr", n=2000, j=8000, nnz=40, l_prime=500)
    g, o = pair(p, n_shards=3)
    for _ in range(12):
        check(g, o, [])


def test_csc_design_with_shards():
    p = si.make("c4_sparse_csc", n=3000, j=6000, nnz_per_col=30, nnz=30, l_prime=300)
    g, o = _pair(p, n_shards=2)
    for _ in range(8):
        assert _check_round(g, o, [], teacher_forced=True)


def test_one_coordinate_per_shard_is_cyclic_coordinate_descent():
    pk = _gpu()
    dev = torch.device("cuda:0")
    p = si.make("c1_dense_iid", n=80, j=8, nnz=3, l_prime=1)
    g = pk.StradsLasso(x=p.x.to(dev), y=p.y.to(dev), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=1, n_shards=8)
    X = p.x.numpy().astype(np.float64).T
    y = p.y.numpy().astype(np.float64)
    b = np.zeros(8)
    for sweep in range(5):
        g.run(8)
        for j in range(8):
            a = X[:, j] @ (y - X @ b) + b[j]
            b[j] = np.sign(a) * max(abs(a) - p.lam, 0)
        assert np.abs(_np(g.get_state()[0]) - b).max() < 1e-5


@pytest.mark.parametrize("kw", [dict(n_shards=2), dict(n_shards=4), dict(n_shards=3, dynamic=True),
                                dict(n_shards=2, tile256=True), dict(n_shards=2, tile256=True, shape=(400, 8000, 2600)),
                                dict(n_shards=2, shape=(400, 8000, 2600), edge=64)])
def test_overlapped_run_equals_serialised_rounds_and_tracks_the_oracle(kw):
    pk = _gpu()
    dev = torch.device("cuda:0")
    kw = dict(kw)
    tile256 = kw.pop("tile256", False)      # the shards' Gram kernels in 256-wide tiles, each with a queue of its own
    # (2600 candidates: 41 mask words per row, where the greedy walk skips the chunks of candidates that the
    # shard's own slot sum has not marked; the marks of overlapping shards must not mix)
    n, j, l_prime = kw.pop("shape", (2000, 8000, 500))
    edge = kw.pop("edge", 0)                # (the last case: short columns under a long list, 64-wide tiles by default)
    p = si.make("c2_dense_block_corr", n=n, j=j, nnz=40, l_prime=l_prime)
    base = dict(x=p.x.to(dev), y=p.y.to(dev), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
    a, b, c = (pk.StradsLasso(**base, **kw) for _ in range(3))
    if tile256:
        for h in (a, b, c):
            h.set_tuning("gram_tile256", 2)
            assert h.gram_tile_edge() == 256
    if edge:
        assert a.gram_tile_edge() == edge
    o = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed, **kw)
    R = 40
    ia = a.run(R)                           # one call: the shards overlap
    ic = c.run(R)
    for _ in range(R):
        b.round()                           # one call per round: each call joins the shards
        o.round()
    for u, v, w in zip(a.get_state()[:3], b.get_state()[:3], c.get_state()[:3]):
        assert torch.equal(u, v) and torch.equal(u, w)
    assert ia.updates_done == ic.updates_done > 0
    fo = o.objective()
    assert abs(a.objective() - fo) <= 1e-5 * abs(fo)


def test_create_rejects_bad_shard_counts():
    pk = _gpu()
    dev = torch.device("cuda:0")
    p = si.make("c1_dense_iid", n=64, j=5, nnz=1, l_prime=2)
    for bad in (9, 6):
        with pytest.raises(pk.StradsError):
            pk.StradsLasso(x=p.x.to(dev), y=p.y.to(dev), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=2, n_shards=bad)
    g = pk.StradsLasso(x=p.x.to(dev), y=p.y.to(dev), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=2, n_shards=2)
    with pytest.raises(pk.StradsError) as e:
        g.set_tuning("profile_level", 1)
    assert e.value.code == pk.E_UNSUPPORTED
