"""Replaying a recorded HIP graph of rounds (strads_lasso_run) against enqueueing the same rounds one
by one: the two must be bit-identical, on every replay, with eager work between the replays."""
import pytest
import torch

from synth import lasso_inputs as si

pytestmark = pytest.mark.gpu


def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1312_5766_amd as pk
    pk.load()
    return pk


@pytest.mark.parametrize("kw", [dict(), dict(n_shards=3), dict(dynamic=True), dict(n_shards=2, dynamic=True),
                                dict(priority="uniform", no_deps=True, p_max=64), dict(tile256=True),
                                dict(tile256=True, n_shards=2), dict(direct=True), dict(direct=True, n_shards=2)])
def test_graph_replays_equal_eager_rounds(kw):
    pk = _gpu()
    kw = dict(kw)
    tile256 = kw.pop("tile256", False)      # the Gram in 256-wide tiles from a queue, whose position the mask kernel resets
    direct = kw.pop("direct", False)        # the Gram in 64-wide tiles that write the conflict bits themselves
    dev = torch.device("cuda:0")
    p = si.make("c2_dense_block_corr", n=1000, j=3000, nnz=20, l_prime=300)
    side = torch.cuda.Stream(dev)               # the legacy default stream cannot be captured
    with torch.cuda.stream(side):
        base = dict(x=p.x.to(dev), y=p.y.to(dev), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
        g = pk.StradsLasso(**base, **kw)        # replays graphs of 4 rounds
        e = pk.StradsLasso(**base, **kw)        # never uses graphs
        if tile256:
            g.set_tuning("gram_tile256", 2)
            e.set_tuning("gram_tile256", 2)
            assert g.gram_tile_edge() == e.gram_tile_edge() == 256
        if direct:
            g.set_tuning("gram_direct", 2)
            e.set_tuning("gram_direct", 2)
            assert g.gram_tile_edge() == e.gram_tile_edge() == 64
        g.set_tuning("graph_rounds", 4)
        e.set_tuning("graph_rounds", 0)
        total = 0
        for chunk in (4, 9, 3, 8, 13):          # replays, left-over rounds, a chunk below one graph
            ig, ie = g.run(chunk), e.run(chunk)
            total += chunk
            assert ig.rounds_done == ie.rounds_done == chunk and ig.updates_done == ie.updates_done
            assert ig.graph_replays == chunk // 4 and ie.graph_replays == 0
            sg, se = g.get_state(), e.get_state()
            for u, v in zip(sg[:3], se[:3]):
                assert torch.equal(u, v), (kw, total)
            assert sg[3] == se[3] == total
            assert g.objective() == e.objective()
            g.round(); e.round()                # an eager round between replays keeps the counters in step
            total += 1
            assert torch.equal(g.get_state()[0], e.get_state()[0])
        # a state restored with its round index continues identically through a replay
        beta, dbeta, r, t = e.get_state()
        g.set_state(beta, dbeta, r, t)
        g.run(8); e.run(8)
        for u, v in zip(g.get_state()[:3], e.get_state()[:3]):
            assert torch.equal(u, v)


def test_default_stream_falls_back_to_eager_rounds():
    pk = _gpu()
    dev = torch.device("cuda:0")
    p = si.make("c1_dense_iid", n=300, j=800, nnz=5, l_prime=64)
    base = dict(x=p.x.to(dev), y=p.y.to(dev), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
    a, b = pk.StradsLasso(**base), pk.StradsLasso(**base)
    a.set_tuning("graph_rounds", 8)             # asked for, but the legacy default stream cannot be captured
    ia = a.run(40); b.run(40)
    assert ia.graph_replays == 0                # capture refused, rounds enqueued one by one
    assert torch.equal(a.get_state()[0], b.get_state()[0])
