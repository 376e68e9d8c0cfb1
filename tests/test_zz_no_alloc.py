"""The entry point that allocates nothing, strads_lasso_filter_static, against the existing
strads_lasso_stage_filter (same kernels, the handle's workspace instead of the library's file-scope
device array): bit-identical kept positions, on two calls in a row of which the second is smaller,
so that whatever the first call left in the shared array is there when the second runs.  The oracle's
greedy filter is the third party to both."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from synth import lasso_inputs as si

pytestmark = pytest.mark.gpu


def _gram(L, scale, rho, seed):
    rng = np.random.default_rng(seed)
    A = (rng.standard_normal((L, L)) * scale).astype(np.float32)
    G = np.triu(A, 1) + np.triu(A, 1).T + np.eye(L, dtype=np.float32)
    if L > 3:
        G[0, 2] = G[2, 0] = np.float32(rho)                                # exactly rho: a conflict
        G[0, 3] = G[3, 0] = np.nextafter(np.float32(rho), np.float32(0))    # just below: admissible
    return G


@pytest.mark.parametrize("sizes", [(3000, 700), (8192, 130), (257, 64), (1000, 1)])
def test_static_filter_equals_the_handle_filter_twice_in_a_row(sizes):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1312_5766_amd as pk
    pk.load()
    dev = torch.device("cuda:0")
    rho = 0.1
    p = si.make("c1_dense_iid", n=8, j=max(sizes), nnz=1, l_prime=max(sizes))
    # the caller's buffers, allocated once, before the calls under test
    kept_pos = torch.full((max(sizes),), -7, dtype=torch.int32, device=dev)
    n_kept = torch.full((1,), -7, dtype=torch.int32, device=dev)
    for call, L in enumerate(sizes):
        for p_max, scale in ((0, 0.035), (max(1, L // 3), 0.06)):
            G = _gram(L, scale, rho, seed=L + p_max)
            Gd = torch.from_numpy(G).to(dev)
            h = pk.StradsLasso(x=p.x.to(dev), y=p.y.to(dev), lam=p.lam, rho=rho, eta=p.eta, l_prime=p.l_prime,
                               seed=0, p_max=p_max)
            want = h.stage_filter(Gd).cpu().numpy()
            h.close()
            torch.cuda.synchronize()
            # (the allocator's count of allocations made so far: frees by the garbage collector leave it alone)
            before = torch.cuda.memory_stats(dev)["allocation.all.allocated"]
            pk.strads_lasso_filter_static(Gd, rho, p_max, kept_pos, n_kept)
            assert torch.cuda.memory_stats(dev)["allocation.all.allocated"] == before   # nothing of torch's either
            torch.cuda.synchronize()
            k = int(n_kept.item())
            got = kept_pos[:k].cpu().numpy()
            assert np.array_equal(got, want), (call, L, p_max)
            assert np.array_equal(got, orc.greedy_filter(G, rho, p_max)), (call, L, p_max)


def test_static_filter_rejects_what_it_cannot_hold():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1312_5766_amd as pk
    lib = pk.load()
    dev = torch.device("cuda:0")
    out = torch.full((4,), 5, dtype=torch.int32, device=dev)
    g = torch.eye(2, device=dev)
    too_big = pk.FILTER_STATIC_MAX_L + 1
    assert lib.strads_lasso_filter_static(g.data_ptr(), too_big, 0.1, 0, out.data_ptr(), out.data_ptr(), None) == pk.E_TOO_LARGE
    assert lib.strads_lasso_filter_static(g.data_ptr(), 2, 0.0, 0, out.data_ptr(), out.data_ptr(), None) == pk.E_INVALID_ARG
    assert lib.strads_lasso_filter_static(None, 2, 0.1, 0, out.data_ptr(), out.data_ptr(), None) == pk.E_INVALID_ARG
    torch.cuda.synchronize()
    assert out.tolist() == [5, 5, 5, 5]                                  # no output written on error
    assert b"maximum" in lib.strads_lasso_strerror(pk.E_TOO_LARGE)
