"""GPU parity for a design stored as packed 2-bit genotype counts (the form of the paper's
Alzheimer's-disease SNP matrix, Section 5: entries 0/1/2, standardised columns).

The library decodes x_ij = fl(fl(g_ij - mean_j) * scale_j) on the fly; the oracle is handed that
fp32 matrix, written out by synth.lasso_inputs.decode_genotypes from the same codes.  Everything
else -- bars, teacher forcing, admissible index differences -- is as for the fp32 layouts.
"""
import numpy as np
import pytest
import torch

from synth import lasso_inputs as si
from test_gpu_parity import DOT_RTOL, OBJ_RTOL, _assert_close, _check_round, _gpu, _np, _pair
import test_gpu_dynamic as dyn

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kw,rounds", [
    (dict(n=500, j=20000, nnz=20, l_prime=700), 8),          # the third configuration's row count, fewer columns
    (dict(n=463, j=3000, nnz=10, l_prime=300), 6),           # last word of a column partly filled
    (dict(n=64, j=500, nnz=5, l_prime=130), 5),              # exactly one 16-byte group per column
    (dict(n=17, j=300, nnz=4, l_prime=64), 5),
    (dict(n=5, j=7, nnz=2, l_prime=7), 4),                   # one word per column, every column a candidate
    (dict(n=129, j=70000, nnz=10, l_prime=200), 3),          # enough columns for the persistent pass over all of them
    (dict(n=5000, j=1500, nnz=10, l_prime=257), 5),          # several row blocks in the residual update
])
def test_teacher_forced_rounds(kw, rounds):
    p = si.make("c3_genotype_packed", **kw)
    g, o = _pair(p)
    log = []
    for _ in range(rounds):
        assert _check_round(g, o, log, teacher_forced=True)
        assert g.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)
    v, gg = g.kkt(want_g=True)
    v_ref, g_ref = o.kkt(want_g=True)
    rn = float(np.linalg.norm(o.r.astype(np.float64)))
    _assert_close(_np(gg), g_ref, DOT_RTOL, 1e-6 * max(rn, 1.0), "x_j^T r for all columns")
    assert v == pytest.approx(v_ref, rel=1e-3, abs=1e-6 * max(rn, 1.0))
    print("logged:", log)


@pytest.mark.parametrize("kw,forced", [(dict(n=500, j=2300, nnz=20, l_prime=2000), False),
                                       (dict(n=463, j=3000, nnz=10, l_prime=300), True),
                                       (dict(n=17, j=300, nnz=4, l_prime=130), True),
                                       (dict(n=5, j=7, nnz=2, l_prime=7), True)])
def test_rounds_with_the_gram_in_64_wide_tiles(kw, forced):
    """The tile kernel for long lists over short columns (64 x 64 tiles that write the conflict bits themselves)
    on the packed design: by default at the third configuration's list length, forced onto shorter lists."""
    p = si.make("c3_genotype_packed", **kw)
    g, o = _pair(p)
    if forced:
        g.set_tuning("gram_direct", 2)
    assert g.gram_tile_edge() == 64
    log = []
    for _ in range(4):
        assert _check_round(g, o, log, teacher_forced=True)
    print("logged:", log)


def test_same_trajectory_as_the_decoded_fp32_design():
    # the decoded matrix given as a dense fp32 design: identical candidate lists and kept sets,
    # beta and r equal up to summation order
    pk = _gpu()
    p = si.make("c3_genotype_packed", n=500, j=8000, nnz=20, l_prime=500)
    g, _ = _pair(p, keep_gram=False)
    dev = torch.device("cuda:0")
    d = pk.StradsLasso(x=p.x.to(dev), y=p.y.to(dev), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
    for t in range(10):
        d.set_state(*g.get_state())
        g.round()
        d.round()
        a, b = g.last_round(), d.last_round()
        assert torch.equal(a["cand"], b["cand"])
        assert torch.equal(a["kept"], b["kept"]), t
        _assert_close(_np(a["z"]), _np(b["z"]), DOT_RTOL, 1e-5, "dots")
        _assert_close(_np(g.get_state()[2]), _np(d.get_state()[2]), DOT_RTOL, 1e-5, "residual")


def test_free_run_is_deterministic_and_tracks_the_oracle():
    p = si.make("c3_genotype_packed", n=500, j=6000, nnz=20, l_prime=400)
    a, _ = _pair(p, keep_gram=False)
    b, _ = _pair(p, keep_gram=False)
    ia, ib = a.run(25), b.run(25)
    assert ia.updates_done == ib.updates_done and ia.objective == ib.objective
    for u, v in zip(a.get_state()[:3], b.get_state()[:3]):
        assert torch.equal(u, v)
    c, o = _pair(p)
    log = []
    for _ in range(25):
        if not _check_round(c, o, log, teacher_forced=False):
            o.set_state(*[_np(x) if isinstance(x, torch.Tensor) else x for x in c.get_state()])
        assert c.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)
    for u, v in zip(a.get_state()[:3], c.get_state()[:3]):
        assert torch.equal(u, v)                              # round() and run() take the same path


def test_run_reaches_the_lasso_solution():
    from sklearn.linear_model import Lasso
    p = si.make("c3_genotype_packed", n=200, j=600, nnz=8, l_prime=64, lam_frac=0.2)
    g, _ = _pair(p, keep_gram=False)
    info = g.run(30000, kkt_tol=1e-4, check_every=100)
    assert info.converged == 1
    ref = Lasso(alpha=p.lam / p.n, fit_intercept=False, tol=1e-13, max_iter=500000)
    ref.fit(p.x.numpy().T.astype(np.float64), p.y.numpy().astype(np.float64))
    _assert_close(_np(g.get_state()[0]), ref.coef_, 1e-3, 2e-4, "converged beta")


def test_dynamic_dependencies_on_packed_design():
    p = si.make("c3_genotype_packed", n=500, j=6000, nnz=20, l_prime=600)
    g, o = dyn._pair(p)
    log, seen = [], 0
    for _ in range(12):
        m, _k = dyn._check_round(g, o, log)
        seen = max(seen, m)
    assert seen > 0
    print("most movers:", seen, "logged:", log)


def test_shards_on_packed_design():
    p = si.make("c3_genotype_packed", n=500, j=9001, nnz=20, l_prime=300)
    g, o = _pair(p, n_shards=4)
    log = []
    for _ in range(12):
        assert _check_round(g, o, log, teacher_forced=True)
    a, _ = _pair(p, keep_gram=False, n_shards=4)
    b, _ = _pair(p, keep_gram=False, n_shards=4)
    a.run(40)
    for _ in range(40):
        b.round()
    for u, v in zip(a.get_state()[:3], b.get_state()[:3]):
        assert torch.equal(u, v)                              # overlapped rounds == serialised rounds


def test_create_checks_the_packed_arguments():
    pk = _gpu()
    p = si.make("c3_genotype_packed", n=100, j=50, nnz=4, l_prime=10)
    dev = torch.device("cuda:0")
    codes, mean, scale, y = p.codes.to(dev), p.col_mean.to(dev), p.col_scale.to(dev), p.y.to(dev)
    kw = dict(lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, n=p.n, y=y)
    pk.StradsLasso(codes=codes, col_mean=mean, col_scale=scale, **kw).close()
    cfg_err = []
    for bad in ("col_mean", "col_scale"):
        args = dict(codes=codes, col_mean=mean, col_scale=scale)
        args[bad] = None
        try:
            pk.StradsLasso(**args, **kw)
        except (pk.StradsError, AssertionError, AttributeError) as e:
            cfg_err.append(e)
    assert len(cfg_err) == 2


def test_full_size_config3_rounds_on_sampled_outputs():
    # 500 x 500000 packed (125 x 16 B per column): three rounds at full size, checked on sampled
    # outputs against the oracle's stage functions on decoded columns
    from oracle import oracle as orc
    pk = _gpu()
    dev = torch.device("cuda:0")
    p = si.make("c3_genotype_packed", device=dev, keep_dense=False)

    def decoded(ids):
        i = torch.as_tensor(np.asarray(ids), device=dev, dtype=torch.int64)
        return si.decode_genotypes(p.codes[i], p.col_mean[i], p.col_scale[i], p.n).cpu().numpy()

    g = pk.StradsLasso(codes=p.codes, col_mean=p.col_mean, col_scale=p.col_scale, n=p.n, y=p.y, lam=p.lam,
                       rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed, keep_gram=True)
    rng = np.random.default_rng(0)
    for t in range(3):
        beta0, dbeta0, r0, _ = [_np(a) if isinstance(a, torch.Tensor) else a for a in g.get_state()]
        g.round()
        lr = g.last_round(want_gram=True)
        cand, kept_pos = _np(lr["cand"]), _np(lr["kept_pos"])
        keys = orc.priority_keys(dbeta0, p.eta, p.seed, t, "squared")
        assert np.array_equal(cand, orc.draw(keys, p.l_prime))
        xc = decoded(cand)
        Ggpu = _np(lr["G"])
        _assert_close(Ggpu, orc.gram_dense(xc, np.arange(len(cand), dtype=np.int32)), DOT_RTOL, 1e-6, "gram")
        assert np.array_equal(kept_pos, orc.greedy_filter(Ggpu, p.rho, 0))
        kept = cand[kept_pos]
        z_ref = xc[kept_pos].astype(np.float64) @ r0.astype(np.float64)
        rn = max(float(np.linalg.norm(r0.astype(np.float64))), 1.0)
        _assert_close(_np(lr["z"]), z_ref, DOT_RTOL, 1e-6 * rn, "dots")
        a = z_ref + beta0[kept]
        nb = np.sign(a) * np.maximum(np.abs(a) - p.lam, 0)
        beta, dbeta, r, _ = g.get_state()
        _assert_close(_np(beta)[kept], nb, 1e-4, 2e-6 * rn, "beta")
        r_ref = r0.astype(np.float64) - (nb - beta0[kept]) @ xc[kept_pos].astype(np.float64)
        _assert_close(_np(r), r_ref, DOT_RTOL, 2e-6 * rn, "residual")
        # optimality pass on sampled columns
        v, gg = g.kkt(want_g=True)
        ids = np.sort(rng.choice(p.j, 4000, replace=False))
        xs = decoded(ids).astype(np.float64)
        _assert_close(_np(gg)[ids], xs @ _np(r).astype(np.float64), DOT_RTOL, 1e-6 * rn, "x_j^T r sampled")
