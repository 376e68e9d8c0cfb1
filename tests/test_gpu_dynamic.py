"""GPU parity of the round with update-aware ("dynamic") dependencies against the oracle's
oracle_round_dynamic, through the C ABI.

Same bars as the static round.  One more floating-point decision feeds an index here: whether a
candidate moves (its tentative change is nonzero), i.e. whether |x_j^T r + beta_j| exceeds lambda.
Both sides take it on their own fp32 result of S(z + beta, lambda) - beta; they may differ only
where that change is zero to within the dot-product tolerance on both sides (|z + beta| at lambda
for a zero coefficient, a coefficient sitting at its coordinate-wise optimum otherwise).  Such
candidates are logged and the oracle then follows the GPU's decision.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from oracle.oracle import OracleLasso
from parity_rules import GRAM_ATOL, GRAM_RTOL, check_kept_against_oracle
from synth import lasso_inputs as si

pytestmark = pytest.mark.gpu

DOT_RTOL, BETA_RTOL, OBJ_RTOL = 1e-4, 1e-4, 1e-5


def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1312_5766_amd as pk
    pk.load()
    return pk


def _pair(p, keep_gram=True, dynamic=True, **kw):
    pk = _gpu()
    dev = torch.device("cuda:0")
    args = dict(lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
    args.update(kw)
    if p.layout == "dense":
        g = pk.StradsLasso(x=p.x.to(dev), y=p.y.to(dev), keep_gram=keep_gram, dynamic=dynamic, **args)
        o = OracleLasso(x=p.x.cpu().numpy(), y=p.y.cpu().numpy(), dynamic=dynamic, **args)
    elif p.layout == "geno2":
        g = pk.StradsLasso(codes=p.codes.to(dev), col_mean=p.col_mean.to(dev), col_scale=p.col_scale.to(dev),
                           n=p.n, y=p.y.to(dev), keep_gram=keep_gram, dynamic=dynamic, **args)
        o = OracleLasso(x=p.x.cpu().numpy(), y=p.y.cpu().numpy(), dynamic=dynamic, **args)
    else:
        g = pk.StradsLasso(values=p.values.to(dev), row_idx=p.row_idx.to(dev), col_ptr=p.col_ptr.to(dev), n=p.n,
                           y=p.y.to(dev), keep_gram=keep_gram, dynamic=dynamic, **args)
        o = OracleLasso(values=p.values.cpu().numpy(), row_idx=p.row_idx.cpu().numpy(),
                        col_ptr=p.col_ptr.cpu().numpy(), n=p.n, y=p.y.cpu().numpy(), dynamic=dynamic, **args)
    return g, o


def _np(t):
    return t.detach().cpu().numpy()


def _ref_candidates(o, dbeta, t):
    """Step 1 from the oracle's stage functions.  With S scheduler shards the candidates of round t are
    the full draw order restricted to shard t mod S (pinned in tests/test_oracle_shards.py)."""
    keys = orc.priority_keys(dbeta, o.eta, o.seed, t, o.priority)
    if o.n_shards == 1:
        return orc.draw(keys, o.l_prime)
    full = orc.draw(keys, o.J)
    return full[full % o.n_shards == t % o.n_shards][:o.l_prime]


def _assert_close(got, ref, rtol, atol, what):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    err = np.abs(got - ref) - (rtol * np.abs(ref) + atol)
    assert err.size == 0 or err.max() <= 0, f"{what}: worst excess {err.max():.3e} at {err.argmax()}"


def _check_round(g, o, log, teacher_forced=True):
    if teacher_forced:
        g.set_state(o.beta, o.dbeta, o.r, o.t)
    beta0, dbeta0, r0, t0 = o.beta.copy(), o.dbeta.copy(), o.r.copy(), o.t
    g.round()
    lr = g.last_round(want_gram=True)
    lc = g.last_candidates()
    cand, kept_pos = _np(lr["cand"]), _np(lr["kept_pos"])
    ref_cand = _ref_candidates(o, dbeta0, t0)
    assert np.array_equal(cand, ref_cand), f"candidate list differs (round {t0})"
    L = len(cand)
    rn = max(float(np.linalg.norm(r0.astype(np.float64))), 1.0)

    # every candidate's dot product and tentative change: the oracle's stage functions on copies of the state
    if o.csc:
        z_ref = orc.dots_csc(o.x, o.row_idx, o.col_ptr, cand, r0)
    else:
        z_ref = orc.dots_dense(o.x, cand, r0)
    z_gpu, d_gpu = _np(lc["z_cand"]), _np(lc["delta_cand"])
    _assert_close(z_gpu, z_ref, DOT_RTOL, 1e-6 * rn, f"candidate dots (round {t0})")
    mover_gpu = d_gpu != 0
    assert lc["n_movers"] == int(mover_gpu.sum())
    d_ref = orc.update(cand, z_ref, o.lam, beta0.copy(), dbeta0.copy())
    mover_ref = d_ref != 0
    differ = mover_gpu != mover_ref
    if differ.any():
        tol = DOT_RTOL * np.abs(z_ref[differ]) + 2e-6 * rn
        assert np.all(np.abs(d_ref[differ]) <= tol) and np.all(np.abs(d_gpu[differ]) <= tol), \
            f"mover decision differs away from the threshold (round {t0})"
        log.append(("near_lambda", t0, int(differ.sum())))

    # dependencies among the movers: the GPU's L x L image must be zero outside mover pairs
    Ggpu = _np(lr["G"])
    assert np.all(Ggpu[~mover_gpu, :] == 0) and np.all(Ggpu[:, ~mover_gpu] == 0)
    mm = np.ix_(mover_gpu, mover_gpu)
    Gref_full = orc.gram_csc(o.x, o.row_idx, o.col_ptr, cand) if o.csc else orc.gram_dense(o.x, cand)
    _assert_close(Ggpu[mm], Gref_full[mm], GRAM_RTOL, GRAM_ATOL, f"mover gram (round {t0})")
    assert np.array_equal(Ggpu, Ggpu.T)
    # the kept set is the greedy result under d_t on the GPU's own values, bit-exact
    assert np.array_equal(kept_pos, orc.greedy_filter(Ggpu, o.rho, o.p_max)), f"filter differs (round {t0})"
    Gref_dt = Gref_full.copy()
    Gref_dt[~mover_gpu, :] = 0
    Gref_dt[:, ~mover_gpu] = 0
    check_kept_against_oracle(Gref_dt, kept_pos, orc.greedy_filter(Gref_dt, o.rho, o.p_max), o.rho, o.p_max, log,
                              f"round {t0}", G_gpu=Ggpu)

    out = o.round(forced_cand=cand, forced_mover=mover_gpu.astype(np.uint8), forced_kept_pos=kept_pos)
    _assert_close(_np(lr["z"]), out["z"], DOT_RTOL, 1e-6 * rn, f"dots (round {t0})")
    _assert_close(_np(lr["delta"]), out["delta"], BETA_RTOL, 2e-6 * rn, f"delta (round {t0})")
    beta, dbeta, r, t = g.get_state()
    assert t == o.t
    _assert_close(_np(beta), o.beta, BETA_RTOL, 2e-6 * rn, f"beta (round {t0})")
    _assert_close(_np(dbeta), o.dbeta, BETA_RTOL, 2e-6 * rn, f"delta beta (round {t0})")
    _assert_close(_np(r), o.r, DOT_RTOL, 2e-6 * rn, f"residual (round {t0})")
    if teacher_forced:
        untouched = np.ones(o.J, bool)
        untouched[out["kept"]] = False
        assert np.array_equal(_np(beta)[untouched], beta0[untouched])
        assert np.array_equal(_np(dbeta)[untouched], dbeta0[untouched])
        nonmovers_kept = out["kept"][~mover_gpu[kept_pos]]
        assert np.all(_np(dbeta)[nonmovers_kept] == 0) and np.array_equal(_np(beta)[nonmovers_kept], beta0[nonmovers_kept])
    return lc["n_movers"], len(kept_pos)


@pytest.mark.parametrize("config,kw,rounds", [
    ("c1_dense_iid", dict(n=1000, j=5000, l_prime=200), 30),
    ("c2_dense_block_corr", dict(n=2000, j=8000, nnz=40, l_prime=500), 24),
    ("c3_genotype", dict(n=500, j=6000, nnz=20, l_prime=600), 20),
    ("c5_dense_duplicates", dict(n=1500, j=6000, nnz=40, l_prime=1300), 12),
    ("c2_dense_block_corr", dict(n=1001, j=900, nnz=30, l_prime=300, lam=0.0), 4),     # everything moves
])
def test_teacher_forced_rounds(config, kw, rounds):
    lam = kw.pop("lam", None)
    p = si.make(config, **kw)
    extra = {} if lam is None else dict(lam=lam)
    g, o = _pair(p, **extra)
    log, seen_movers = [], 0
    for _ in range(rounds):
        m, k = _check_round(g, o, log)
        seen_movers = max(seen_movers, m)
    assert seen_movers > 0
    print(f"{config}: most movers in a round {seen_movers}; logged {log}")


def test_cap_on_the_kept_set():
    p = si.make("c2_dense_block_corr", n=1000, j=3000, nnz=30, l_prime=300)
    g, o = _pair(p, p_max=77)
    for _ in range(6):
        m, k = _check_round(g, o, [])
        assert k == 77


def test_no_conflicts_equals_the_static_round_bit_for_bit():
    # rho above every correlation: nothing is ever rejected in either variant, and both variants
    # compute the dot products with the same kernel code, so the states must be identical
    pk = _gpu()
    dev = torch.device("cuda:0")
    p = si.make("c2_dense_block_corr", n=2000, j=4000, nnz=30, l_prime=400)
    kw = dict(x=p.x.to(dev), y=p.y.to(dev), lam=p.lam, rho=10.0, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
    a, b = pk.StradsLasso(**kw), pk.StradsLasso(dynamic=True, **kw)
    for _ in range(15):
        a.round(); b.round()
    sa, sb = a.get_state(), b.get_state()
    for u, v in zip(sa[:3], sb[:3]):
        assert torch.equal(u, v)
    assert a.objective() == b.objective()


def test_free_run_tracks_the_oracle_and_is_deterministic():
    p = si.make("c1_dense_iid", n=1000, j=5000, l_prime=200)
    g, o = _pair(p, keep_gram=False)
    g2, _ = _pair(p, keep_gram=False)
    for t in range(40):
        g.round(); g2.round(); o.round()
        fg, fo = g.objective(), o.objective()
        assert abs(fg - fo) <= OBJ_RTOL * abs(fo), (t, fg, fo)
    for u, v in zip(g.get_state()[:3], g2.get_state()[:3]):
        assert torch.equal(u, v)


def test_degenerate_cases():
    pk = _gpu()
    dev = torch.device("cuda:0")
    # lambda above max |x^T y|: nobody ever moves, every candidate is kept, beta stays 0
    p = si.make("c1_dense_iid", n=300, j=500, nnz=5, l_prime=64)
    g, o = _pair(p, lam=1e3)
    for _ in range(3):
        m, k = _check_round(g, o, [])
        assert m == 0 and k == 64
    assert float(g.get_state()[0].abs().max()) == 0.0
    # one column, one candidate; and L' = J
    for j, lp in ((1, 1), (7, 7), (130, 130)):
        p = si.make("c1_dense_iid", n=64, j=j, nnz=1, l_prime=lp)
        g, o = _pair(p)
        for _ in range(3):
            _check_round(g, o, [])


def test_csc_design_teacher_forced():
    for kw, rounds in ((dict(n=3000, j=6000, nnz_per_col=30, nnz=30, l_prime=300), 16),
                       (dict(n=500, j=2000, nnz_per_col=60, nnz=20, l_prime=700, rho=0.2), 10)):
        p = si.make("c4_sparse_csc", **kw)
        g, o = _pair(p)
        log, most = [], 0
        for _ in range(rounds):
            m, k = _check_round(g, o, log)
            most = max(most, m)
        assert most > 0
        print("csc", kw, "most movers", most, log)


def test_run_reaches_the_lasso_solution():
    p = si.make("c1_dense_iid", n=400, j=600, nnz=10, l_prime=100)
    g, o = _pair(p, keep_gram=False)
    info = g.run(4000, kkt_tol=1e-4, check_every=50)
    assert info.converged == 1
    viol = g.kkt()
    assert viol <= 1e-4 * p.lam * 1.01
    for _ in range(3000):
        o.round()
    _assert_close(_np(g.get_state()[0]), o.beta, 1e-3, 1e-4, "converged beta")


def test_full_size_config2_three_rounds():
    # the bench workload at full size (N=10000, J=100000, L'=1000), in the launch shape the bench times
    p = si.make("c2_dense_block_corr", device=torch.device("cuda:0"))
    pk = _gpu()
    g = pk.StradsLasso(x=p.x, y=p.y, lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed,
                       keep_gram=True, dynamic=True)
    o = OracleLasso(x=p.x.cpu().numpy(), y=p.y.cpu().numpy(), lam=p.lam, rho=p.rho, eta=p.eta,
                    l_prime=p.l_prime, seed=p.seed, dynamic=True)
    log = []
    for _ in range(3):
        m, k = _check_round(g, o, log)
        print("movers", m, "kept", k)
