"""GPU parity: libstrads_lasso (through its C ABI) against the CPU oracle on the same seeded inputs.

Bars: index work (candidate lists; kept sets given identical Gram values) bit-exact; Gram and dot
products within 1e-4 relative + a small absolute floor; beta within 1e-4 relative + 1e-6;
objective trajectory within 1e-5 relative.  A candidate pair whose |x_a^T x_b| lies within the Gram
tolerance of rho may be decided differently by the two sides; the GPU's kept set must then be the
greedy result on its own Gram values AND every decision of its walk must follow from the oracle's
Gram with only such pairs decided the other way (tests/parity_rules.py); the pairs are logged.
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


def _pair(p, keep_gram=True, **kw):
    """(GPU solver, oracle) on the same arrays."""
    pk = _gpu()
    dev = torch.device("cuda:0")
    args = dict(lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
    if getattr(p, "loss", "squared") != "squared":
        args["loss"] = p.loss
    args.update(kw)
    if p.layout == "dense":
        xg = p.x.to(dev)
        g = pk.StradsLasso(x=xg, y=p.y.to(dev), keep_gram=keep_gram, **args)
        o = OracleLasso(x=p.x.cpu().numpy(), y=p.y.cpu().numpy(), **args)
    elif p.layout == "geno2":
        # packed 2-bit design on the GPU; the oracle gets the fp32 matrix the codes stand for
        g = pk.StradsLasso(codes=p.codes.to(dev), col_mean=p.col_mean.to(dev), col_scale=p.col_scale.to(dev),
                           n=p.n, y=p.y.to(dev), keep_gram=keep_gram, **args)
        o = OracleLasso(x=p.x.cpu().numpy(), y=p.y.cpu().numpy(), **args)
    else:
        g = pk.StradsLasso(values=p.values.to(dev), row_idx=p.row_idx.to(dev), col_ptr=p.col_ptr.to(dev), n=p.n,
                           y=p.y.to(dev), keep_gram=keep_gram, **args)
        o = OracleLasso(values=p.values.cpu().numpy(), row_idx=p.row_idx.cpu().numpy(),
                        col_ptr=p.col_ptr.cpu().numpy(), n=p.n, y=p.y.cpu().numpy(), **args)
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


def _check_round(g, o, log, teacher_forced):
    """One round on both sides, every stage compared.  The oracle follows the GPU's index
    decisions once they have been shown admissible."""
    if teacher_forced:
        g.set_state(o.beta, o.dbeta, o.r, o.t)
    # r0: the vector the round's dot products are taken with (the residual; the weights under the logistic loss)
    beta0, dbeta0, r0, t0 = o.beta.copy(), o.dbeta.copy(), o.dots_vector().copy(), o.t
    gb0, gd0 = (beta0, dbeta0) if teacher_forced else [_np(a) for a in g.get_state()[:2]]
    g.round()
    lr = g.last_round(want_gram=not o.no_deps)
    cand, kept_pos = _np(lr["cand"]), _np(lr["kept_pos"])
    # Step 1: candidate list, set and order, bit-exact (from the oracle's own delta-beta in
    # teacher-forced mode; from the GPU's delta-beta otherwise, which the oracle has followed)
    ref_cand = _ref_candidates(o, dbeta0, t0)
    if not np.array_equal(cand, ref_cand):
        # admissible only if delta-beta differs in the last bits between the two sides
        assert not teacher_forced, "candidate list differs on identical delta-beta"
        log.append(("cand_fork", t0))
        return False
    L = len(cand)
    if o.no_deps:
        # no dependency check: B_1 is the head of the draw
        k = min(L, o.p_max) if o.p_max > 0 else L
        assert np.array_equal(kept_pos, np.arange(k, dtype=np.int32))
        return _finish_round(g, o, lr, cand, kept_pos, r0, t0, gb0, gd0)
    # Step 2a: Gram values
    if o.csc:
        Gref = orc.gram_csc(o.x, o.row_idx, o.col_ptr, cand)
    else:
        Gref = orc.gram_dense(o.x, cand)
    Ggpu = _np(lr["G"])
    _assert_close(Ggpu, Gref, GRAM_RTOL, GRAM_ATOL, f"gram (round {t0})")
    # Step 2b: the GPU's kept set is the greedy result on the GPU's own Gram values, bit-exact
    kept_from_gpu_gram = orc.greedy_filter(Ggpu, o.rho, o.p_max)
    assert np.array_equal(kept_pos, kept_from_gpu_gram), f"filter differs on identical Gram (round {t0})"
    # and it is the oracle's kept set, or differs from it only through pairs within the Gram tolerance of rho
    kept_ref = orc.greedy_filter(Gref, o.rho, o.p_max)
    check_kept_against_oracle(Gref, kept_pos, kept_ref, o.rho, o.p_max, log, f"round {t0}", G_gpu=Ggpu)
    return _finish_round(g, o, lr, cand, kept_pos, r0, t0, gb0, gd0)


def _finish_round(g, o, lr, cand, kept_pos, r0, t0, gb0, gd0):
    # Steps 3-4 with the oracle following the GPU's (admissible) decisions
    out = o.round(forced_cand=cand, forced_kept_pos=kept_pos)
    rn = float(np.linalg.norm(r0.astype(np.float64)))
    _assert_close(_np(lr["z"]), out["z"], DOT_RTOL, 1e-6 * max(rn, 1.0), f"dots (round {t0})")
    _assert_close(_np(lr["delta"]), out["delta"], BETA_RTOL, 2e-6 * max(rn, 1.0), f"delta (round {t0})")
    beta, dbeta, r, t = g.get_state()
    assert t == o.t
    _assert_close(_np(beta), o.beta, BETA_RTOL, 2e-6 * max(rn, 1.0), f"beta (round {t0})")
    _assert_close(_np(r), o.r, DOT_RTOL, 2e-6 * max(rn, 1.0), f"residual (round {t0})")
    # coordinates outside the kept set are untouched, bit for bit
    untouched = np.ones(o.J, bool)
    untouched[out["kept"]] = False
    assert np.array_equal(_np(beta)[untouched], gb0[untouched])
    assert np.array_equal(_np(dbeta)[untouched], gd0[untouched])
    return True


# ---------------------------------------------------------------------------------------------
# Step 1: keys and candidate lists
# ---------------------------------------------------------------------------------------------
def test_sampling_keys_are_bit_identical():
    p = si.make("c1_dense_iid", n=64, j=70001, nnz=5, l_prime=100)
    g, o = _pair(p, keep_gram=False)
    rng = np.random.default_rng(0)
    db = np.abs(rng.normal(size=p.j)).astype(np.float32)
    db[::7] = 1e6
    db[1::7] = 0.0
    db[2::7] = 1e-20
    db[3::7] = np.float32(3.4e18)
    for t in (0, 1, 12345678901):
        g.set_state(None, db, None, t)
        got = _np(g.stage_keys(t))
        ref = orc.priority_keys(db, p.eta, p.seed, t)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("j,l_prime", [(1, 1), (5, 5), (63, 7), (257, 256), (1000, 1000), (5000, 200),
                                       (70001, 1000), (300000, 8192), (300000, 1)])
def test_candidate_lists_are_bit_identical(j, l_prime):
    p = si.make("c1_dense_iid", n=8, j=j, nnz=1, l_prime=l_prime)
    g, o = _pair(p, keep_gram=False)
    rng = np.random.default_rng(j)
    for t, mode in enumerate(["init", "mixed", "equal", "few_large"]):
        if mode == "init":
            db = np.full(j, 1e6, np.float32)
        elif mode == "mixed":
            db = np.abs(rng.normal(size=j)).astype(np.float32)
            db[rng.random(j) < 0.3] = 1e6
            db[rng.random(j) < 0.3] = 0.0
        elif mode == "equal":
            db = np.zeros(j, np.float32)               # all weights = eta: many exactly equal keys
        else:
            db = np.zeros(j, np.float32)
            db[rng.integers(0, j, max(1, l_prime // 3))] = 0.5
        g.set_state(None, db, None, t)
        g.round()
        cand = _np(g.last_round()["cand"])
        ref = orc.draw(orc.priority_keys(db, p.eta, p.seed, t), l_prime)
        assert np.array_equal(cand, ref), (mode, j, l_prime)


def test_selection_fallback_path_gives_the_same_list():
    # force the multi-pass boundary selection by shrinking the list length it is meant for
    p = si.make("c1_dense_iid", n=8, j=200000, nnz=1, l_prime=3000)
    g, o = _pair(p, keep_gram=False)
    db = np.zeros(p.j, np.float32)
    for cap in (1, 7, 64):
        g.set_tuning("select_cap", cap)
        g.set_state(None, db, None, 3)
        g.round()
        cand = _np(g.last_round()["cand"])
        ref = orc.draw(orc.priority_keys(db, p.eta, p.seed, 3), p.l_prime)
        assert np.array_equal(cand, ref), cap


# ---------------------------------------------------------------------------------------------
# Step 2: Gram and filter
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,j,l_prime", [(1000, 600, 200), (1001, 300, 130), (37, 400, 257), (4096, 300, 128),
                                         (10, 200, 64), (3, 50, 50)])
def test_gram_matches_oracle_across_shapes(n, j, l_prime):
    p = si.make("c2_dense_block_corr", n=n, j=j, nnz=5, l_prime=l_prime)
    g, o = _pair(p)
    g.round()
    lr = g.last_round(want_gram=True)
    cand = _np(lr["cand"])
    Gref = orc.gram_dense(o.x, cand)
    _assert_close(_np(lr["G"]), Gref, DOT_RTOL, 1e-6, "gram")
    assert np.array_equal(_np(lr["G"]), _np(lr["G"]).T)


def test_gram_split_k_variants_agree_with_oracle():
    p = si.make("c2_dense_block_corr", n=5000, j=600, nnz=5, l_prime=300)
    for split in (1, 2, 5, 0):
        g, o = _pair(p)
        g.set_tuning("gram_split_k", split)
        g.round()
        lr = g.last_round(want_gram=True)
        Gref = orc.gram_dense(o.x, _np(lr["cand"]))
        _assert_close(_np(lr["G"]), Gref, DOT_RTOL, 1e-6, f"gram split {split}")


@pytest.mark.parametrize("n,j,l_prime", [(1000, 900, 700), (5000, 700, 513), (1004, 600, 300), (4096, 300, 128),
                                         (260, 1200, 1100), (8, 600, 511), (996, 800, 512), (2052, 900, 768)])
def test_gram_in_256_wide_tiles_matches_oracle(n, j, l_prime):
    """The tile kernel for long lists (256 x 256 tiles, stage ranges of tiles handed out from a queue), forced
    onto short lists: whole Gram against the oracle, including a last tile column of 128 columns, a ragged
    last K stage, a single diagonal tile and one-stage items."""
    p = si.make("c2_dense_block_corr", n=n, j=j, nnz=5, l_prime=l_prime)
    g, o = _pair(p)
    assert g.gram_tile_edge() == (64 if (n, l_prime) == (260, 1100) else 128)   # (1100 candidates over 260 rows: 64-wide)
    g.set_tuning("gram_tile256", 2)
    assert g.gram_tile_edge() == 256
    for _ in range(2):                                  # twice: stale tile slots must not leak into a round
        g.round()
        lr = g.last_round(want_gram=True)
        cand = _np(lr["cand"])
        Gref = orc.gram_dense(o.x, cand)
        _assert_close(_np(lr["G"]), Gref, DOT_RTOL, 1e-6, "gram")
        assert np.array_equal(_np(lr["G"]), _np(lr["G"]).T)
        kept = _np(lr["kept_pos"])
        assert np.array_equal(kept, orc.greedy_filter(_np(lr["G"]), o.rho, o.p_max))


@pytest.mark.parametrize("n,j,l_prime,forced", [(500, 2300, 2000, False), (1000, 1700, 1600, False),
                                                (1000, 900, 700, True), (1001, 500, 300, True), (37, 300, 260, True),
                                                (3, 200, 130, True), (64, 90, 64, True), (8, 3, 2, True)])
def test_gram_in_64_wide_tiles_matches_oracle(n, j, l_prime, forced):
    """A long list over short columns is multiplied in 64 x 64 tiles that run over all rows and write the conflict
    bits themselves (no K-slices, no slot sum).  Whole Gram against the oracle and the kept set against the greedy
    walk on it: the shapes that take the route by default, and the route forced onto short lists (unaligned
    columns, a single ragged K stage, one tile)."""
    p = si.make("c2_dense_block_corr", n=n, j=j, nnz=5, l_prime=l_prime)
    g, o = _pair(p)
    if forced:
        assert g.gram_tile_edge() == 128
        g.set_tuning("gram_direct", 2)
    assert g.gram_tile_edge() == 64
    for _ in range(2):
        g.round()
        lr = g.last_round(want_gram=True)
        cand, G = _np(lr["cand"]), _np(lr["G"])
        _assert_close(G, orc.gram_dense(o.x, cand), DOT_RTOL, 1e-6, "gram")
        assert np.array_equal(G, G.T)
        assert np.array_equal(_np(lr["kept_pos"]), orc.greedy_filter(G, o.rho, o.p_max))
    h, o2 = _pair(p)                                   # and whole rounds against the oracle, stage by stage
    if forced:
        h.set_tuning("gram_direct", 2)
    log = []
    for _ in range(3):
        assert _check_round(h, o2, log, teacher_forced=True)
    g.set_tuning("gram_direct", 0)
    assert g.gram_tile_edge() == 128


@pytest.mark.parametrize("n,j,l_prime", [(4096, 4500, 4300), (4096, 8192, 8192), (45056, 2100, 2048)])
def test_gram_of_a_long_list_takes_the_256_wide_route_and_matches_oracle_rows(n, j, l_prime):
    """A list longer than 4096 over columns of at least 4096 rows takes the 256-wide tiles by default, and so does
    a shorter list over columns long enough (2048 candidates over 45056 rows): sampled rows of the Gram against
    the oracle, the rest against the 128-wide kernel's result on the same candidates.
    (8192 is the longest list the library takes: every column is a candidate, 32 x 32 tiles, nothing padded.)"""
    p = si.make("c5_dense_duplicates", n=n, j=j, nnz=20, l_prime=l_prime)
    g, o = _pair(p)
    assert g.gram_tile_edge() == 256
    g.round()
    lr = g.last_round(want_gram=True)
    cand, G = _np(lr["cand"]), _np(lr["G"])
    rows = np.unique(np.concatenate([np.minimum([0, 127, 128, 255, 256, 4095, 4096, 4223, l_prime - 1], l_prime - 1),
                                     np.random.default_rng(5).integers(0, l_prime, 24)])).astype(np.int32)
    ref = orc.gram_rows_dense(o.x, cand, rows)
    _assert_close(G[rows], ref, DOT_RTOL, 1e-6, "gram rows")
    assert np.array_equal(G, G.T)
    g2, _ = _pair(p)
    g2.set_tuning("gram_tile256", 0)
    assert g2.gram_tile_edge() == 128
    g2.round()
    lr2 = g2.last_round(want_gram=True)
    assert np.array_equal(_np(lr2["cand"]), cand)
    _assert_close(_np(lr2["G"]), G, 2e-5, 2e-6, "128-wide against 256-wide tiles")
    assert np.array_equal(_np(lr2["kept_pos"]), orc.greedy_filter(_np(lr2["G"]), o.rho, o.p_max))
    assert np.array_equal(_np(lr["kept_pos"]), orc.greedy_filter(G, o.rho, o.p_max))


def test_rounds_with_256_wide_tiles_repeat_bit_for_bit():
    """Which workgroup takes which item of the tile queue differs from launch to launch; the results must not.
    Two handles run the same 25 rounds with the 256-wide tiles (forced onto a list of 1500, so that the queue has
    several items per tile): every round's Gram and the final state are bit-identical, and the objective
    follows the 128-wide kernel's within the parity tolerance."""
    p = si.make("c5_dense_duplicates", n=6000, j=4000, nnz=20, l_prime=1500)
    (a, _), (b, _), (c, _) = _pair(p), _pair(p), _pair(p)
    a.set_tuning("gram_tile256", 2)
    b.set_tuning("gram_tile256", 2)
    assert a.gram_tile_edge() == b.gram_tile_edge() == 256 and c.gram_tile_edge() == 128
    for t in range(25):
        a.round(); b.round(); c.round()
        if t % 6 == 0:
            ga, gb = a.last_round(want_gram=True), b.last_round(want_gram=True)
            assert torch.equal(ga["cand"], gb["cand"]) and torch.equal(ga["G"], gb["G"]), t
            assert torch.equal(ga["kept_pos"], gb["kept_pos"])
    for u, v in zip(a.get_state()[:3], b.get_state()[:3]):
        assert torch.equal(u, v)
    assert a.objective() == b.objective()
    assert a.objective() == pytest.approx(c.objective(), rel=1e-4)


@pytest.mark.parametrize("j,l_prime,p_max", [(3000, 2500, 0), (6000, 5000, 0), (6000, 5000, 1800), (8192, 8192, 0)])
def test_greedy_walk_after_256_wide_tiles_with_many_conflicts(j, l_prime, p_max):
    """With the 256-wide tiles the mask kernel marks the chunks of 64 candidates whose rows the greedy walk has
    to read, and the walk skips the others.  Block-correlated columns put conflicts in most chunks (the
    near-duplicate designs of the other tests in few): the kept set is the oracle's greedy walk on the same
    Gram, in three rounds in a row (the marks of one round must not leak into the next, nor be missed)."""
    p = si.make("c2_dense_block_corr", n=260, j=j, nnz=5, l_prime=l_prime)
    g, o = _pair(p, p_max=p_max)
    g.set_tuning("gram_tile256", 2)
    assert g.gram_tile_edge() == 256
    rejected = 0
    for _ in range(3):
        g.round()
        lr = g.last_round(want_gram=True)
        G, kept = _np(lr["G"]), _np(lr["kept_pos"])
        assert np.array_equal(kept, orc.greedy_filter(G, o.rho, o.p_max))
        rejected += l_prime - len(kept)
    assert rejected > 0


@pytest.mark.parametrize("L", [1, 2, 63, 64, 65, 200, 1000, 2500, 4100, 8192])
def test_filter_is_bit_exact_on_given_gram(L):
    p = si.make("c1_dense_iid", n=8, j=max(L, 2), nnz=1, l_prime=L)
    rng = np.random.default_rng(L)
    for p_max, scale in ((0, 0.035), (0, 0.08), (max(1, L // 3), 0.035), (0, 0.02)):
        g, o = _pair(p, keep_gram=False, p_max=p_max)
        A = (rng.standard_normal((L, L)) * scale).astype(np.float32)
        G = np.triu(A, 1) + np.triu(A, 1).T + np.eye(L, dtype=np.float32)
        if L > 3:
            G[0, 2] = G[2, 0] = np.float32(p.rho)                               # exactly rho: conflict
            G[0, 3] = G[3, 0] = np.nextafter(np.float32(p.rho), np.float32(0))   # just below: admissible
        got = _np(g.stage_filter(torch.from_numpy(G)))
        ref = orc.greedy_filter(G, p.rho, p_max)
        assert np.array_equal(got, ref), (L, p_max, scale)
        assert 1 <= len(ref) <= L


# ---------------------------------------------------------------------------------------------
# whole rounds
# ---------------------------------------------------------------------------------------------
def test_config1_teacher_forced_rounds():
    p = si.make("c1_dense_iid")                      # the full first configuration: 1000 x 5000, L'=200
    g, o = _pair(p)
    log = []
    for _ in range(p.rounds):
        assert _check_round(g, o, log, teacher_forced=True)
        assert g.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)
    print("logged:", log)


def test_config1_free_run_objective_trajectory():
    p = si.make("c1_dense_iid")
    g, o = _pair(p)
    log = []
    f_prev = g.objective()
    assert f_prev == pytest.approx(o.objective(), rel=OBJ_RTOL)
    for t in range(p.rounds):
        ok = _check_round(g, o, log, teacher_forced=False)
        if not ok:                                   # admissible fork of the draw: re-synchronise and go on
            o.set_state(*[_np(a) if isinstance(a, torch.Tensor) else a for a in g.get_state()])
        assert g.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)
    v_gpu, v_ref = g.kkt(), o.kkt()
    assert v_gpu == pytest.approx(v_ref, rel=1e-3, abs=1e-6)
    print("logged:", log)


@pytest.mark.parametrize("config,kw,rounds", [
    ("c2_dense_block_corr", dict(n=2000, j=6000, nnz=40, l_prime=500), 8),
    ("c3_genotype", dict(n=500, j=20000, nnz=20, l_prime=700), 6),
    ("c5_dense_duplicates", dict(n=3000, j=5000, nnz=30, l_prime=400), 8),
    ("c1_dense_iid", dict(n=1003, j=900, nnz=10, l_prime=150), 6),        # N not a multiple of 4
    # long columns, a list between 1024 and 4096: x_j^T r two columns per workgroup (ragged: odd kept counts occur),
    # the residual update in one kernel with 256 rows per workgroup and a ragged last workgroup
    ("c5_dense_duplicates", dict(n=33004, j=2600, nnz=30, l_prime=1300, lam_frac=0.01), 3),
])
def test_reduced_configs_teacher_forced(config, kw, rounds):
    p = si.make(config, **kw)
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


@pytest.mark.parametrize("ride,fused", [(1, 1), (0, 0), (1, 0), (0, 1)])
@pytest.mark.parametrize("kw", [
    dict(n=2000, j=6000, nnz=40, l_prime=500),
    dict(n=1003, j=3000, nnz=40, l_prime=1024, lam_frac=0.001, rho=0.9),     # nearly every candidate is kept and moves
    dict(n=61, j=500, nnz=5, l_prime=90, lam_frac=0.001),                    # fewer rows than one workgroup owns
    dict(n=403, j=9000, nnz=40, l_prime=2500, lam_frac=0.001, rho=0.9),      # more than 1024 movers: the kept list is compacted in pieces
])
def test_short_list_route_and_general_route(kw, ride, fused):
    # lists of at most 4096 candidates: x_j^T r rides along with the Gram launch and the filter commits B_1
    # unless "dots_with_gram" is 0; the residual is updated in one kernel unless "residual_fused" is 0
    p = si.make("c2_dense_block_corr", **kw)
    g, o = _pair(p)
    g.set_tuning("dots_with_gram", ride)
    g.set_tuning("residual_fused", fused)
    log = []
    for _ in range(5):
        assert _check_round(g, o, log, teacher_forced=True)
    assert g.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)
    # the round summary comes from the same kernel(s)
    g.set_state(o.beta, o.dbeta, o.r, o.t)
    info = g.round(want_info=True)
    delta = _np(g.last_round(want_gram=False)["delta"])
    assert info.n_moved == int(np.count_nonzero(delta))
    assert info.max_abs_delta == np.float32(np.abs(delta).max(initial=0.0))
    assert info.n_kept == len(_np(g.last_round(want_gram=False)["kept"]))
    if kw["l_prime"] == 2500:
        assert info.n_moved > 1024
    if kw["l_prime"] == 1024:
        assert info.n_moved > 200          # every wavefront of the one-kernel update has several columns


@pytest.mark.parametrize("loss", ["squared", "logistic"])
def test_products_taken_with_the_gram_are_the_same_bits(loss):
    # "dots_with_gram" moves the pass over the candidates' columns, not its arithmetic
    p = si.make("c2_dense_block_corr", n=3000, j=5000, nnz=40, l_prime=600, lam_frac=0.01)
    if loss == "logistic":
        p = si.with_labels(p)
    a, _ = _pair(p, keep_gram=False)
    b, _ = _pair(p, keep_gram=False)
    b.set_tuning("dots_with_gram", 0)
    for _ in range(6):
        ia, ib = a.round(want_info=True), b.round(want_info=True)
        assert (ia.n_kept, ia.n_moved, ia.max_abs_delta) == (ib.n_kept, ib.n_moved, ib.max_abs_delta)
        la, lb = a.last_round(want_gram=False), b.last_round(want_gram=False)
        for k in ("kept", "kept_pos", "z", "delta"):
            assert torch.equal(la[k], lb[k]), k
    assert ia.n_moved > 0
    for u, v in zip(a.get_state()[:3], b.get_state()[:3]):
        assert torch.equal(u, v)


@pytest.mark.parametrize("kw,rounds", [
    (dict(n=3000, j=20000, nnz_per_col=30, nnz=20, l_prime=600, rho=0.05), 8),
    (dict(n=257, j=900, nnz_per_col=12, nnz=8, l_prime=130, rho=0.2), 10),
    (dict(n=64, j=300, nnz_per_col=64, nnz=5, l_prime=300, rho=0.3), 5),      # every column is dense: heavy buckets
])
def test_csc_design_teacher_forced(kw, rounds):
    p = si.make("c4_sparse_csc", **kw)
    g, o = _pair(p)
    log = []
    for _ in range(rounds):
        assert _check_round(g, o, log, teacher_forced=True)
    assert g.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)
    v, gg = g.kkt(want_g=True)
    v_ref, g_ref = o.kkt(want_g=True)
    rn = float(np.linalg.norm(o.r.astype(np.float64)))
    _assert_close(_np(gg), g_ref, DOT_RTOL, 1e-6 * max(rn, 1.0), "x_j^T r for all columns (CSC)")
    assert v == pytest.approx(v_ref, rel=1e-3, abs=1e-6 * max(rn, 1.0))
    print("logged:", log)


def test_csc_free_run_is_deterministic_and_tracks_oracle():
    p = si.make("c4_sparse_csc", n=2000, j=6000, nnz_per_col=20, nnz=15, l_prime=256, rho=0.1)
    a, o = _pair(p, keep_gram=False)
    b, _ = _pair(p, keep_gram=False)
    a.run(12)
    b.run(12)
    for u, v in zip(a.get_state()[:3], b.get_state()[:3]):
        assert torch.equal(u, v)
    c, o = _pair(p, keep_gram=True)
    log = []
    for _ in range(12):
        if not _check_round(c, o, log, teacher_forced=False):
            o.set_state(*[_np(x) if isinstance(x, torch.Tensor) else x for x in c.get_state()])
        assert c.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)


def test_csc_create_checks_column_bound():
    pk = _gpu()
    p = si.make("c4_sparse_csc", n=500, j=400, nnz_per_col=10, nnz=5, l_prime=50)
    dev = torch.device("cuda:0")
    kw = dict(values=p.values.to(dev), row_idx=p.row_idx.to(dev), col_ptr=p.col_ptr.to(dev), n=p.n, y=p.y.to(dev),
              lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime)
    pk.StradsLasso(max_col_nnz=10, **kw).close()
    with pytest.raises(pk.StradsError) as e:
        pk.StradsLasso(max_col_nnz=9, **kw)
    assert e.value.code == -1


@pytest.mark.parametrize("n", [2052, 5000, 10000, 16000, 16384, 16388, 2050])
def test_kkt_pass_matches_oracle_across_row_counts(n):
    # covers the register-resident streaming kernel (4/8/12/16 float4 of r per thread), its
    # ragged last slice, and the fallbacks (N not a multiple of 4, N above the register budget)
    p = si.make("c1_dense_iid", n=n, j=301, nnz=10, l_prime=64)
    g, o = _pair(p, keep_gram=False)
    for _ in range(3):
        g.round()
    o.set_state(*[_np(x) if isinstance(x, torch.Tensor) else x for x in g.get_state()])
    v, gg = g.kkt(want_g=True)
    v_ref, g_ref = o.kkt(want_g=True)
    rn = float(np.linalg.norm(o.r.astype(np.float64)))
    _assert_close(_np(gg), g_ref, DOT_RTOL, 1e-6 * max(rn, 1.0), "x_j^T r")
    assert v == pytest.approx(v_ref, rel=1e-4, abs=1e-6 * max(rn, 1.0))


def test_run_matches_repeated_rounds_and_is_deterministic():
    p = si.make("c1_dense_iid", n=800, j=2000, nnz=20, l_prime=128)
    a, _ = _pair(p, keep_gram=False)
    b, _ = _pair(p, keep_gram=False)
    info = a.run(15)
    kept = 0
    for _ in range(15):
        kept += b.round(want_info=True).n_kept
    assert info.rounds_done == 15 and info.updates_done == kept
    sa, sb = a.get_state(), b.get_state()
    for u, v in zip(sa[:3], sb[:3]):
        assert torch.equal(u, v)                      # bit-identical: no order-dependent arithmetic
    assert info.objective == b.objective()
    # save / restore: 15 rounds == 10 + restore + 5
    c, _ = _pair(p, keep_gram=False)
    c.run(10)
    st = c.get_state()
    d, _ = _pair(p, keep_gram=False)
    d.set_state(*st)
    d.run(5)
    for u, v in zip(d.get_state()[:3], sa[:3]):
        assert torch.equal(u, v)


def test_run_stops_on_kkt_and_solution_is_optimal():
    p = si.make("c1_dense_iid", n=300, j=400, nnz=8, l_prime=64)
    g, o = _pair(p, keep_gram=False)
    info = g.run(20000, kkt_tol=1e-4, check_every=50)
    assert info.converged == 1 and info.rounds_done < 20000
    assert info.kkt_violation <= 1e-4 * p.lam
    beta = _np(g.get_state()[0])
    # the oracle, run to the same tolerance, reaches the same minimiser
    for _ in range(info.rounds_done):
        o.round()
    assert o.kkt() <= 2e-4 * p.lam
    _assert_close(beta, o.beta, 1e-3, 1e-4, "converged beta")


def test_degenerate_cases():
    # lambda above max |X^T y|: nothing ever moves
    p = si.make("c1_dense_iid", n=200, j=300, nnz=5, l_prime=300)
    g, o = _pair(p, keep_gram=False, lam=float(p.lam) * 11.0)
    for _ in range(3):
        info = g.round(want_info=True)
        assert info.n_moved == 0 and info.max_abs_delta == 0.0 and info.n_cand == 300
    beta, dbeta, r, t = g.get_state()
    assert not beta.any() and torch.equal(r.cpu(), p.y) and t == 3
    # l_prime above J is clamped; p_max = 1 is sequential coordinate descent
    p = si.make("c1_dense_iid", n=100, j=40, nnz=4, l_prime=40)
    g, o = _pair(p, keep_gram=True, l_prime=4000, p_max=1)
    f = g.objective()
    log = []
    for _ in range(30):
        assert _check_round(g, o, log, teacher_forced=True)
        assert len(g.last_round()["kept"]) == 1
        f2 = g.objective()
        assert f2 <= f * (1 + 1e-6)
        f = f2


def test_pass_over_all_columns_is_timed_only_while_profiling():
    p = si.make("c1_dense_iid", n=500, j=2000, nnz=5, l_prime=64)
    g, _ = _pair(p, keep_gram=False)
    v0 = g.kkt()
    assert g.last_kkt_ms() == 0.0
    g.set_tuning("profile_level", 1)
    v1 = g.kkt()
    ms = g.last_kkt_ms()
    assert v1 == v0 and 0.0 < ms < 50.0
    g.set_tuning("profile_level", 0)
    g.kkt()
    assert g.last_kkt_ms() == 0.0


def test_gram_job_numbering_does_not_change_results():
    # "gram_xcd_map": which workgroup takes which (tile, K-slice) job; also after a change of the slice count
    p = si.make("c2_dense_block_corr", n=3000, j=4000, nnz=30, l_prime=700)
    a, _ = _pair(p, keep_gram=True)
    b, _ = _pair(p, keep_gram=True)
    b.set_tuning("gram_xcd_map", 0)
    for k in (0, 3):
        if k:
            a.set_tuning("gram_split_k", k)
            b.set_tuning("gram_split_k", k)
        for _ in range(3):
            a.round()
            b.round()
            la, lb = a.last_round(want_gram=True), b.last_round(want_gram=True)
            assert torch.equal(la["G"], lb["G"]) and torch.equal(la["kept"], lb["kept"])
    for u, v in zip(a.get_state()[:3], b.get_state()[:3]):
        assert torch.equal(u, v)
