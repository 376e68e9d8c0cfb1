"""GPU parity at the configurations' full sizes, in the launch configuration bench.py times
(no debug Gram, automatic K-slices).  The oracle cannot hold or sweep these designs whole, so it is
run on what a round actually touches: the candidate columns are gathered to the host and the oracle's
own stage functions (oracle/strads_oracle.c through oracle/oracle.py: draw, Gram, greedy filter, dot
products, eq. (2) update, residual update, objective) are applied to that sub-matrix; candidate lists
come from the full delta-beta vector.  Nothing of the method is computed in this file.

Checked per round: candidate list bit-exact; kept set equal to the oracle's, or admissible through
pairs within the Gram tolerance of rho (tests/parity_rules.py; every such pair is logged); dots,
changes, all of beta and delta-beta, the whole residual within the stated tolerances; objective
within 1e-5.  Where the candidate set is too large for a whole oracle Gram (L' = 8000), complete
rows of it are computed for every position the GPU rejected, for planted near-duplicate pairs and for
a random sample, each such row is compared entry by entry with the GPU's Gram (a second handle that
keeps it), and the GPU's keep/reject decision for that position is checked against the oracle's row.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from parity_rules import GRAM_ATOL, GRAM_RTOL, check_kept_against_oracle, explain_row, rho_window
from synth import lasso_inputs as si

pytestmark = pytest.mark.gpu


def _np(t):
    return t.detach().cpu().numpy()


def _close(got, ref, rtol, atol, what):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    err = np.abs(got - ref) - (rtol * np.abs(ref) + atol)
    assert err.size == 0 or err.max() <= 0, f"{what}: worst excess {err.max():.3e} at {err.argmax()}"


def _ref_candidates(p, dbeta0, t, l_prime, n_shards):
    keys = orc.priority_keys(dbeta0, p.eta, p.seed, t)
    if n_shards == 1:
        return orc.draw(keys, l_prime)
    full = orc.draw(keys, p.j)                          # the full draw order restricted to shard t mod S
    return full[full % n_shards == t % n_shards][:l_prime]


def _check_updates(p, g, lr, xs, cand, kept_pos, beta0, dbeta0, r0, t, logistic):
    """eq. (2), Step 4, the residual update and the objective: the oracle's stage functions on the
    gathered candidate columns xs (row a = column cand[a]) and on host copies of the state."""
    step = 4.0 if logistic else 1.0                     # 1 / curvature of the coordinate step
    kept = cand[kept_pos]
    y = _np(p.y)
    v0 = orc.logistic_weights(y, r0) if logistic else r0            # what the dot products are taken with
    rn = max(float(np.linalg.norm(v0.astype(np.float64))), 1.0)
    z_ref = orc.dots_dense(xs, kept_pos, v0)
    _close(_np(lr["z"]), z_ref, 1e-4, 1e-6 * rn, f"dots (round {t})")
    beta_ref, dbeta_ref, r_ref = beta0.copy(), dbeta0.copy(), r0.copy()
    d_ref = orc.update(kept, z_ref, p.lam, beta_ref, dbeta_ref, inv_kappa=step)
    _close(_np(lr["delta"]), d_ref, 1e-4, 2e-6 * step * rn, f"delta (round {t})")
    orc.residual_dense(xs, kept_pos, d_ref, r_ref)
    beta1, dbeta1, r1, _ = g.get_state()
    _close(_np(beta1), beta_ref, 1e-4, 2e-6 * step * rn, f"beta (round {t})")
    _close(_np(dbeta1), dbeta_ref, 1e-4, 2e-6 * step * rn, f"dbeta (round {t})")
    _close(_np(r1), r_ref, 1e-4, 2e-6 * step * rn, f"residual (round {t})")
    # nothing outside the kept set moved, bit for bit
    untouched = np.ones(p.j, bool)
    untouched[kept] = False
    assert np.array_equal(_np(beta1)[untouched], beta0[untouched])
    assert np.array_equal(_np(dbeta1)[untouched], dbeta0[untouched])
    f_ref = orc.objective_logistic(y, r_ref, beta_ref, p.lam) if logistic else orc.objective(r_ref, beta_ref, p.lam)
    assert g.objective() == pytest.approx(f_ref, rel=1e-5)


def _rounds_dense(p, rounds, n_shards=1):
    """Candidate sets small enough for a whole oracle Gram (L' <= 2000)."""
    import paper_1312_5766_amd as pk
    logistic = getattr(p, "loss", "squared") == "logistic"
    l_prime = min(p.l_prime, p.j // n_shards)
    g = pk.StradsLasso(x=p.x, y=p.y, lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed,
                       n_shards=n_shards, loss="logistic" if logistic else "squared")
    logged = []
    for t in range(rounds):
        beta0, dbeta0, r0, t0 = [_np(a) if isinstance(a, torch.Tensor) else a for a in g.get_state()]
        assert t0 == t
        g.round()
        lr = g.last_round()
        cand, kept_pos = _np(lr["cand"]), _np(lr["kept_pos"])
        assert np.array_equal(cand, _ref_candidates(p, dbeta0, t, l_prime, n_shards)), f"candidate list differs in round {t}"
        xs = _np(p.x[torch.from_numpy(cand.astype(np.int64)).to(p.x.device)])         # (L, N) gathered columns
        local = np.arange(len(cand), dtype=np.int32)
        Gref = orc.gram_dense(xs, local)
        kept_ref = orc.greedy_filter(Gref, p.rho, 0)
        check_kept_against_oracle(Gref, kept_pos, kept_ref, p.rho, 0, logged, f"round {t}")
        _check_updates(p, g, lr, xs, cand, kept_pos, beta0, dbeta0, r0, t, logistic)
    g.close()
    return logged


def _rounds_dense_large(p, rounds, n_plant=8, n_random_rows=48, seed=0):
    """L' = 8000: the timed launch configuration on one handle, a second handle that keeps the Gram for
    the entry-by-entry comparison; oracle Gram rows instead of the whole oracle Gram."""
    import paper_1312_5766_amd as pk
    dev = p.x.device
    kw = dict(x=p.x, y=p.y, lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
    g = pk.StradsLasso(**kw)
    gk = pk.StradsLasso(keep_gram=True, **kw)
    rng = np.random.default_rng(seed)
    window = rho_window(p.rho)
    logged = []
    # near-duplicate pairs (correlation 0.9) to plant among the candidates: a huge delta-beta puts both
    # columns of a pair at the head of the draw, so entries with |g| ~ 0.9 are present in every round
    dups = torch.nonzero(p.dup_src >= 0).flatten()
    pick = dups[torch.from_numpy(rng.permutation(dups.numel())[:n_plant]).to(dev)]
    planted = torch.cat([pick, p.dup_src[pick]]).unique()
    for t in range(rounds):
        beta0_d, dbeta0_d, r0_d, t0 = g.get_state()
        assert t0 == t
        dbeta0_d[planted] = 1e15
        g.set_state(None, dbeta0_d, None, t)
        beta0, dbeta0, r0 = _np(beta0_d), _np(dbeta0_d), _np(r0_d)
        gk.set_state(beta0_d, dbeta0_d, r0_d, t)
        g.round()
        gk.round()
        lr, lrk = g.last_round(), gk.last_round(want_gram=True)
        cand, kept_pos = _np(lr["cand"]), _np(lr["kept_pos"])
        L = len(cand)
        assert np.array_equal(cand, orc.draw(orc.priority_keys(dbeta0, p.eta, p.seed, t), p.l_prime)), f"candidate list differs in round {t}"
        assert set(_np(planted).tolist()) <= set(cand[:2 * len(planted)].tolist()), "planted pairs are not at the head of the draw"
        # keeping the Gram changes nothing the round decides
        assert torch.equal(lr["kept_pos"], lrk["kept_pos"]) and torch.equal(lr["cand"], lrk["cand"])
        for a, b in zip(g.get_state()[:3], gk.get_state()[:3]):
            assert torch.equal(a, b)
        Ggpu_d = lrk["G"]
        assert torch.equal(Ggpu_d, Ggpu_d.T)
        assert np.array_equal(kept_pos, orc.greedy_filter(_np(Ggpu_d), p.rho, 0)), f"filter differs on identical Gram ({t})"
        xs = _np(p.x[torch.from_numpy(cand.astype(np.int64)).to(dev)])                # (L, N)
        local = np.arange(L, dtype=np.int32)
        is_kept = np.zeros(L, bool)
        is_kept[kept_pos] = True
        rejected = np.flatnonzero(~is_kept)
        where_planted = np.flatnonzero(np.isin(cand, _np(planted)))
        assert len(rejected) >= n_plant, "each planted pair must cost one rejection"
        rows = np.unique(np.concatenate([rejected[:200], where_planted, rng.integers(0, L, n_random_rows)])).astype(np.int32)
        assert len(rows) >= 64
        Gref_rows = orc.gram_rows_dense(xs, local, rows)                                # oracle, complete rows
        Ggpu_rows = _np(Ggpu_d[torch.from_numpy(rows.astype(np.int64)).to(dev)])
        _close(Ggpu_rows, Gref_rows, GRAM_RTOL, GRAM_ATOL, f"Gram rows (round {t})")
        assert float(np.abs(Gref_rows[np.isin(rows, where_planted)]).max()) > 0.99      # the diagonal is among them
        big = np.abs(Gref_rows) >= 0.5
        big[np.arange(len(rows)), rows] = False
        assert big.sum() >= n_plant, "no near-duplicate entries among the compared rows"
        # the decision the GPU took at each of these positions follows from the oracle's row
        for i, a in enumerate(rows):
            logged += explain_row(int(a), Gref_rows[i], kept_pos[kept_pos < a], p.rho, bool(is_kept[a]), window)
        # every entry the GPU flags as a conflict anywhere in its Gram is one for the oracle too
        flagged = torch.nonzero(torch.triu(Ggpu_d.abs() >= p.rho, diagonal=1))
        fa, fb = _np(flagged[:, 0]).astype(np.int32), _np(flagged[:, 1]).astype(np.int32)
        assert len(fa) >= n_plant
        ref_pairs = orc.gram_pairs_dense(xs, local, fa, fb)
        _close(_np(Ggpu_d[flagged[:, 0], flagged[:, 1]]), ref_pairs, GRAM_RTOL, GRAM_ATOL, f"flagged entries (round {t})")
        assert np.all(np.abs(ref_pairs) >= p.rho - window)
        _check_updates(p, g, lr, xs, cand, kept_pos, beta0, dbeta0, r0, t, False)
    g.close()
    gk.close()
    return logged


def _skip_without_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def test_config2_full_size():
    _skip_without_gpu()
    p = si.make("c2_dense_block_corr", device="cuda:0")          # 10^4 x 10^5, L' = 1000
    assert (p.n, p.j, p.l_prime) == (10000, 100000, 1000)
    print("logged:", _rounds_dense(p, 4))


def test_config2_full_size_with_scheduler_shards_and_with_the_logistic_loss():
    _skip_without_gpu()
    p = si.make("c2_dense_block_corr", device="cuda:0")
    print("logged (4 shards):", _rounds_dense(p, 5, n_shards=4))
    print("logged (logistic):", _rounds_dense(si.with_labels(p), 3))


def test_config3_full_size():
    _skip_without_gpu()
    p = si.make("c3_genotype", device="cuda:0")                  # 500 x 5*10^5, L' = 2000
    assert (p.n, p.j, p.l_prime) == (500, 500000, 2000)
    print("logged:", _rounds_dense(p, 3))


def test_config5_shape_at_maximum_candidate_count():
    _skip_without_gpu()
    # the fifth configuration's row count, duplicate structure and L' = 8000 (the largest supported
    # neighbourhood: 8192-wide tiles, 128-word mask rows, LDS bitonic sort), with J cut from 10^6 to
    # 6*10^4 so that the design (12 GB) is generated in seconds
    p = si.make("c5_dense_duplicates", device="cuda:0", j=60000, nnz=200)
    assert (p.n, p.l_prime) == (50000, 8000)
    print("logged:", _rounds_dense_large(p, 2))


def test_config5_full_size():
    _skip_without_gpu()
    # the whole fifth configuration (the workload bench.py times): 5*10^4 x 10^6 fp32 = 200 GB of X
    # resident in HBM, L' = 8000
    torch.cuda.empty_cache()
    free, _total = torch.cuda.mem_get_info()
    if free < 215 * 10 ** 9:
        pytest.skip(f"needs 215 GB of free HBM, {free / 1e9:.0f} GB available")
    p = si.make("c5_dense_duplicates", device="cuda:0")
    assert (p.n, p.j, p.l_prime) == (50000, 1000000, 8000)
    print("logged:", _rounds_dense_large(p, 2))
    del p
    torch.cuda.empty_cache()


def test_config4_full_size_csc():
    _skip_without_gpu()
    import paper_1312_5766_amd as pk
    p = si.make("c4_sparse_csc", device="cuda:0")                # 10^5 x 10^6, 100 nonzeros per column, L' = 4000
    assert (p.n, p.j, p.l_prime) == (100000, 1000000, 4000)
    g = pk.StradsLasso(values=p.values, row_idx=p.row_idx, col_ptr=p.col_ptr, n=p.n, y=p.y, lam=p.lam, rho=p.rho,
                       eta=p.eta, l_prime=p.l_prime, seed=p.seed, max_col_nnz=100)
    k = 100
    logged = []
    for t in range(3):
        beta0, dbeta0, r0, _ = [_np(a) if isinstance(a, torch.Tensor) else a for a in g.get_state()]
        g.round()
        lr = g.last_round()
        cand, kept_pos = _np(lr["cand"]), _np(lr["kept_pos"])
        ref_cand = orc.draw(orc.priority_keys(dbeta0, p.eta, p.seed, t), p.l_prime)
        assert np.array_equal(cand, ref_cand)
        # gather the candidate columns into a small CSC of their own (column a = candidate position a)
        ci = torch.from_numpy(cand.astype(np.int64)).to(p.values.device)
        idx = (ci[:, None] * k + torch.arange(k, device=ci.device)[None, :]).flatten()
        vals, rows = _np(p.values[idx]), _np(p.row_idx[idx])
        cp = np.arange(len(cand) + 1, dtype=np.int64) * k
        local = np.arange(len(cand), dtype=np.int32)
        Gref = orc.gram_csc(vals, rows, cp, local)
        kept_ref = orc.greedy_filter(Gref, p.rho, 0)
        check_kept_against_oracle(Gref, kept_pos, kept_ref, p.rho, 0, logged, f"round {t}")
        kept = cand[kept_pos]
        rn = max(float(np.linalg.norm(r0.astype(np.float64))), 1.0)
        z_ref = orc.dots_csc(vals, rows, cp, kept_pos, r0)
        _close(_np(lr["z"]), z_ref, 1e-4, 1e-6 * rn, "dots")
        beta_ref, dbeta_ref, r_ref = beta0.copy(), dbeta0.copy(), r0.copy()
        d_ref = orc.update(kept, z_ref, p.lam, beta_ref, dbeta_ref)
        _close(_np(lr["delta"]), d_ref, 1e-4, 2e-6 * rn, "delta")
        orc.residual_csc(vals, rows, cp, kept_pos, d_ref, r_ref)
        beta1, dbeta1, r1, _ = g.get_state()
        _close(_np(beta1), beta_ref, 1e-4, 2e-6 * rn, "beta")
        _close(_np(dbeta1), dbeta_ref, 1e-4, 2e-6 * rn, "dbeta")
        _close(_np(r1), r_ref, 1e-4, 2e-6 * rn, "residual")
        assert g.objective() == pytest.approx(orc.objective(r_ref, beta_ref, p.lam), rel=1e-5)
    print("logged:", logged)
    g.close()
