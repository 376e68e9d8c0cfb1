"""Every combination of design layout, dependency rule, priority, shard count and loss on a small
problem: a few teacher-forced rounds each.  The candidate list must be the oracle's own draw, bit
for bit; the GPU's mover and keep decisions must be the oracle's own or admissible variants of them
(a tentative change within the dot-product tolerance of zero; a Gram entry within the Gram tolerance
of rho, tests/parity_rules.py); the oracle then follows them and all floating-point state is compared
after every round.  The entry-by-entry checks of the Gram live in the per-feature test files; this one
is about the options working together.
"""
import dataclasses
import itertools

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from oracle.oracle import OracleLasso
from parity_rules import check_kept_against_oracle
from synth import lasso_inputs as si
from test_gpu_parity import BETA_RTOL, DOT_RTOL, OBJ_RTOL, _assert_close, _gpu, _np, _ref_candidates

pytestmark = pytest.mark.gpu


def _designs():
    dense = si.make("c2_dense_block_corr", n=260, j=900, nnz=12, l_prime=96, rho=0.2)
    sparse = si.make("c4_sparse_csc", n=700, j=900, nnz_per_col=14, nnz=12, l_prime=96, rho=0.2)
    packed = si.make("c3_genotype_packed", n=203, j=900, nnz=12, l_prime=96, rho=0.2)
    return {"dense": dense, "csc": sparse, "geno2": packed}


_DESIGNS = None


def _case(layout, loss):
    global _DESIGNS
    if _DESIGNS is None:
        _DESIGNS = _designs()
    p = _DESIGNS[layout]
    if loss == "logistic":
        x = si.csc_to_dense(p) if layout == "csc" else p.x
        lab = si.with_labels(dataclasses.replace(p, layout="dense", x=x))
        p = dataclasses.replace(p, y=lab.y, lam=lab.lam, loss="logistic")
    return p


def _build(pk, p, **kw):
    dev = torch.device("cuda:0")
    if p.layout == "dense":
        g = pk.StradsLasso(x=p.x.to(dev), y=p.y.to(dev), **kw)
        o = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), **kw)
    elif p.layout == "geno2":
        g = pk.StradsLasso(codes=p.codes.to(dev), col_mean=p.col_mean.to(dev), col_scale=p.col_scale.to(dev), n=p.n,
                           y=p.y.to(dev), **kw)
        o = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), **kw)
    else:
        g = pk.StradsLasso(values=p.values.to(dev), row_idx=p.row_idx.to(dev), col_ptr=p.col_ptr.to(dev), n=p.n,
                           y=p.y.to(dev), **kw)
        o = OracleLasso(values=p.values.numpy(), row_idx=p.row_idx.numpy(), col_ptr=p.col_ptr.numpy(), n=p.n,
                        y=p.y.numpy(), **kw)
    return g, o


_COMBOS = list(itertools.product(("dense", "csc", "geno2"), ("static", "dynamic", "none"),
                                 ("squared", "linear", "uniform"), (1, 3), ("squared", "logistic")))


@pytest.mark.parametrize("layout,deps,priority,shards,loss", _COMBOS,
                         ids=["-".join(map(str, c)) for c in _COMBOS])
def test_options_work_together(layout, deps, priority, shards, loss):
    pk = _gpu()
    p = _case(layout, loss)
    kw = dict(lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=5, priority=priority, n_shards=shards,
              dynamic=deps == "dynamic", no_deps=deps == "none", p_max=40 if deps == "none" else 0)
    if loss != "squared":
        kw["loss"] = loss
    g, o = _build(pk, p, **kw)
    assert g.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)
    for t in range(4):
        g.set_state(o.beta, o.dbeta, o.r, o.t)
        dbeta0, t0 = o.dbeta.copy(), o.t
        wn = max(float(np.linalg.norm(o.dots_vector().astype(np.float64))), 1.0)
        g.round()
        lr = g.last_round()
        cand = _np(lr["cand"])
        assert np.array_equal(cand, _ref_candidates(o, dbeta0, t0)), f"candidate list (round {t})"
        kept_pos = _np(lr["kept_pos"])
        forced = dict(forced_cand=cand, forced_kept_pos=kept_pos)
        scale = 4.0 if loss == "logistic" else 1.0
        if deps != "none":
            # the index decisions the oracle is about to follow are its own, or admissible variants
            Gref = orc.gram_csc(o.x, o.row_idx, o.col_ptr, cand) if o.csc else orc.gram_dense(o.x, cand)
            if deps == "dynamic":
                d_gpu = _np(g.last_candidates()["delta_cand"])
                mover_gpu = d_gpu != 0
                dv = o.dots_vector()
                z_ref = orc.dots_csc(o.x, o.row_idx, o.col_ptr, cand, dv) if o.csc else orc.dots_dense(o.x, cand, dv)
                d_ref = orc.update(cand, z_ref, o.lam, o.beta.copy(), o.dbeta.copy(), inv_kappa=scale)
                differ = mover_gpu != (d_ref != 0)
                tol = DOT_RTOL * np.abs(z_ref[differ]) * scale + 2e-6 * scale * wn
                assert np.all(np.abs(d_ref[differ]) <= tol) and np.all(np.abs(d_gpu[differ]) <= tol), "mover decision"
                Gref[~mover_gpu, :] = 0
                Gref[:, ~mover_gpu] = 0
                forced["forced_mover"] = mover_gpu.astype(np.uint8)
            check_kept_against_oracle(Gref, kept_pos, orc.greedy_filter(Gref, o.rho, o.p_max), o.rho, o.p_max, [],
                                      f"round {t}")
        out = o.round(**forced)
        assert np.array_equal(_np(lr["kept"]), out["kept"])
        beta, dbeta, r, tt = g.get_state()
        assert tt == o.t
        _assert_close(_np(lr["z"]), out["z"], DOT_RTOL, 1e-6 * wn, f"dots (round {t})")
        _assert_close(_np(beta), o.beta, BETA_RTOL, 2e-6 * scale * wn, f"beta (round {t})")
        _assert_close(_np(dbeta), o.dbeta, BETA_RTOL, 2e-6 * scale * wn, f"delta beta (round {t})")
        _assert_close(_np(r), o.r, DOT_RTOL, 2e-6 * scale * wn, f"state vector (round {t})")
        assert g.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)
    v, v_ref = g.kkt(), o.kkt()
    assert v == pytest.approx(v_ref, rel=1e-3, abs=1e-5 * wn)
    g.close()
