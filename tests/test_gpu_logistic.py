"""GPU parity of the rounds under the logistic loss (Section 2.1 allows it in eq. (1)) against the
oracle's logistic variant, through the C ABI.  Same bars as for the squared loss; the vector the dot
products are taken with is w_i = y_i / (1 + exp(y_i x_i^T beta)), computed in fp32 (expf) on the GPU
and in fp64 by the oracle, and the tolerances' absolute floors scale with its norm.
"""
import numpy as np
import pytest
import torch

from oracle.oracle import OracleLasso
from synth import lasso_inputs as si
from test_gpu_parity import BETA_RTOL, DOT_RTOL, OBJ_RTOL, _assert_close, _check_round, _gpu, _np, _pair

pytestmark = pytest.mark.gpu


def _problem(config="c1_dense_iid", **kw):
    lab = {k: kw.pop(k) for k in ("margin_scale", "lam_frac") if k in kw}
    return si.with_labels(si.make(config, **kw), **lab)


@pytest.mark.parametrize("config,kw,rounds", [
    ("c1_dense_iid", dict(n=1000, j=5000, l_prime=200), 20),
    ("c2_dense_block_corr", dict(n=2000, j=6000, nnz=40, l_prime=500), 8),
    ("c1_dense_iid", dict(n=1003, j=900, nnz=10, l_prime=150), 6),           # N not a multiple of 4
    ("c5_dense_duplicates", dict(n=3000, j=5000, nnz=30, l_prime=400), 6),
])
def test_teacher_forced_rounds(config, kw, rounds):
    p = _problem(config, **kw)
    g, o = _pair(p)
    assert g.objective() == pytest.approx(p.n * np.log(2.0), rel=1e-6)
    log = []
    for _ in range(rounds):
        assert _check_round(g, o, log, teacher_forced=True)
        assert g.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)
    v, gg = g.kkt(want_g=True)
    v_ref, g_ref = o.kkt(want_g=True)
    wn = max(float(np.linalg.norm(o.dots_vector().astype(np.float64))), 1.0)
    _assert_close(_np(gg), g_ref, DOT_RTOL, 1e-6 * wn, "x_j^T w for all columns")
    assert v == pytest.approx(v_ref, rel=1e-3, abs=1e-6 * wn)
    print("logged:", log)


def test_free_run_tracks_the_oracle_and_decreases_the_objective():
    p = _problem(n=800, j=2000, nnz=20, l_prime=128)
    g, o = _pair(p)
    log = []
    f = [g.objective()]
    for _ in range(40):
        if not _check_round(g, o, log, teacher_forced=False):
            o.set_state(*[_np(a) if isinstance(a, torch.Tensor) else a for a in g.get_state()])
        f.append(g.objective())
        assert f[-1] == pytest.approx(o.objective(), rel=OBJ_RTOL)
    assert f[-1] < 0.9 * f[0]
    # run() takes the same path as round(), and twice the same
    a, _ = _pair(p, keep_gram=False)
    b, _ = _pair(p, keep_gram=False)
    ia = a.run(40)
    ib = b.run(40)
    assert ia.objective == ib.objective == f[-1]
    for u, v in zip(a.get_state()[:3], g.get_state()[:3]):
        assert torch.equal(u, v)


def test_run_to_tolerance_reaches_the_scikit_learn_solution():
    from sklearn.linear_model import LogisticRegression
    p = _problem(n=300, j=200, nnz=8, l_prime=32, lam_frac=0.15)
    g, _ = _pair(p, keep_gram=False)
    info = g.run(40000, kkt_tol=1e-4, check_every=200)
    assert info.converged == 1
    ref = LogisticRegression(penalty="l1", solver="liblinear", C=1.0 / p.lam, fit_intercept=False, tol=1e-8,
                             max_iter=1000000)
    ref.fit(p.x.numpy().T.astype(np.float64), p.y.numpy().astype(np.float64))
    _assert_close(_np(g.get_state()[0]), ref.coef_[0], 1e-3, 3e-3, "converged beta")


@pytest.mark.parametrize("kw", [dict(dynamic=True), dict(n_shards=4), dict(no_deps=True, priority="uniform", p_max=20)])
def test_other_schedulers_follow_the_oracle(kw):
    # the oracle follows the GPU's index decisions (candidates bit-exact; kept set checked as for the
    # squared loss in the schedulers' own tests); here: the floating-point state after every round
    p = _problem(n=600, j=3000, nnz=15, l_prime=160)
    args = dict(lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed, loss="logistic", **kw)
    pk = _gpu()
    dev = torch.device("cuda:0")
    g = pk.StradsLasso(x=p.x.to(dev), y=p.y.to(dev), **args)
    o = OracleLasso(x=p.x.numpy(), y=p.y.numpy(), **args)
    for t in range(12):
        g.set_state(o.beta, o.dbeta, o.r, o.t)
        wn = max(float(np.linalg.norm(o.dots_vector().astype(np.float64))), 1.0)
        g.round()
        lr = g.last_round()
        forced = dict(forced_cand=_np(lr["cand"]), forced_kept_pos=_np(lr["kept_pos"]))
        if kw.get("dynamic"):
            forced["forced_mover"] = (_np(g.last_candidates()["delta_cand"]) != 0).astype(np.uint8)
        out = o.round(**forced)
        beta, dbeta, r, tt = g.get_state()
        assert tt == o.t
        _assert_close(_np(lr["z"]), out["z"], DOT_RTOL, 1e-6 * wn, f"dots (round {t})")
        _assert_close(_np(beta), o.beta, BETA_RTOL, 8e-6 * wn, f"beta (round {t})")
        _assert_close(_np(r), o.r, DOT_RTOL, 8e-6 * wn, f"state vector (round {t})")
        assert g.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)


def test_csc_and_packed_designs():
    pk = _gpu()
    dev = torch.device("cuda:0")
    # CSC: labels from the dense image of a sparse design
    ps = si.make("c4_sparse_csc", n=2000, j=5000, nnz_per_col=20, nnz=15, l_prime=200, rho=0.1)
    dense = dataclass_dense(ps)
    lab = si.with_labels(dense)
    kws = dict(lam=lab.lam, rho=ps.rho, eta=ps.eta, l_prime=ps.l_prime, seed=ps.seed, loss="logistic")
    g = pk.StradsLasso(values=ps.values.to(dev), row_idx=ps.row_idx.to(dev), col_ptr=ps.col_ptr.to(dev), n=ps.n,
                       y=lab.y.to(dev), keep_gram=True, **kws)
    o = OracleLasso(values=ps.values.numpy(), row_idx=ps.row_idx.numpy(), col_ptr=ps.col_ptr.numpy(), n=ps.n,
                    y=lab.y.numpy(), **kws)
    log = []
    for _ in range(6):
        assert _check_round(g, o, log, teacher_forced=True)
    assert g.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)
    assert g.kkt() == pytest.approx(o.kkt(), rel=1e-3, abs=1e-5)
    # packed genotypes
    pg = si.make("c3_genotype_packed", n=463, j=3000, nnz=10, l_prime=300)
    lab = si.with_labels(dataclass_dense(pg))
    kwg = dict(lam=lab.lam, rho=pg.rho, eta=pg.eta, l_prime=pg.l_prime, seed=pg.seed, loss="logistic")
    g = pk.StradsLasso(codes=pg.codes.to(dev), col_mean=pg.col_mean.to(dev), col_scale=pg.col_scale.to(dev), n=pg.n,
                       y=lab.y.to(dev), keep_gram=True, **kwg)
    o = OracleLasso(x=pg.x.numpy(), y=lab.y.numpy(), **kwg)
    for _ in range(6):
        assert _check_round(g, o, log, teacher_forced=True)
    assert g.objective() == pytest.approx(o.objective(), rel=OBJ_RTOL)
    assert g.kkt() == pytest.approx(o.kkt(), rel=1e-3, abs=1e-5)


def dataclass_dense(p):
    """A problem's design as a dense problem (for the label generator)."""
    import dataclasses
    x = si.csc_to_dense(p) if p.layout == "csc" else p.x
    return dataclasses.replace(p, layout="dense", x=x)
