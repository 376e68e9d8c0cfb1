"""GPU parity of the other schedulers against the oracle: linear priority (Algorithm 1 as printed),
uniform draw with the dependency check ("static correlation" scheduler of Section 5.1), and
uniform draw without a check (Shotgun).  Same bars as the default round."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from synth import lasso_inputs as si
from test_gpu_parity import _check_round, _gpu, _np, _pair

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("priority", ["linear", "uniform", "squared"])
def test_keys_and_candidate_lists_are_bit_identical(priority):
    p = si.make("c1_dense_iid", n=64, j=20000, nnz=20, l_prime=700)
    g, o = _pair(p, keep_gram=False, priority=priority)
    rng = np.random.default_rng(1)
    db = np.where(rng.random(p.j) < 0.3, 1e6, np.abs(rng.normal(size=p.j)) * 0.1).astype(np.float32)
    db[rng.random(p.j) < 0.2] = 0.0
    g.set_state(None, db, None, 5)
    keys = _np(g.stage_keys(5))
    ref = orc.priority_keys(db, p.eta, p.seed, 5, priority)
    assert np.array_equal(keys.view(np.uint32), (ref + np.float32(0.0)).view(np.uint32))
    g.round()
    assert np.array_equal(_np(g.last_round()["cand"]), orc.draw(ref, p.l_prime))


@pytest.mark.parametrize("kw", [
    dict(priority="linear"),
    dict(priority="uniform"),
    dict(priority="uniform", no_deps=True),
    dict(priority="uniform", no_deps=True, p_max=100),
    dict(priority="linear", dynamic=True),
])
def test_teacher_forced_rounds(kw):
    p = si.make("c2_dense_block_corr", n=2000, j=8000, nnz=40, l_prime=500)
    if kw.get("dynamic"):
        from test_gpu_dynamic import _check_round as check, _pair as pair
        g, o = pair(p, **{k: v for k, v in kw.items() if k != "dynamic"})
    else:
        check, (g, o) = _check_round, _pair(p, **kw)
    log = []
    for _ in range(20):
        if kw.get("dynamic"):
            check(g, o, log)
        else:
            assert check(g, o, log, teacher_forced=True)
    print(kw, log)


def test_csc_design_with_uniform_draw_and_no_check():
    p = si.make("c4_sparse_csc", n=3000, j=6000, nnz_per_col=30, nnz=30, l_prime=300)
    g, o = _pair(p, priority="uniform", no_deps=True)
    for _ in range(8):
        assert _check_round(g, o, [], teacher_forced=True)


def test_shotgun_on_duplicated_columns_overshoots_as_the_closed_form_says():
    pk = _gpu()
    dev = torch.device("cuda:0")
    x = torch.zeros((2, 4), dtype=torch.float32)
    x[:, 0] = 1.0
    y = torch.tensor([2.0, 0, 0, 0])
    g = pk.StradsLasso(x=x.to(dev), y=y.to(dev), lam=0.5, rho=0.1, eta=1e-6, l_prime=2, priority="uniform",
                       no_deps=True)
    g.round()
    beta, _, r, _ = g.get_state()
    assert beta.tolist() == [1.5, 1.5] and r.tolist() == [-1.0, 0, 0, 0] and g.objective() == 2.0
