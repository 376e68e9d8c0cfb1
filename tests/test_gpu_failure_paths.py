"""Failure paths that the host can force while every kernel still exits normally.

Section 2 of the paper remarks that updating correlated variables in parallel can make the iteration
diverge; the dependency check is there to prevent it.  Switching the check off (or setting rho above every
correlation) on a design made of copies of one column makes each round overshoot by the number of copies,
the state overflows fp32 within a few dozen rounds, and strads_lasso_run must report STRADS_E_DIVERGED:
no fault, no hang, the handle stays usable.  The oracle does the same on the same input (pinned on the CPU
in tests/test_oracle_solver.py).  Also here: the debug build of the library (sync and error check after every
launch, unit-norm check at create), run in a process of its own.
"""
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

from synth import lasso_inputs as si

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _copies(n=256, copies=64, seed=0):
    g = torch.Generator().manual_seed(seed)
    col = torch.randn(n, generator=g, dtype=torch.float64)
    col -= col.mean()
    col /= col.norm()
    x = col.to(torch.float32).repeat(copies, 1).contiguous()           # (J, N): every column the same unit vector
    y = (3.0 * col + 0.01 * torch.randn(n, generator=g, dtype=torch.float64)).to(torch.float32)
    return x, y


@pytest.mark.parametrize("mode", ["no_check", "rho_above_every_correlation", "dynamic_rho_above_every_correlation"])
def test_dense_divergence_is_reported_not_crashed(mode):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1312_5766_amd as pk
    dev = torch.device("cuda:0")
    x, y = _copies()
    kw = dict(x=x.to(dev), y=y.to(dev), lam=0.01, rho=0.1, eta=1e-6, l_prime=64, seed=0)
    if mode == "no_check":
        kw.update(no_deps=True, priority="uniform")
    elif mode == "rho_above_every_correlation":
        kw.update(rho=10.0)
    else:
        kw.update(rho=10.0, dynamic=True)
    g = pk.StradsLasso(**kw)
    f0 = g.objective()
    with pytest.raises(pk.StradsError) as e:
        g.run(60)
    assert e.value.code == pk.E_DIVERGED
    assert not np.isfinite(g.objective())
    # the handle is still alive: the state can be read, reset and used again
    beta, dbeta, r, t = g.get_state()
    assert t == 60 and not torch.isfinite(r).all()
    g.set_state(torch.zeros_like(beta), torch.full_like(dbeta, 1e6), y.to(dev), 0)
    assert g.objective() == pytest.approx(f0, rel=1e-6)
    # with the paper's threshold the same design is handled: one copy per round, objective goes down
    g.close()
    kw.update(rho=0.1, no_deps=False, dynamic=False, priority="squared")
    g = pk.StradsLasso(**kw)
    info = g.run(5)
    assert info.updates_done == 5 and info.objective < f0
    g.close()


def test_csc_divergence_is_reported_not_wrapped():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1312_5766_amd as pk
    dev = torch.device("cuda:0")
    n, copies, k = 512, 64, 16
    g0 = torch.Generator().manual_seed(1)
    rows = torch.sort(torch.randperm(n, generator=g0)[:k]).values.to(torch.int32)
    vals = torch.randn(k, generator=g0, dtype=torch.float64)
    vals /= vals.norm()
    values = vals.to(torch.float32).repeat(copies)
    row_idx = rows.repeat(copies)
    col_ptr = torch.arange(copies + 1, dtype=torch.int64) * k
    y = torch.zeros(n, dtype=torch.float32)
    y[rows.long()] = (3.0 * vals).to(torch.float32)
    g = pk.StradsLasso(values=values.to(dev), row_idx=row_idx.to(dev), col_ptr=col_ptr.to(dev), n=n, y=y.to(dev),
                       lam=0.01, rho=10.0, eta=1e-6, l_prime=copies, seed=0, max_col_nnz=k)
    with pytest.raises(pk.StradsError) as e:
        g.run(60)
    assert e.value.code == pk.E_DIVERGED
    r = g.get_state()[2]
    assert torch.isnan(r).any()                                   # the range check wrote NaN instead of wrapping
    # setting the state again clears the condition
    g.set_state(torch.zeros(copies), torch.full((copies,), 1e6), y, 0)
    info = g.round(want_info=True)
    assert info.n_kept == copies and torch.isfinite(g.get_state()[2]).all()
    g.close()


_DEBUG_SCRIPT = r"""
import os, sys
import torch
sys.path.insert(0, os.environ["STRADS_ROOT"])
import paper_1312_5766_amd as pk
import __graft_entry__ as ge
lib = pk.load()
assert lib.strads_lasso_debug_build() == 1, "not the debug build"
ge.smoke()                                            # a few rounds against the oracle, every launch waited for
from synth import lasso_inputs as si
dev = torch.device("cuda:0")
p = si.make("c1_dense_iid", n=300, j=500, nnz=5, l_prime=64)
kw = dict(y=p.y.to(dev), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime)
g = pk.StradsLasso(x=p.x.to(dev), **kw)
try:
    g.set_tuning("graph_rounds", 4)
    raise SystemExit("graph capture was not refused")
except pk.StradsError as e:
    assert e.code == pk.E_UNSUPPORTED
for shards in (1, 3):
    h = pk.StradsLasso(x=p.x.to(dev), n_shards=shards, dynamic=shards == 1, **kw)
    info = h.run(12, kkt_tol=1e-3, check_every=4)
    assert info.rounds_done >= 4
    h.close()
bad = p.x.clone()
bad[7] *= 1.5                                         # one column off unit norm
try:
    pk.StradsLasso(x=bad.to(dev), **kw)
    raise SystemExit("a design with a column of norm 1.5 was accepted")
except pk.StradsError as e:
    assert e.code == pk.E_INVALID_ARG
q = si.make("c4_sparse_csc", n=400, j=300, nnz_per_col=10, nnz=5, l_prime=50)
c = pk.StradsLasso(values=q.values.to(dev), row_idx=q.row_idx.to(dev), col_ptr=q.col_ptr.to(dev), n=q.n, y=q.y.to(dev),
                   lam=q.lam, rho=q.rho, eta=q.eta, l_prime=q.l_prime)
c.run(5)
c.close()
v2 = q.values.clone(); v2[:10] *= 2
try:
    pk.StradsLasso(values=v2.to(dev), row_idx=q.row_idx.to(dev), col_ptr=q.col_ptr.to(dev), n=q.n, y=q.y.to(dev),
                   lam=q.lam, rho=q.rho, eta=q.eta, l_prime=q.l_prime)
    raise SystemExit("a CSC design with a column of norm 2 was accepted")
except pk.StradsError as e:
    assert e.code == pk.E_INVALID_ARG
print("DEBUG_BUILD_OK")
"""


def test_debug_build_runs_rounds_and_checks_unit_norms():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    lib = os.path.join(ROOT, "paper_1312_5766_amd", "libstrads_lasso_debug.so")
    assert os.path.exists(lib), "build it with `python -m paper_1312_5766_amd.build --debug`"
    env = dict(os.environ, STRADS_LASSO_DEBUG="1", STRADS_ROOT=ROOT)
    r = subprocess.run([sys.executable, "-c", _DEBUG_SCRIPT], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0 and "DEBUG_BUILD_OK" in r.stdout, (r.stdout[-1500:], r.stderr[-3000:])
