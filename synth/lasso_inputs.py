"""Seeded synthetic Lasso problems shaped like the paper's workloads.

This module only *produces inputs* (design matrix, response, regularisation
weight, scheduler parameters).  It holds none of the scheduling method's
arithmetic and is the one piece of code that both the CPU oracle's tests and
the HIP path's tests/bench may use.  Everything is drawn from a seeded
``torch.Generator`` so a (config, seed, device) triple always yields the same
arrays; the arrays handed to the oracle and to the GPU are the *same* arrays
(copied across the PCIe bus), never two independent draws.

The paper (Experimental Results, "Datasets") ran Lasso on a genotype matrix of
463 x 508,999 SNP covariates and on a synthetic 450 x 1,000,000 design with
10,000 true non-zeros; neither is available here, so the five configurations
below stand in for them.  Dense designs are stored column-major: ``x`` is a
``(J, N)`` contiguous fp32 tensor whose row ``j`` is covariate ``x_j``.
Columns are standardised (zero mean, unit l2 norm) as the paper's problem
statement for eq. (1) assumes; the sparse design is unit-normalised only.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import torch


@dataclasses.dataclass
class LassoProblem:
    name: str
    n: int                      # rows (samples)
    j: int                      # columns (covariates)
    layout: str                 # "dense" | "csc" | "geno2"
    y: torch.Tensor             # (n,) fp32
    lam: float                  # lambda of eq. (1)
    rho: float                  # dependency threshold
    eta: float                  # priority floor
    l_prime: int                # candidates per round (P')
    rounds: int                 # rounds the config asks for
    seed: int
    beta_true: torch.Tensor     # (j,) fp32, the planted coefficients
    x: Optional[torch.Tensor] = None        # dense: (j, n) fp32 contiguous
    values: Optional[torch.Tensor] = None   # csc: (nnz,) fp32
    row_idx: Optional[torch.Tensor] = None  # csc: (nnz,) int32, sorted per column
    col_ptr: Optional[torch.Tensor] = None  # csc: (j+1,) int64
    codes: Optional[torch.Tensor] = None    # geno2: (j, 4*ceil(n/64)) int32, 16 two-bit genotype counts per word
    col_mean: Optional[torch.Tensor] = None   # geno2: (j,) fp32
    col_scale: Optional[torch.Tensor] = None  # geno2: (j,) fp32; x_ij = fl(fl(g_ij - mean_j) * scale_j)
    loss: str = "squared"                   # "squared" | "logistic" (then y holds labels in {-1, +1})
    dup_src: Optional[torch.Tensor] = None  # config 5: (j,) int64, the column a duplicate was copied from, -1 elsewhere

    def to(self, device) -> "LassoProblem":
        kw = {}
        for f in dataclasses.fields(self):
            v = getattr(self, f.name)
            kw[f.name] = v.to(device) if isinstance(v, torch.Tensor) else v
        return LassoProblem(**kw)


# ----------------------------------------------------------------------------
# helpers (data preparation only)
# ----------------------------------------------------------------------------

def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _standardize_rows_(block: torch.Tensor, center: bool = True) -> torch.Tensor:
    """Centre (optionally) and scale every row of an fp64 block to unit l2 norm."""
    if center:
        block -= block.mean(dim=1, keepdim=True)
    nrm = block.norm(dim=1, keepdim=True)
    nrm = torch.where(nrm > 0, nrm, torch.ones_like(nrm))
    block /= nrm
    return block


def _planted_beta(j: int, nnz: int, lo: float, hi: float, g: torch.Generator, device) -> torch.Tensor:
    nnz = min(nnz, j)
    idx = torch.randperm(j, generator=g, device=device)[:nnz]
    mag = lo + (hi - lo) * torch.rand(nnz, generator=g, device=device, dtype=torch.float64)
    sgn = torch.where(torch.rand(nnz, generator=g, device=device) < 0.5, -1.0, 1.0).to(torch.float64)
    beta = torch.zeros(j, dtype=torch.float64, device=device)
    beta[idx] = mag * sgn
    return beta


def _dense_response(x: torch.Tensor, beta64: torch.Tensor, sigma: float, g: torch.Generator,
                    chunk: int = 8192) -> torch.Tensor:
    """y = X beta* + N(0, sigma^2), accumulated in fp64 over column chunks."""
    j, n = x.shape
    y = torch.zeros(n, dtype=torch.float64, device=x.device)
    nz = torch.nonzero(beta64).flatten()
    for s in range(0, nz.numel(), chunk):
        ids = nz[s:s + chunk]
        y += beta64[ids] @ x[ids].to(torch.float64)
    y += sigma * torch.randn(n, generator=g, device=x.device, dtype=torch.float64)
    return y


def _dense_max_abs_xty(x: torch.Tensor, y64: torch.Tensor, chunk: int = 8192) -> float:
    j, _ = x.shape
    m = 0.0
    for s in range(0, j, chunk):
        m = max(m, float((x[s:s + chunk].to(torch.float64) @ y64).abs().max()))
    return m


def _finish_dense(name, x, nnz, lo, hi, sigma, lam_frac, rho, eta, l_prime, rounds, seed, g):
    j, n = x.shape
    beta64 = _planted_beta(j, nnz, lo, hi, g, x.device)
    y64 = _dense_response(x, beta64, sigma, g)
    y32 = y64.to(torch.float32)
    lam = lam_frac * _dense_max_abs_xty(x, y32.to(torch.float64))
    lam = float(torch.tensor(lam, dtype=torch.float32))
    return LassoProblem(name=name, n=n, j=j, layout="dense", x=x, y=y32, lam=lam, rho=rho, eta=eta,
                        l_prime=min(l_prime, j), rounds=rounds, seed=seed,
                        beta_true=beta64.to(torch.float32))


# ----------------------------------------------------------------------------
# the five configurations
# ----------------------------------------------------------------------------

def dense_iid(n=1000, j=5000, nnz=50, sigma=0.1, lam_frac=0.1, l_prime=200, rho=0.1, eta=1e-6,
              rounds=20, seed=0, device="cpu", chunk=4096, name="dense_iid") -> LassoProblem:
    """Config 1: i.i.d. N(0,1) entries, standardised columns."""
    g = _gen(seed, device)
    x = torch.empty((j, n), dtype=torch.float32, device=device)
    for s in range(0, j, chunk):
        e = min(j, s + chunk)
        blk = torch.randn((e - s, n), generator=g, device=device, dtype=torch.float64)
        x[s:e] = _standardize_rows_(blk).to(torch.float32)
    return _finish_dense(name, x, nnz, 0.5, 1.5, sigma, lam_frac, rho, eta, l_prime, rounds, seed, g)


def dense_block_corr(n=10000, j=100000, block=20, corr=0.5, nnz=500, sigma=0.1, lam_frac=0.05,
                     l_prime=1000, rho=0.1, eta=1e-6, rounds=100, seed=0, device="cpu",
                     name="dense_block_corr") -> LassoProblem:
    """Config 2: blocks of ``block`` columns share a latent factor (pairwise corr ``corr``)."""
    g = _gen(seed, device)
    x = torch.empty((j, n), dtype=torch.float32, device=device)
    a, b = math.sqrt(corr), math.sqrt(1.0 - corr)
    blocks_per_chunk = max(1, 4000 // block)
    step = blocks_per_chunk * block
    for s in range(0, j, step):
        e = min(j, s + step)
        nb = (e - s + block - 1) // block
        f = torch.randn((nb, n), generator=g, device=device, dtype=torch.float32)
        blk = torch.randn((e - s, n), generator=g, device=device, dtype=torch.float32)
        blk = (b * blk + a * f.repeat_interleave(block, dim=0)[: e - s]).to(torch.float64)
        x[s:e] = _standardize_rows_(blk).to(torch.float32)
    return _finish_dense(name, x, nnz, 0.5, 1.5, sigma, lam_frac, rho, eta, l_prime, rounds, seed, g)


def genotype(n=500, j=500000, nnz=100, sigma=0.5, lam_frac=0.05, l_prime=2000, rho=0.1, eta=1e-6,
             rounds=200, seed=0, device="cpu", chunk=20000, name="genotype") -> LassoProblem:
    """Config 3: entries in {0,1,2} ~ Binomial(2, p_j), p_j ~ U(0.05, 0.5), standardised."""
    g = _gen(seed, device)
    x = torch.empty((j, n), dtype=torch.float32, device=device)
    for s in range(0, j, chunk):
        e = min(j, s + chunk)
        p = 0.05 + 0.45 * torch.rand((e - s, 1), generator=g, device=device)
        blk = ((torch.rand((e - s, n), generator=g, device=device) < p).to(torch.float64)
               + (torch.rand((e - s, n), generator=g, device=device) < p).to(torch.float64))
        # a constant column carries no information: redraw it as a single minor-allele carrier
        const = (blk.max(dim=1).values == blk.min(dim=1).values)
        if bool(const.any()):
            rows = torch.nonzero(const).flatten()
            pos = torch.randint(0, n, (rows.numel(),), generator=g, device=device)
            blk[rows] = 0.0
            blk[rows, pos] = 1.0
        x[s:e] = _standardize_rows_(blk).to(torch.float32)
    return _finish_dense(name, x, nnz, 0.2, 1.0, sigma, lam_frac, rho, eta, l_prime, rounds, seed, g)


def geno_words(n: int) -> int:
    """32-bit words per packed genotype column: 16 rows per word, columns padded to 16 bytes."""
    return (n + 63) // 64 * 4


def pack_genotypes(g: torch.Tensor) -> torch.Tensor:
    """(j, n) integer counts in {0,1,2} -> (j, geno_words(n)) int32: row 16w+e of a column sits in
    bits 2e, 2e+1 of its word w; rows past n are 0."""
    j, n = g.shape
    words = geno_words(n)
    pad = torch.zeros((j, words * 16), dtype=torch.int64, device=g.device)
    pad[:, :n] = g.to(torch.int64)
    shifts = (2 * torch.arange(16, device=g.device, dtype=torch.int64)).view(1, 1, 16)
    packed = (pad.view(j, words, 16) << shifts).sum(dim=2)              # < 2^32
    return torch.where(packed >= 2 ** 31, packed - 2 ** 32, packed).to(torch.int32)


def unpack_genotypes(codes: torch.Tensor, n: int) -> torch.Tensor:
    """Inverse of pack_genotypes: (j, n) uint8."""
    j, words = codes.shape
    w = codes.to(torch.int64) & 0xFFFFFFFF
    shifts = (2 * torch.arange(16, device=codes.device, dtype=torch.int64)).view(1, 1, 16)
    return ((w.view(j, words, 1) >> shifts) & 3).view(j, words * 16)[:, :n].to(torch.uint8)


def decode_genotypes(codes: torch.Tensor, mean: torch.Tensor, scale: torch.Tensor, n: int) -> torch.Tensor:
    """The fp32 design a packed genotype matrix stands for: x_ij = fl(fl(g_ij - mean_j) * scale_j),
    both operations in fp32 (exactly what the library's kernels decode)."""
    g = unpack_genotypes(codes, n).to(torch.float32)
    return (g - mean.view(-1, 1).to(torch.float32)) * scale.view(-1, 1).to(torch.float32)


def genotype_packed(n=500, j=500000, nnz=100, sigma=0.5, lam_frac=0.05, l_prime=2000, rho=0.1, eta=1e-6,
                    rounds=200, seed=0, device="cpu", chunk=20000, keep_dense=True,
                    name="genotype_packed") -> LassoProblem:
    """Config 3 stored as 2-bit genotype counts plus a mean and a scale per column.  The counts are
    drawn as in `genotype`; mean and scale are the fp64 column mean and 1 / l2-norm of the centred
    column, rounded to fp32.  With keep_dense the decoded fp32 design (what the oracle is given) is
    kept in `x`; y and lambda are always computed from it, chunk by chunk."""
    g = _gen(seed, device)
    words = geno_words(n)
    codes = torch.empty((j, words), dtype=torch.int32, device=device)
    mean = torch.empty(j, dtype=torch.float32, device=device)
    scale = torch.empty(j, dtype=torch.float32, device=device)
    x = torch.empty((j, n), dtype=torch.float32, device=device) if keep_dense else None
    for s in range(0, j, chunk):
        e = min(j, s + chunk)
        p = 0.05 + 0.45 * torch.rand((e - s, 1), generator=g, device=device)
        blk = ((torch.rand((e - s, n), generator=g, device=device) < p).to(torch.int64)
               + (torch.rand((e - s, n), generator=g, device=device) < p).to(torch.int64))
        const = (blk.max(dim=1).values == blk.min(dim=1).values)
        if bool(const.any()):
            rows = torch.nonzero(const).flatten()
            pos = torch.randint(0, n, (rows.numel(),), generator=g, device=device)
            blk[rows] = 0
            blk[rows, pos] = 1
        b64 = blk.to(torch.float64)
        mu = b64.mean(dim=1)
        nrm = (b64 - mu.view(-1, 1)).norm(dim=1)
        mean[s:e] = mu.to(torch.float32)
        scale[s:e] = (1.0 / nrm).to(torch.float32)
        codes[s:e] = pack_genotypes(blk)
        if keep_dense:
            x[s:e] = decode_genotypes(codes[s:e], mean[s:e], scale[s:e], n)

    def cols(ids):                                       # decoded columns, on demand
        return x[ids] if keep_dense else decode_genotypes(codes[ids], mean[ids], scale[ids], n)

    beta64 = _planted_beta(j, nnz, 0.2, 1.0, g, device)
    nz = torch.nonzero(beta64).flatten()
    y64 = beta64[nz] @ cols(nz).to(torch.float64)
    y64 += sigma * torch.randn(n, generator=g, device=device, dtype=torch.float64)
    y32 = y64.to(torch.float32)
    m = 0.0
    for s in range(0, j, chunk):
        ids = torch.arange(s, min(j, s + chunk), device=device)
        m = max(m, float((cols(ids).to(torch.float64) @ y32.to(torch.float64)).abs().max()))
    lam = float(torch.tensor(lam_frac * m, dtype=torch.float32))
    return LassoProblem(name=name, n=n, j=j, layout="geno2", x=x, y=y32, lam=lam, rho=rho, eta=eta,
                        l_prime=min(l_prime, j), rounds=rounds, seed=seed, beta_true=beta64.to(torch.float32),
                        codes=codes, col_mean=mean, col_scale=scale)


def dense_duplicates(n=50000, j=1000000, dup_frac=0.3, dup_corr=0.9, nnz=2000, sigma=0.1,
                     lam_frac=0.02, l_prime=8000, rho=0.1, eta=1e-6, rounds=0, seed=0, device="cpu",
                     chunk=2048, name="dense_duplicates") -> LassoProblem:
    """Config 5: 30% of the columns are noisy copies (corr 0.9) of other columns."""
    g = _gen(seed, device)
    x = torch.empty((j, n), dtype=torch.float32, device=device)
    perm = torch.randperm(j, generator=g, device=device)
    n_dup = int(round(dup_frac * j))
    n_dup = min(n_dup, j - 1)
    dup_ids, src_pool = perm[:n_dup], perm[n_dup:]
    is_dup = torch.zeros(j, dtype=torch.bool, device=device)
    is_dup[dup_ids] = True
    src_of = torch.full((j,), -1, dtype=torch.int64, device=device)
    if n_dup:
        src_of[dup_ids] = src_pool[torch.randint(0, src_pool.numel(), (n_dup,), generator=g, device=device)]
    # originals first, chunk by chunk
    for s in range(0, j, chunk):
        e = min(j, s + chunk)
        blk = torch.randn((e - s, n), generator=g, device=device, dtype=torch.float32).to(torch.float64)
        x[s:e] = _standardize_rows_(blk).to(torch.float32)
    # overwrite duplicates: x_d = c * x_s + sqrt(1 - c^2) * e, then standardise again
    c, d = dup_corr, math.sqrt(1.0 - dup_corr * dup_corr)
    ids = torch.nonzero(is_dup).flatten()
    for s in range(0, ids.numel(), chunk):
        di = ids[s:s + chunk]
        e = torch.randn((di.numel(), n), generator=g, device=device, dtype=torch.float32).to(torch.float64)
        e = _standardize_rows_(e)
        blk = c * x[src_of[di]].to(torch.float64) + d * e
        x[di] = _standardize_rows_(blk).to(torch.float32)
    p = _finish_dense(name, x, nnz, 0.5, 1.5, sigma, lam_frac, rho, eta, l_prime, rounds, seed, g)
    p.dup_src = src_of
    return p


def sparse_csc(n=100000, j=1000000, nnz_per_col=100, nnz=1000, sigma=0.1, lam_frac=0.02,
               l_prime=4000, rho=0.05, eta=1e-6, rounds=200, seed=0, device="cpu", chunk=20000,
               name="sparse_csc") -> LassoProblem:
    """Config 4: CSC design, exactly ``nnz_per_col`` distinct uniform rows per column, N(0,1)
    values, unit-normalised (not centred)."""
    g = _gen(seed, device)
    k = min(nnz_per_col, n)
    values = torch.empty(j * k, dtype=torch.float32, device=device)
    row_idx = torch.empty(j * k, dtype=torch.int32, device=device)
    col_ptr = (torch.arange(j + 1, dtype=torch.int64, device=device) * k)
    for s in range(0, j, chunk):
        e = min(j, s + chunk)
        c = e - s
        # k distinct rows per column: take the k smallest of n random keys when n is small,
        # otherwise draw with replacement, and repair the (rare) repeats by redrawing.
        if n <= 4 * k:
            rows = torch.rand((c, n), generator=g, device=device).argsort(dim=1)[:, :k]
        else:
            rows = torch.randint(0, n, (c, k), generator=g, device=device)
            for _ in range(64):
                rows, _ = rows.sort(dim=1)
                dup = torch.zeros_like(rows, dtype=torch.bool)
                dup[:, 1:] = rows[:, 1:] == rows[:, :-1]
                nd = int(dup.sum())
                if nd == 0:
                    break
                rows[dup] = torch.randint(0, n, (nd,), generator=g, device=device)
        rows, _ = rows.sort(dim=1)
        vals = torch.randn((c, k), generator=g, device=device, dtype=torch.float64)
        vals = _standardize_rows_(vals, center=False)
        values[s * k:e * k] = vals.to(torch.float32).flatten()
        row_idx[s * k:e * k] = rows.to(torch.int32).flatten()
    beta64 = _planted_beta(j, nnz, 0.5, 1.5, g, device)
    # y = X beta* + noise via the planted columns only
    y64 = torch.zeros(n, dtype=torch.float64, device=device)
    nzc = torch.nonzero(beta64).flatten()
    for cidx in nzc.tolist():
        sl = slice(cidx * k, (cidx + 1) * k)
        y64.index_add_(0, row_idx[sl].to(torch.int64), values[sl].to(torch.float64) * beta64[cidx])
    y64 += sigma * torch.randn(n, generator=g, device=device, dtype=torch.float64)
    y32 = y64.to(torch.float32)
    # lambda = frac * max_j |x_j^T y|
    m = 0.0
    yy = y32.to(torch.float64)
    for s in range(0, j, chunk * 8):
        e = min(j, s + chunk * 8)
        sl = slice(s * k, e * k)
        dots = (values[sl].to(torch.float64) * yy[row_idx[sl].to(torch.int64)]).view(e - s, k).sum(dim=1)
        m = max(m, float(dots.abs().max()))
    lam = float(torch.tensor(lam_frac * m, dtype=torch.float32))
    return LassoProblem(name=name, n=n, j=j, layout="csc", values=values, row_idx=row_idx,
                        col_ptr=col_ptr, y=y32, lam=lam, rho=rho, eta=eta, l_prime=min(l_prime, j),
                        rounds=rounds, seed=seed, beta_true=beta64.to(torch.float32))


def csc_to_dense(p: LassoProblem) -> torch.Tensor:
    """Dense (j, n) fp32 copy of a CSC problem's design (for small test sizes only)."""
    x = torch.zeros((p.j, p.n), dtype=torch.float32, device=p.values.device)
    counts = (p.col_ptr[1:] - p.col_ptr[:-1])
    cols = torch.repeat_interleave(torch.arange(p.j, device=x.device), counts)
    x[cols, p.row_idx.to(torch.int64)] = p.values
    return x


def with_labels(p: LassoProblem, margin_scale: float = 4.0, lam_frac: float = 0.1, seed: int = 1) -> LassoProblem:
    """The same design as a classification problem (the logistic loss of Section 2.1): the planted
    coefficients give margins m = X beta*, scaled so that their standard deviation is margin_scale;
    label y_i = +1 with probability 1 / (1 + exp(-m_i)), else -1.  lambda = lam_frac * max |X^T y| / 2
    (all coefficients stay at zero from lambda = max |X^T y| / 2 upwards).  Dense designs only."""
    assert p.layout == "dense"
    g = _gen(seed, p.x.device)
    b64 = p.beta_true.to(torch.float64)
    nz = torch.nonzero(b64).flatten()
    m = b64[nz] @ p.x[nz].to(torch.float64)
    m = m * (margin_scale / float(m.std()))
    u = torch.rand(p.n, generator=g, device=p.x.device, dtype=torch.float64)
    y = torch.where(u < torch.sigmoid(m), 1.0, -1.0).to(torch.float32)
    lam = 0.5 * lam_frac * _dense_max_abs_xty(p.x, y.to(torch.float64))
    lam = float(torch.tensor(lam, dtype=torch.float32))
    return dataclasses.replace(p, name=p.name + "_logistic", y=y, lam=lam, loss="logistic")


CONFIGS = {
    "c1_dense_iid": dense_iid,
    "c2_dense_block_corr": dense_block_corr,
    "c3_genotype": genotype,
    "c4_sparse_csc": sparse_csc,
    "c5_dense_duplicates": dense_duplicates,
    "c3_genotype_packed": genotype_packed,
}


def make(config: str, device="cpu", **overrides) -> LassoProblem:
    """Build one of the named configurations; ``overrides`` shrink it for tests
    (same recipe, smaller n / j / l_prime)."""
    fn = CONFIGS[config]
    return fn(device=device, name=config, **overrides)
