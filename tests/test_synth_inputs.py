"""The synthetic inputs have the structure the configurations ask for (CPU only, reduced sizes)."""
import numpy as np
import torch

from synth import lasso_inputs as si


def _check_standardized(x, center=True):
    x = x.double()
    assert (x.norm(dim=1) - 1).abs().max() < 1e-5
    if center:
        assert x.mean(dim=1).abs().max() < 1e-6


def test_c1_iid():
    p = si.make("c1_dense_iid")
    assert p.x.shape == (5000, 1000) and p.l_prime == 200 and p.rounds == 20
    _check_standardized(p.x)
    assert int((p.beta_true != 0).sum()) == 50
    mags = p.beta_true[p.beta_true != 0].abs()
    assert mags.min() >= 0.5 and mags.max() <= 1.5
    xty = (p.x.double() @ p.y.double()).abs().max()
    assert abs(p.lam / float(xty) - 0.1) < 1e-6
    q = si.make("c1_dense_iid")
    assert torch.equal(p.x, q.x) and torch.equal(p.y, q.y)           # seeded


def test_c2_block_correlation():
    p = si.make("c2_dense_block_corr", n=2000, j=400, nnz=20, l_prime=100)
    _check_standardized(p.x)
    g = (p.x[:40].double() @ p.x[:40].double().T)
    inb = torch.stack([g[i, j] for i in range(40) for j in range(40) if i != j and i // 20 == j // 20])
    outb = torch.stack([g[i, j] for i in range(40) for j in range(40) if i // 20 != j // 20])
    assert abs(float(inb.mean()) - 0.5) < 0.05 and float(outb.abs().max()) < 0.15


def test_c3_genotype_values():
    p = si.make("c3_genotype", n=200, j=1000, nnz=10, l_prime=50)
    _check_standardized(p.x)
    # before standardisation each column had at most three distinct values
    assert max(len(torch.unique(p.x[j])) for j in range(0, 1000, 37)) <= 3


def test_c4_csc_structure():
    p = si.make("c4_sparse_csc", n=5000, j=2000, nnz_per_col=20, nnz=10, l_prime=100)
    assert p.col_ptr.tolist() == list(range(0, 20 * 2001, 20))
    rows = p.row_idx.view(2000, 20).long()
    assert bool((rows[:, 1:] > rows[:, :-1]).all()) and rows.min() >= 0 and rows.max() < 5000
    assert (p.values.view(2000, 20).double().norm(dim=1) - 1).abs().max() < 1e-6
    xd = si.csc_to_dense(p)
    _check_standardized(xd, center=False)


def test_c5_duplicates():
    p = si.make("c5_dense_duplicates", n=1000, j=600, nnz=10, l_prime=100)
    _check_standardized(p.x)
    g = (p.x.double() @ p.x.double().T).abs() - torch.eye(600, dtype=torch.float64)
    n_corr = int((g.max(dim=1).values > 0.8).sum())
    assert 0.3 * 600 <= n_corr <= 0.62 * 600          # each duplicate and (at most) its source


def test_packed_genotypes_bit_layout_and_decoding():
    # bit layout written out by hand: rows 0, 1, 2, 17 of one column hold 1, 2, 0, 2
    g = torch.zeros((1, 20), dtype=torch.int64)
    g[0, 0], g[0, 1], g[0, 17] = 1, 2, 2
    w = si.pack_genotypes(g)
    assert w.shape == (1, 4) and w.tolist() == [[1 | (2 << 2), 2 << 2, 0, 0]]
    # the top pair of bits of a word (row 15) survives the signed 32-bit storage
    g = torch.zeros((1, 16), dtype=torch.int64)
    g[0, 15] = 2
    w = si.pack_genotypes(g)
    assert int(w[0, 0]) == -(1 << 31) and si.unpack_genotypes(w, 16)[0].tolist() == [0] * 15 + [2]
    # column stride: multiples of 16 bytes
    assert [si.geno_words(n) for n in (1, 16, 64, 65, 128, 500)] == [4, 4, 4, 8, 8, 32]
    # round trip, and the decoded matrix is a standardised design whose columns take three values
    p = si.make("c3_genotype_packed", n=203, j=700, nnz=10, l_prime=50)
    gg = si.unpack_genotypes(p.codes, p.n)
    assert int(gg.max()) <= 2 and torch.equal(si.pack_genotypes(gg), p.codes)
    assert p.codes.dtype == torch.int32 and p.codes.shape == (700, si.geno_words(203))
    _check_standardized(p.x)
    x64 = (gg.double() - p.col_mean.double().view(-1, 1)) * p.col_scale.double().view(-1, 1)
    assert (p.x.double() - x64).abs().max() < 1e-6
    assert max(len(torch.unique(p.x[j])) for j in range(0, 700, 31)) <= 3
    # the two roundings of the decode, one at a time
    j, i = 5, 11
    d = (gg[j, i].float() - p.col_mean[j])            # fp32 subtraction
    assert float(p.x[j, i]) == float(d * p.col_scale[j])
