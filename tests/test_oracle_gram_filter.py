"""Pins for the oracle's dependency step (Step 2 of SAP): Gram entries and the greedy choice of B_1."""
import itertools

import numpy as np
import torch

from synth import lasso_inputs as si


def test_gram_matches_fp64_matmul_and_has_unit_diagonal(oracle_mod):
    p = si.make("c2_dense_block_corr", n=400, j=600, nnz=10, l_prime=50)
    x = p.x.numpy()
    cand = np.random.default_rng(0).permutation(p.j)[:97].astype(np.int32)
    G = oracle_mod.gram_dense(x, cand)
    xs = x[cand].astype(np.float64)
    ref = xs @ xs.T
    assert np.abs(G - ref).max() < 1e-7
    assert np.abs(np.diag(G) - 1.0).max() < 1e-6
    assert np.array_equal(G, G.T)
    # same-block columns of this design are correlated ~0.5, others ~0
    cand = np.arange(40, dtype=np.int32)
    G = oracle_mod.gram_dense(x, cand)
    assert 0.3 < G[0, 1] < 0.7 and abs(G[0, 25]) < 0.25


def test_gram_is_not_transposed_or_shifted(oracle_mod):
    # columns with a known, asymmetric pattern: x_0 = e_0, x_1 = (e_0 + e_1)/sqrt2, x_2 = e_2
    x = np.zeros((3, 5), np.float32)
    x[0, 0] = 1
    x[1, 0] = x[1, 1] = 2 ** -0.5
    x[2, 2] = 1
    G = oracle_mod.gram_dense(x, np.array([2, 0, 1], np.int32))
    ref = np.array([[1, 0, 0], [0, 1, 2 ** -0.5], [0, 2 ** -0.5, 1]])
    assert np.allclose(G, ref, atol=1e-7)


def test_gram_rows_and_pairs_are_the_same_numbers_as_the_whole_gram(oracle_mod):
    p = si.make("c5_dense_duplicates", n=300, j=400, nnz=10, l_prime=50)
    x = p.x.numpy()
    rng = np.random.default_rng(4)
    cand = rng.permutation(p.j)[:83].astype(np.int32)
    G = oracle_mod.gram_dense(x, cand)
    rows = np.array([82, 0, 17, 17, 40], np.int32)
    R = oracle_mod.gram_rows_dense(x, cand, rows)
    assert R.shape == (5, 83) and np.array_equal(R, G[rows])
    pa, pb = rng.integers(0, 83, 500).astype(np.int32), rng.integers(0, 83, 500).astype(np.int32)
    assert np.array_equal(oracle_mod.gram_pairs_dense(x, cand, pa, pb), G[pa, pb])
    # and against an fp64 matmul, so that a transposed or shifted index in the row variant shows
    xs = x[cand].astype(np.float64)
    assert np.abs(R - (xs[rows] @ xs.T)).max() < 1e-7


def test_gram_csc_equals_dense(oracle_mod):
    p = si.make("c4_sparse_csc", n=300, j=500, nnz_per_col=12, nnz=10, l_prime=40)
    xd = si.csc_to_dense(p).numpy()
    cand = np.random.default_rng(2).permutation(p.j)[:60].astype(np.int32)
    Gs = oracle_mod.gram_csc(p.values.numpy(), p.row_idx.numpy(), p.col_ptr.numpy(), cand)
    Gd = oracle_mod.gram_dense(xd, cand)
    assert np.abs(Gs - Gd).max() < 1e-7
    assert np.abs(np.diag(Gs) - 1).max() < 1e-6


def _lexicographically_first_maximal(G, rho):
    """Brute force over all subsets: pairwise-admissible sets, keep the maximal ones (no candidate
    can be added), return the lexicographically smallest as a sorted tuple."""
    L = G.shape[0]
    ok = np.abs(G) < rho
    best = None
    for mask in range(1 << L):
        s = [i for i in range(L) if mask >> i & 1]
        if any(not ok[a, b] for a, b in itertools.combinations(s, 2)):
            continue
        if any(all(ok[c, a] for a in s) for c in range(L) if c not in s):
            continue                      # not maximal
        t = tuple(s)
        if best is None or t < best:
            best = t
    return best


def test_filter_equals_brute_force(oracle_mod):
    rng = np.random.default_rng(5)
    for trial in range(60):
        L = int(rng.integers(1, 11))
        A = rng.uniform(-0.3, 0.3, (L, L)).astype(np.float32)
        G = np.triu(A, 1) + np.triu(A, 1).T + np.eye(L, dtype=np.float32)
        rho = float(rng.uniform(0.05, 0.3))
        kept = oracle_mod.greedy_filter(G, rho)
        assert tuple(kept.tolist()) == _lexicographically_first_maximal(G, rho)


def test_filter_is_strict_and_respects_cap(oracle_mod):
    rho = np.float32(0.1)
    G = np.eye(3, dtype=np.float32)
    G[0, 1] = G[1, 0] = rho                               # |g| == rho is a conflict (strict <)
    G[0, 2] = G[2, 0] = np.nextafter(rho, np.float32(0))  # just below: admissible
    assert oracle_mod.greedy_filter(G, rho).tolist() == [0, 2]
    G = np.eye(6, dtype=np.float32)
    assert oracle_mod.greedy_filter(G, rho, p_max=4).tolist() == [0, 1, 2, 3]
    assert oracle_mod.greedy_filter(G, rho, p_max=0).tolist() == [0, 1, 2, 3, 4, 5]
    # negative correlations count through the absolute value
    G = np.eye(2, dtype=np.float32)
    G[0, 1] = G[1, 0] = -0.5
    assert oracle_mod.greedy_filter(G, rho).tolist() == [0]
    assert oracle_mod.greedy_filter(np.zeros((0, 0), np.float32), rho).tolist() == []
