"""CPU tests of the admission rule for kept sets that differ from the oracle's (tests/parity_rules.py).

Algorithm 1 constrains B_1 by |x_j^T x_k| < rho; a Gram entry within the Gram tolerance of rho may be
decided either way by fp32 and fp64 sums.  The rule must accept exactly the kept sets that follow from
such entries, and must not let an unrelated near-rho pair excuse a wrong decision elsewhere.  The
"other side" is played by the oracle's own greedy filter on a perturbed Gram, so every planted mistake
is planted on the CPU.
"""
import numpy as np
import pytest

from oracle import oracle as orc
from parity_rules import (GRAM_ATOL, GRAM_RTOL, check_kept_against_oracle, explain_kept_set, first_divergence,
                          rho_window)

RHO = np.float32(0.1)


def _base(L=40, seed=0, scale=0.03):
    rng = np.random.default_rng(seed)
    A = (rng.standard_normal((L, L)) * scale).astype(np.float32)
    G = np.triu(A, 1) + np.triu(A, 1).T + np.eye(L, dtype=np.float32)
    # keep every random entry clear of rho, so that only planted entries are near it
    far = np.abs(np.abs(G) - RHO) < 0.01
    np.fill_diagonal(far, False)
    G[far] = 0.0
    return G


def _set(G, a, b, v):
    G[a, b] = G[b, a] = np.float32(v)


def test_window_is_the_gram_tolerance_at_rho():
    assert rho_window(0.1) == pytest.approx(GRAM_RTOL * 0.1 + GRAM_ATOL)
    assert rho_window(0.1) > 5e-6          # an fp32 flip at distance 5e-6 is inside it


def test_a_pair_at_rho_minus_eps_decided_the_other_way_is_accepted_and_logged():
    G_ref = _base()
    _set(G_ref, 5, 2, RHO - np.float32(5e-6))           # the oracle: admissible
    G_gpu = G_ref.copy()
    _set(G_gpu, 5, 2, RHO + np.float32(5e-6))           # the other side: conflict
    kept_ref = orc.greedy_filter(G_ref, RHO, 0)
    kept_gpu = orc.greedy_filter(G_gpu, RHO, 0)
    assert 5 in kept_ref and 5 not in kept_gpu and 2 in kept_gpu
    assert first_divergence(kept_gpu, kept_ref) == 5
    log = []
    check_kept_against_oracle(G_ref, kept_gpu, kept_ref, RHO, 0, log, "t", G_gpu=G_gpu)
    assert [(e[2], e[3]) for e in log] == [(5, 2)]
    assert log[0][4] == pytest.approx(float(RHO) - 5e-6, abs=1e-7) and log[0][5] == pytest.approx(float(RHO) + 5e-6, abs=1e-7)
    # and the mirror image: the oracle sees the conflict, the other side does not
    log = []
    check_kept_against_oracle(G_gpu, kept_ref, kept_gpu, RHO, 0, log, "t")
    assert [(e[2], e[3]) for e in log] == [(5, 2)]


def test_an_unrelated_near_pair_does_not_excuse_a_wrong_decision():
    G_ref = _base()
    _set(G_ref, 5, 2, RHO - np.float32(5e-7))           # a near pair exists ...
    kept_ref = orc.greedy_filter(G_ref, RHO, 0)
    assert 30 in kept_ref
    # ... but the other side's mistake is elsewhere: it drops position 30, which conflicts with nothing
    kept_bad = kept_ref[kept_ref != 30]
    with pytest.raises(AssertionError, match="position 30 was rejected"):
        check_kept_against_oracle(G_ref, kept_bad, kept_ref, RHO, 0, [], "t")
    # or it keeps a position that has a plain conflict (0.5) with a kept one
    G2 = G_ref.copy()
    _set(G2, 20, 7, 0.5)
    kept_ref2 = orc.greedy_filter(G2, RHO, 0)
    assert 7 in kept_ref2 and 20 not in kept_ref2
    kept_bad2 = np.sort(np.append(kept_ref2, 20)).astype(np.int32)
    with pytest.raises(AssertionError, match="position 20 was kept"):
        check_kept_against_oracle(G2, kept_bad2, kept_ref2, RHO, 0, [], "t")


def test_a_flip_outside_the_window_is_rejected():
    for dist, ok in ((5e-6, True), (9e-6, True), (5e-5, False), (1e-3, False)):
        G_ref = _base(seed=3)
        _set(G_ref, 9, 4, float(RHO) - dist)
        G_gpu = G_ref.copy()
        _set(G_gpu, 9, 4, float(RHO) + dist)
        kept_ref, kept_gpu = orc.greedy_filter(G_ref, RHO, 0), orc.greedy_filter(G_gpu, RHO, 0)
        assert not np.array_equal(kept_ref, kept_gpu)
        if ok:
            check_kept_against_oracle(G_ref, kept_gpu, kept_ref, RHO, 0, [], "t")
        else:
            with pytest.raises(AssertionError):
                check_kept_against_oracle(G_ref, kept_gpu, kept_ref, RHO, 0, [], "t")


def test_what_follows_an_admissible_flip_may_differ_too():
    # position 6 is kept by one side only; position 12 conflicts (0.7) with 6 and with nothing else, so it is
    # kept exactly where 6 is not; position 18 conflicts with 12 ...
    G_ref = _base(seed=5)
    _set(G_ref, 6, 1, RHO + np.float32(4e-6))           # the oracle rejects 6
    _set(G_ref, 12, 6, 0.7)
    _set(G_ref, 18, 12, 0.7)
    G_gpu = G_ref.copy()
    _set(G_gpu, 6, 1, RHO - np.float32(4e-6))           # the other side keeps it
    kept_ref, kept_gpu = orc.greedy_filter(G_ref, RHO, 0), orc.greedy_filter(G_gpu, RHO, 0)
    assert {6, 18} <= set(kept_gpu) and 12 not in kept_gpu
    assert 12 in kept_ref and 6 not in kept_ref and 18 not in kept_ref
    log = []
    check_kept_against_oracle(G_ref, kept_gpu, kept_ref, RHO, 0, log, "t")
    assert [(e[2], e[3]) for e in log] == [(6, 1)]      # only the near entry is leaned on; the rest follows plainly


def test_cap_on_the_kept_set():
    G = _base(seed=7)
    kept = orc.greedy_filter(G, RHO, 9)
    assert len(kept) == 9
    assert explain_kept_set(G, kept, RHO, p_max=9) == []
    with pytest.raises(AssertionError):
        explain_kept_set(G, orc.greedy_filter(G, RHO, 0), RHO, p_max=9)          # more than the cap
    with pytest.raises(AssertionError):
        explain_kept_set(G, kept[:-1], RHO, p_max=9)                              # stopped early for no reason


@pytest.mark.parametrize("seed", range(8))
def test_random_perturbations_inside_the_tolerance_are_always_admitted(seed):
    rng = np.random.default_rng(seed)
    L = 120
    A = (rng.standard_normal((L, L)) * 0.06).astype(np.float32)
    G_ref = np.triu(A, 1) + np.triu(A, 1).T + np.eye(L, dtype=np.float32)
    # push a good number of entries right next to rho
    for _ in range(60):
        a, b = rng.integers(0, L, 2)
        if a != b:
            _set(G_ref, a, b, rng.choice([-1, 1]) * (float(RHO) + rng.uniform(-8e-6, 8e-6)))
    E = rng.uniform(-1, 1, (L, L)) * 0.9 * (GRAM_RTOL * np.abs(G_ref) + GRAM_ATOL)
    E = np.triu(E, 1) + np.triu(E, 1).T
    G_gpu = (G_ref.astype(np.float64) + E).astype(np.float32)
    kept_ref, kept_gpu = orc.greedy_filter(G_ref, RHO, 0), orc.greedy_filter(G_gpu, RHO, 0)
    log = []
    check_kept_against_oracle(G_ref, kept_gpu, kept_ref, RHO, 0, log, "t", G_gpu=G_gpu)
    if not np.array_equal(kept_ref, kept_gpu):
        assert log and all(abs(abs(e[4]) - float(RHO)) <= rho_window(RHO) for e in log)
    # the oracle's own kept set needs no entry of the window
    assert explain_kept_set(G_ref, kept_ref, RHO) == []
