"""Pins for the oracle's candidate draw (Step 1 of SAP): the draw order must follow
successive sampling without replacement with weights w_j = dbeta_j^2 + eta."""
import itertools

import numpy as np


def _draws(o, dbeta, eta, l_prime, rounds, seed=7):
    out = np.empty((rounds, l_prime), np.int32)
    for t in range(rounds):
        out[t] = o.draw(o.priority_keys(dbeta, eta, seed, t), l_prime)
    return out


def test_first_and_second_draw_probabilities(oracle_mod):
    dbeta = np.array([0.5, 1.0, 0.25, 2.0, 0.1], np.float32)
    eta = 1e-2
    w = dbeta.astype(np.float64) ** 2 + eta
    W = w.sum()
    R = 60000
    d = _draws(oracle_mod, dbeta, eta, 2, R)
    # P(first = a) = w_a / W
    cnt = np.bincount(d[:, 0], minlength=5)
    exp = R * w / W
    chi2 = ((cnt - exp) ** 2 / exp).sum()
    assert chi2 < 30.0, (chi2, cnt, exp)          # 4 dof, 1e-5 tail ~ 28.5
    # P(first = a, second = b) = w_a/W * w_b/(W - w_a)
    chi2 = 0.0
    for a, b in itertools.permutations(range(5), 2):
        e = R * w[a] / W * w[b] / (W - w[a])
        c = int(((d[:, 0] == a) & (d[:, 1] == b)).sum())
        chi2 += (c - e) ** 2 / e
    assert chi2 < 60.0, chi2                       # 19 dof, 1e-5 tail ~ 55


def test_square_not_linear_weight(oracle_mod):
    # Theorem 1's weight is the square of delta beta: with dbeta = (1, 3) and negligible eta the
    # first draw is coordinate 1 with probability 9/10 (a linear weight would give 3/4).
    d = _draws(oracle_mod, np.array([1.0, 3.0], np.float32), 1e-9, 1, 40000, seed=3)
    frac = (d[:, 0] == 1).mean()
    assert abs(frac - 0.9) < 0.01


def test_equal_weights_give_uniform_subsets(oracle_mod):
    J, L, R = 6, 3, 40000
    d = _draws(oracle_mod, np.full(J, 0.3, np.float32), 1e-6, L, R, seed=1)
    assert all(len(set(row)) == L for row in d[:2000])
    subsets = {}
    for row in d:
        key = tuple(sorted(row))
        subsets[key] = subsets.get(key, 0) + 1
    assert len(subsets) == 20
    exp = R / 20
    chi2 = sum((c - exp) ** 2 / exp for c in subsets.values())
    assert chi2 < 60.0                             # 19 dof


def test_order_is_descending_key_then_index(oracle_mod):
    keys = np.array([1.0, 5.0, 5.0, -2.0, 7.0, 5.0, 0.0], np.float32)
    assert oracle_mod.draw(keys, 5).tolist() == [4, 1, 2, 5, 0]
    assert oracle_mod.draw(keys, 100).tolist() == [4, 1, 2, 5, 0, 6, 3]   # P' clamped to J
    assert oracle_mod.draw(keys, 0).tolist() == []


def test_deterministic_in_seed_round(oracle_mod):
    db = np.abs(np.random.default_rng(0).normal(size=300)).astype(np.float32)
    a = oracle_mod.draw(oracle_mod.priority_keys(db, 1e-6, 5, 9), 40)
    b = oracle_mod.draw(oracle_mod.priority_keys(db, 1e-6, 5, 9), 40)
    c = oracle_mod.draw(oracle_mod.priority_keys(db, 1e-6, 5, 10), 40)
    assert a.tolist() == b.tolist() and a.tolist() != c.tolist()


def test_untouched_coordinates_outrank_touched_ones(oracle_mod):
    # Algorithm 1 starts every coordinate with delta beta = C (very large), so until every
    # coordinate has been visited the draw is a sweep over the unvisited ones.
    J, L = 1000, 100
    db = np.full(J, 1e6, np.float32)
    db[:600] = np.abs(np.random.default_rng(1).normal(size=600)).astype(np.float32)   # visited
    for t in range(5):
        cand = oracle_mod.draw(oracle_mod.priority_keys(db, 1e-6, 0, t), L)
        assert cand.min() >= 600
