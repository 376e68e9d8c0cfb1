"""Rules the GPU parity tests share (no arithmetic of the method: only what counts as agreement).

Gram entries from the fp32 matrix cores and from the oracle's fp64 sums agree to
GRAM_RTOL * |g| + GRAM_ATOL.  The greedy choice of B_1 compares |g| with rho, so an entry that close to
rho may fall on either side of it, and everything decided after such an entry may differ too.  A kept
set that is not the oracle's own is therefore admitted only if it is the greedy result for *some* Gram
inside that tolerance of the oracle's: every single decision of the walk (keep position a / reject it)
must be justified by the oracle's values of row a against the positions kept before a, and where a
decision needs the tolerance, the entries it leans on are named.
"""
import numpy as np

GRAM_RTOL, GRAM_ATOL = 1e-4, 1e-6


def rho_window(rho: float) -> float:
    """Half-width around rho inside which a Gram entry may be decided either way: the Gram tolerance at |g| = rho."""
    return GRAM_RTOL * float(rho) + GRAM_ATOL


def explain_row(a, g_row, kept_before, rho, kept_a, window):
    """One decision of the greedy walk against the oracle's values.  g_row: the oracle's Gram row of
    position a (indexable by position); kept_before: positions < a the GPU kept, increasing; kept_a: did
    the GPU keep a.  Returns the list of (a, b, g_ref) entries the decision leans on inside the window
    (empty if it is the oracle's own decision); raises AssertionError if no Gram inside the tolerance
    gives this decision."""
    rho = float(rho)
    kb = np.asarray(kept_before, dtype=np.int64)
    mag = np.abs(np.asarray(g_row, dtype=np.float64)[kb]) if kb.size else np.zeros(0)
    if kept_a:
        # every kept b must be admissible for a: |g| < rho, or inside the window above it
        bad = mag >= rho + window
        assert not bad.any(), (f"position {a} was kept although |g| = {mag[bad].max():.9g} with kept position "
                               f"{int(kb[bad][mag[bad].argmax()])} is above rho = {rho:.9g} by more than the window")
        lean = mag >= rho
    else:
        # some kept b must conflict with a: |g| >= rho, or inside the window below it
        strict = mag >= rho
        if strict.any():
            return []
        lean = mag >= rho - window
        assert lean.any(), (f"position {a} was rejected although its largest |g| with a kept position is "
                            f"{mag.max() if mag.size else 0.0:.9g}, below rho = {rho:.9g} by more than the window")
    return [(int(a), int(b), float(np.asarray(g_row)[b])) for b in kb[lean]]


def explain_kept_set(G_ref, kept_gpu, rho, p_max=0, window=None, n_cand=None):
    """The whole walk.  G_ref: the oracle's L x L Gram; kept_gpu: the GPU's kept positions (increasing).
    Returns the list of entries (a, b, g_ref) on which a decision needed the window (empty = the kept set
    is exactly the oracle's greedy set); raises AssertionError if the kept set is not admissible."""
    G_ref = np.asarray(G_ref)
    L = G_ref.shape[0] if n_cand is None else int(n_cand)
    window = rho_window(rho) if window is None else float(window)
    kept_gpu = np.asarray(kept_gpu, dtype=np.int64)
    assert np.all(np.diff(kept_gpu) > 0) and (kept_gpu.size == 0 or (0 <= kept_gpu[0] and kept_gpu[-1] < L))
    is_kept = np.zeros(L, bool)
    is_kept[kept_gpu] = True
    cap = int(p_max) if p_max and p_max > 0 else L
    assert kept_gpu.size <= cap, "more kept than the cap allows"
    leaned = []
    n_before = 0
    for a in range(L):
        if n_before >= cap:
            assert not is_kept[a:].any(), "a position was kept after the cap was reached"
            break
        leaned += explain_row(a, G_ref[a], kept_gpu[:n_before], rho, bool(is_kept[a]), window)
        n_before += int(is_kept[a])
    return leaned


def first_divergence(kept_a, kept_b):
    """First position that is in one kept list and not in the other (None if the lists are equal)."""
    sa, sb = set(int(v) for v in kept_a), set(int(v) for v in kept_b)
    d = sa ^ sb
    return min(d) if d else None


def check_kept_against_oracle(G_ref, kept_gpu, kept_ref, rho, p_max, log, tag, G_gpu=None):
    """kept_gpu must be kept_ref (the oracle's greedy set on G_ref) or an admissible variant of it; in
    the second case the first diverging position must itself lean on an entry inside the window, and
    every such entry is logged with both sides' values."""
    if np.array_equal(kept_gpu, kept_ref):
        return
    leaned = explain_kept_set(G_ref, kept_gpu, rho, p_max)
    a0 = first_divergence(kept_gpu, kept_ref)
    at_a0 = [e for e in leaned if e[0] == a0]
    assert at_a0, f"{tag}: kept sets first differ at position {a0}, where no Gram entry lies within the window of rho"
    for (a, b, g) in leaned:
        log.append(("near_rho", tag, a, b, g, None if G_gpu is None else float(G_gpu[a, b])))
