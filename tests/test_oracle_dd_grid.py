"""Pins of the oracle's grid-constrained data-derived codebook (oracle/dd.py: fit_grid, grid_cost):
the dynamic programme against exhaustive search over every subset (the problem's plain definition,
evaluated in exact rational arithmetic), exact-recovery and mirror cases, and the property the paper
gives as the reason for the construction (Section "Per-Layer Pair Search", step 1: selecting on the
grid costs no more than a free Lloyd fit followed by a snap to the grid)."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

from oracle import atoms as OA, dd as DD
import sop_inputs as si


def _exact_cost(hist, values):
    """Summed mass * squared distance to the nearest entry, in rational arithmetic."""
    H = len(hist)
    L = [Fraction(float(v)) for v in values]
    total = Fraction(0)
    for b, m in enumerate(hist):
        if m:
            x = Fraction(2 * b + 1 - H, H)
            total += int(m) * min((x - v) ** 2 for v in L)
    return total


@pytest.mark.parametrize("seed", range(8))
def test_dynamic_programme_equals_exhaustive_search(seed):
    rng = np.random.default_rng(100 + seed)
    H = int(rng.choice([16, 32, 48]))
    h = rng.integers(0, 1000, size=H)
    h[rng.random(H) < 0.3] = 0                                        # empty stretches
    nG = int(rng.integers(6, 11))
    cand = np.sort(np.round(rng.uniform(-1.1, 1.1, nG) * 64) / 64)    # some candidates outside the bins' span
    if np.unique(cand).size < nG:
        cand = np.unique(cand)
        nG = cand.size
    n = int(rng.integers(1, min(5, nG) + 1))
    idx, cost = DD.fit_grid(h, cand, n)
    assert idx.size == n and np.all(np.diff(idx) > 0) and 0 <= idx[0] and idx[-1] < nG
    exact = {s: _exact_cost(h, cand[list(s)]) for s in itertools.combinations(range(nG), n)}
    least = min(exact.values())
    assert exact[tuple(int(i) for i in idx)] == least                # an optimal subset (exactly, not to rounding)
    assert abs(cost - float(least)) <= 1e-12 * max(1.0, float(least))
    assert abs(DD.grid_cost(h, cand[idx]) - float(least)) <= 1e-12 * max(1.0, float(least))


def test_mass_on_grid_points_is_recovered_with_zero_cost():
    H = 64
    centres = DD.bin_centres(H)
    cand = centres[::4].copy()                                        # 16 candidates that are bin centres
    h = np.zeros(H, dtype=np.int64)
    keep = [0, 3, 4, 9, 15]
    for j in keep:
        h[4 * j] = 7 + j
    idx, cost = DD.fit_grid(h, cand, len(keep))
    assert cost == 0.0 and list(idx) == keep
    # one entry fewer must merge the cheapest neighbours: bins 3 and 4 (one candidate step apart, small masses)
    idx4, cost4 = DD.fit_grid(h, cand, 4)
    step = cand[1] - cand[0]
    assert abs(cost4 - min(10, 11) * step ** 2) < 1e-12 and (3 in idx4) != (4 in idx4)
    assert set(idx4) >= {0, 9, 15}


def test_single_entry_is_the_candidate_nearest_the_mean():
    rng = np.random.default_rng(7)
    h = rng.integers(0, 50, size=128)
    cand = np.linspace(-1, 1, 41)
    idx, cost = DD.fit_grid(h, cand, 1)
    mean = float((h * DD.bin_centres(128)).sum() / h.sum())
    assert idx[0] == int(np.argmin(np.abs(cand - mean)))              # squared error about a point grows with its distance from the mean
    assert abs(cost - DD.grid_cost(h, cand[idx])) <= 1e-9 * cost


def test_mirror_image():
    rng = np.random.default_rng(9)
    h = rng.integers(0, 1000, size=256)
    cand = np.sort(rng.uniform(-1, 1, 24))
    idx, cost = DD.fit_grid(h, cand, 6)
    idx_m, cost_m = DD.fit_grid(h[::-1].copy(), -cand[::-1], 6)
    assert abs(cost - cost_m) <= 1e-12 * cost and list(idx_m) == [23 - i for i in idx[::-1]]


def test_more_entries_never_cost_more_and_all_candidates_cost_the_snap():
    W = si.bf16_round(si.student_t_weights(32, 512, 4.0, 61))
    c = si.channel_norms(512, 1.0, 62)
    h = DD.histogram(W, c, 16, 256)
    cand = OA.exmy_grid(2, 3) / 7.5                                   # the 63 values of E2M3 on [-1, 1]
    costs = [DD.fit_grid(h, cand, n)[1] for n in (2, 4, 8, 16, 32, 63)]
    assert all(b <= a for a, b in zip(costs, costs[1:]))
    assert abs(costs[-1] - DD.grid_cost(h, cand)) <= 1e-9 * costs[-1]


@pytest.mark.parametrize("fmt", [(2, 3), (4, 3)])
def test_selection_on_the_grid_beats_free_fit_then_snap(fmt):
    """The paper's reason for the construction: a free Lloyd fit followed by a snap to the grid pays
    a displacement the grid-constrained selection does not."""
    W = si.bf16_round(si.student_t_weights(64, 1024, 4.0, 71, row_sigma=0.5))
    c = si.channel_norms(1024, 1.0, 72)
    h = DD.histogram(W, c, 16, 1024)
    grid = OA.exmy_grid(*fmt)
    cand = grid / np.abs(grid).max()
    free = DD.fit(h, 16, 20, OA.nf(4))
    snapped = np.unique(cand[np.abs(cand[None, :] - free[:, None]).argmin(axis=1)])
    idx, cost = DD.fit_grid(h, cand, 16)
    assert cost <= DD.grid_cost(h, snapped) * (1 + 1e-12)
    assert cost >= DD.grid_cost(h, free) * 0.5                        # and it is no miracle either
    L = cand[idx]
    assert L[0] < 0 < L[-1]                                           # usable as an atom
    # the end bins hold every block's largest element: the ends of the grid are taken
    assert L[0] == -1.0 and L[-1] == 1.0
