"""Host side of the grid-constrained data-derived codebook: the library's selection
(sop_dd_fit_grid, sop_weight_grid) against the oracle's dynamic programme and its plain cost."""
import ctypes as C

import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, dd as DD
import sop_inputs as si


def _same_selection(h, cand, n):
    idx, cost = sop.sop_dd_fit_grid(h, cand, n)
    ridx, rcost = DD.fit_grid(h, cand, n)
    # valid: ascending indices into cand; its cost, recomputed by the definition, is what it reports
    assert idx.size == n and np.all(np.diff(idx) > 0) and idx[0] >= 0 and idx[-1] < cand.size
    assert abs(DD.grid_cost(h, cand[idx]) - cost) <= 1e-11 * max(rcost, 1e-300)
    # optimal: the cost is the oracle's; the selection too unless two selections tie to rounding
    assert abs(cost - rcost) <= 1e-11 * max(rcost, 1e-300)
    return np.array_equal(idx, ridx)


@pytest.mark.parametrize("x,y,mc,top", [(2, 3, -1, 0.0), (2, 3, -1, 1.875), (4, 3, 0x7E, 0.0), (3, 2, -1, 0.0), (2, 1, -1, 0.0), (5, 2, -1, 1.75)])
def test_weight_grid_lists_the_formats_values(x, y, mc, top):
    mine = sop.sop_weight_grid(sop.WeightFmt(x, y, -1, mc), top)
    bias = 2 ** (x - 1) - 1
    codes = np.arange((mc if mc >= 0 else 2 ** (x + y) - 1) + 1)
    e, f = codes >> y, codes & (2 ** y - 1)
    mag = np.where(e == 0, f * 2.0 ** (1 - bias - y), (2 ** y + f) * 2.0 ** (e.astype(np.float64) - bias - y))
    if top > 0:
        mag = mag[mag <= top]
    ref = np.unique(np.concatenate([-mag, mag]))
    assert np.array_equal(mine, ref)
    if mc < 0 and top == 0.0:
        assert np.array_equal(mine, OA.exmy_grid(x, y))               # the oracle's own generator
    if (x, y, top) == (2, 3, 0.0):
        assert mine.size == 63 and mine[-1] == 7.5                    # the 63-value E2M3 grid of the paper


def test_selection_equals_the_oracle_on_layer_histograms():
    W = si.bf16_round(si.student_t_weights(64, 1024, 4.0, 81, row_sigma=0.5, outlier_frac=0.001))
    c = si.channel_norms(1024, 1.0, 82)
    same = 0
    cases = 0
    for H in (256, 1024, 4096):
        for cc in (c, None):
            h = DD.histogram(W, cc, 16, H)
            for grid in (OA.exmy_grid(2, 3), OA.exmy_grid(3, 3), OA.exmy_grid(4, 3)[::2]):
                cand = grid / np.abs(grid).max()
                for n in (4, 16, 32):
                    same += _same_selection(h, cand, n)
                    cases += 1
    assert same >= cases - 1                                          # ties to rounding are rare


def test_random_histograms_and_candidates():
    rng = np.random.default_rng(83)
    same = 0
    for trial in range(60):
        H = int(rng.choice([64, 128, 512]))
        if trial % 3 == 0:
            h = rng.integers(0, 1 << 40, size=H)                      # heavy masses: 128-bit prefix sums
        elif trial % 3 == 1:
            h = np.zeros(H, dtype=np.int64)
            h[rng.integers(0, H, size=12)] = rng.integers(1, 1000, size=12)   # few occupied bins
            h[0] += 5
            h[-1] += 5
        else:
            x = np.clip(rng.standard_t(3, size=3000) / 6, -1, 1)
            h = np.histogram(x, bins=H, range=(-1, 1))[0].astype(np.int64)
            h[0] += 50
            h[-1] += 50
        nG = int(rng.integers(8, 40))
        cand = np.unique(np.round(rng.uniform(-1.2, 1.2, nG) * 256) / 256)
        cand = np.unique(np.concatenate([cand, [-1.0, 1.0]]))
        n = int(rng.integers(2, min(cand.size, 12) + 1))
        same += _same_selection(h, cand, n)
    assert same >= 57


def test_bin_centres_on_midpoints_go_to_the_lower_value():
    # candidates at -0.5 and 0.5 + 1/32: the midpoint 1/64 is the centre of bin 32 of 64, which must
    # go to the lower value; the reported cost says which way it went
    H = 64
    h = np.zeros(H, dtype=np.int64)
    h[32] = 1000
    h[0] = h[63] = 1
    cand = np.array([-0.5, 0.5 + 1.0 / 32])
    idx, cost = sop.sop_dd_fit_grid(h, cand, 2)
    assert list(idx) == [0, 1]
    x = DD.bin_centres(H)
    assert cost == pytest.approx(1000 * (x[32] + 0.5) ** 2 + (x[0] + 0.5) ** 2 + (x[63] - cand[1]) ** 2, rel=1e-13)
    assert cost == pytest.approx(DD.fit_grid(h, cand, 2)[1], rel=1e-13)


def test_argument_errors():
    h = np.ones(64, dtype=np.int64)
    cand = np.linspace(-1, 1, 9)
    L = sop.lib()
    out = (C.c_int * 8)()
    hp, cp = h.ctypes.data, cand.ctypes.data
    assert L.sop_dd_fit_grid(None, 64, cp, 9, 4, out, None) == 1
    assert L.sop_dd_fit_grid(hp, 60, cp, 9, 4, out, None) == 1                      # bins: a power of two
    assert L.sop_dd_fit_grid(hp, 64, cp, 9, 1, out, None) == 1                      # an atom has two entries at least
    assert L.sop_dd_fit_grid(hp, 64, cp, 9, 10, out, None) == 1                     # more entries than candidates
    bad = cand.copy()
    bad[3] = bad[2]
    assert L.sop_dd_fit_grid(hp, 64, bad.ctypes.data, 9, 4, out, None) == 3         # not strictly ascending
    bad = cand.copy()
    bad[8] = np.nan
    assert L.sop_dd_fit_grid(hp, 64, bad.ctypes.data, 9, 4, out, None) == 3
    neg = h.copy()
    neg[5] = -1
    assert L.sop_dd_fit_grid(neg.ctypes.data, 64, cp, 9, 4, out, None) == 1
    one_sided = np.zeros(64, dtype=np.int64)
    one_sided[40:] = 3
    assert L.sop_dd_fit_grid(one_sided.ctypes.data, 64, cp, 9, 2, out, None) == 3   # cannot serve as an atom
    assert L.sop_dd_fit_grid(hp, 64, cp, 9, 4, out, None) == 0                      # cost may be NULL
    v = (C.c_double * 64)()
    n = C.c_int(0)
    assert L.sop_weight_grid(sop.WeightFmt(6, 6, -1, -1), 0.0, v, C.byref(n)) == 4  # x + y <= 10
    assert L.sop_weight_grid(sop.WeightFmt(2, 3, -1, -1), 0.0, None, C.byref(n)) == 1
    assert L.sop_weight_grid(sop.WeightFmt(2, 3, -1, -1), 1e-9, v, C.byref(n)) == 1  # nothing but zero left
