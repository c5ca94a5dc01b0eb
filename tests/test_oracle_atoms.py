"""Pins for the oracle's codebook builders and format arithmetic against values the paper prints."""
import numpy as np
import pytest

from conftest import load_golden
from oracle import atoms as A
import sop_inputs as si


def test_nf4_structure_and_ratio():
    g = load_golden("hosting_ratios.txt")
    L = A.nf(4)
    assert L.size == 16 and np.all(np.diff(L) > 0)
    assert (L < 0).sum() == g["NF4_negative_entries"] and (L > 0).sum() == g["NF4_positive_entries"]
    assert L[0] == -1.0 and L[-1] == 1.0 and 0.0 in L            # equal endpoints, exact zero
    assert round(A.hosting_ratio(L), 1) == g["NF4_ratio"]
    # not closed under negation: negating interior entries does not give entries
    assert not np.allclose(np.sort(-L), L)


def test_nf4_is_gaussian_quantile_grid():
    # independent statement of the construction: every non-zero entry, un-normalised, is a standard
    # normal quantile whose probabilities are evenly spaced on each side of 1/2
    from scipy.stats import norm
    L = A.nf(4)
    zmax = norm.ppf(0.5 * ((1 - 1 / 32) + (1 - 1 / 30)))
    p = norm.cdf(L * zmax)
    assert np.allclose(np.diff(p[8:]), np.diff(p[8:])[0], rtol=1e-9)      # 0.5 ... delta, 8 steps
    assert np.allclose(np.diff(p[:8]), np.diff(p[:8])[0], rtol=1e-9)      # 1-delta ... 0.5, 7 steps
    assert abs(p[7] - 0.5) < 1e-15


def test_nf5_ratio():
    g = load_golden("hosting_ratios.txt")
    L = A.nf(5)
    assert L.size == 32 and (L < 0).sum() == 15 and (L > 0).sum() == 16
    assert round(A.hosting_ratio(L), 1) == g["NF5_ratio"]


def test_sh_ratios_and_asymmetry():
    g = load_golden("hosting_ratios.txt")
    for n, key in ((4, "SH4_ratio"), (5, "SH5_ratio")):
        L = A.sh(n)
        assert L.size == 2 ** n and np.all(np.diff(L) > 0)
        assert round(A.hosting_ratio(L), 1) == g[key]
    L = A.sh(4)
    assert L[0] == -1.0 and abs(L[-1] - (np.sinh(1.5) - 0.02) / (np.sinh(1.5) + 0.02)) < 1e-15
    # un-normalised grid is exactly sinh(1.5 t) - 0.02 on uniform t
    t = np.arcsinh(L * (np.sinh(1.5) + 0.02) + 0.02) / 1.5
    assert np.allclose(np.diff(t), 2 / 15, rtol=1e-9)


def test_exmy_grids():
    g = load_golden("hosting_ratios.txt")
    e2m3 = A.exmy_grid(2, 3)
    assert e2m3.size == g["E2M3_distinct_values"]
    m = A.exmy_magnitudes(2, 3)
    normals = m[m >= 1.0]
    assert normals.max() / normals.min() == g["E2M3_normal_ratio"]
    assert m.max() / m[m > 0].min() == g["E2M3_subnormal_ratio"]
    assert round(A.exmy_magnitudes(2, 5, reserve_top=True).max(), 2) == g["E2M5_max"]


def test_hif_grid_counts():
    g = load_golden("hosting_ratios.txt")
    for shifts, nkey, rkey in ((4, "HIF7_values", "HIF7_ratio"), (5, "HIF8_values", "HIF8_ratio")):
        vals = sorted({c * 2 ** s for c in range(-16, 16) for s in range(shifts)})
        assert len(vals) == g[nkey]
        mags = [abs(v) for v in vals if v != 0]
        assert max(mags) / min(mags) >= g[rkey]      # 16*2^3 = 128 >= 120: ratio quoted on the normal range
        assert max(v for v in vals) == 15 * 2 ** (shifts - 1) == g[rkey]


def test_bpw_identity():
    for key, val in load_golden("bpw.txt").items():
        s, g_, b = (int(t) for t in key.split("_"))
        assert A.bits_per_weight(s, g_, b) == val


def test_metabit_count():
    for key, m in load_golden("scale_words.txt").items():
        _, b, w, x, y = key.split("_")
        assert int(b) - int(w) - int(x) - int(y) == m


def test_negate():
    L = A.sh(4)
    Ln = A.negate(L)
    assert np.all(np.diff(Ln) > 0) and Ln[0] == -L[-1] and Ln[-1] == 1.0
    assert np.array_equal(A.negate(Ln), L)


def test_lloyd_fixed_point_and_bof_invariants():
    draws = si.normal_draws(1 << 18, 77)
    x = A.block_normalise(draws, 16)
    assert np.isclose(x.reshape(-1, 16).max(axis=1), 1.0).all() and np.abs(x).max() == 1.0
    cent = A.lloyd_1d(x, None, A.nf(4), 200)
    # fixed point: each centroid is the mean of its cell
    mids = 0.5 * (cent[:-1] + cent[1:])
    cell = np.searchsorted(mids, x, side="left")
    means = np.bincount(cell, weights=x, minlength=16) / np.bincount(cell, minlength=16)
    assert np.allclose(cent, means, atol=2e-4)
    # Lloyd lowers the quantisation MSE of its own training set relative to the start grid
    def mse(c):
        m_ = 0.5 * (c[:-1] + c[1:])
        return np.mean((x - c[np.searchsorted(m_, x, side="left")]) ** 2)
    assert mse(cent) < mse(A.nf(4))
    L = A.bof(4, draws)
    assert L.size == 16 and np.all(np.diff(L) > 0) and L[0] == -1 and L[-1] == 1 and 0.0 in L
    # weighted Lloyd with weights = integer multiplicities equals unweighted Lloyd on repeated samples
    xs = x[:4096]
    wts = (np.arange(xs.size) % 3 + 1).astype(float)
    a = A.lloyd_1d(xs, wts, A.nf(4), 5)
    b = A.lloyd_1d(np.repeat(xs, wts.astype(int)), None, A.nf(4), 5)
    assert np.allclose(a, b, atol=1e-12)


def test_lloyd_on_cases_the_mathematics_fixes():
    # (1) Uniform mass on [0,1): the optimal n-level quantiser of a uniform density has equally spaced
    #     levels (2j+1)/(2n) (the Lloyd-Max conditions: each level is its cell's mean, each boundary the
    #     midpoint of its levels).  A fine regular grid of samples stands for the density; the fixed point
    #     is then exact up to the grid's spacing.
    n, N = 8, 1 << 16
    x = (np.arange(N) + 0.5) / N
    start = np.sort(np.random.default_rng(3).uniform(0, 1, n))
    cent = A.lloyd_1d(x, None, start, 4000)
    assert np.max(np.abs(cent - (2 * np.arange(n) + 1) / (2 * n))) < 2e-4
    # (2) Point masses: with as many centroids as distinct points, each centroid ends on a point (zero
    #     distortion is reachable and is a fixed point); with weights, a centroid shared by two points
    #     sits at their weighted mean.
    pts = np.array([-3.0, -1.0, 0.5, 2.0])
    xs = np.repeat(pts, [5, 1, 7, 2])
    cent = A.lloyd_1d(xs, None, np.array([-2.5, -0.5, 0.4, 1.0]), 3)
    assert np.array_equal(cent, pts)
    cent = A.lloyd_1d(np.array([0.0, 1.0, 10.0]), np.array([3.0, 1.0, 2.0]), np.array([0.2, 9.0]), 5)
    assert np.array_equal(cent, np.array([0.25, 10.0]))               # (3*0 + 1*1) / 4, and the lone point
    # (3) one step, by hand: samples 0,1,2,3 with centroids (0.4, 2.1): midpoint 1.25 -> cells {0,1} and
    #     {2,3} -> (0.5, 2.5); a sample on a midpoint goes to the lower centroid
    assert np.array_equal(A.lloyd_1d(np.arange(4.0), None, np.array([0.4, 2.1]), 1), np.array([0.5, 2.5]))
    assert np.array_equal(A.lloyd_1d(np.array([0.0, 1.0, 2.0]), None, np.array([0.0, 2.0]), 1), np.array([0.5, 2.0]))
    # (4) an empty cell keeps its centroid
    assert np.array_equal(A.lloyd_1d(np.array([0.0, 0.1]), None, np.array([0.0, 5.0]), 2), np.array([0.05, 5.0]))


def test_block_normalise_hand_worked():
    # blocks of 4: (1, -2, 0.5, 1.5) has signed absmax -2 -> (-0.5, 1, -0.25, -0.75);
    #              (3, 1, -1, 0) has signed absmax 3 -> (1, 1/3, -1/3, 0); the trailing partial block is dropped
    x = A.block_normalise(np.array([1, -2, 0.5, 1.5, 3, 1, -1, 0, 9, 9], dtype=np.float64), 4)
    assert np.array_equal(x, np.array([-0.5, 1, -0.25, -0.75, 1, 1 / 3, -1 / 3, 0]))
    # every block holds +1 exactly once it has a unique largest magnitude, and nothing exceeds 1
    d = si.normal_draws(1 << 12, 5)
    xb = A.block_normalise(d, 16).reshape(-1, 16)
    assert np.all(xb.max(axis=1) == 1.0) and np.all(np.abs(xb) <= 1.0)


def test_midpoint_is_the_sum_of_the_halves():
    """A code boundary is the binary64 mean of two neighbouring entries rounded once to binary32 (the oracle's definition).
    It equals the binary32 sum of the entries' halves, which is how the GPU kernels form it: both are one rounding of
    the same real number, because the binary64 mean is exact whenever its low bits can change the binary32 result.
    Checked on random pairs of every relative magnitude, on neighbours in the last place and around powers of two."""
    rng = np.random.default_rng(5)
    n = 400000
    a = (rng.standard_normal(n) * np.exp2(rng.integers(-40, 40, n))).astype(np.float32)
    b = (rng.standard_normal(n) * np.exp2(rng.integers(-40, 40, n))).astype(np.float32)
    # pairs a few units in the last place apart, and pairs straddling a power of two
    c = np.nextafter(a, np.float32(np.inf), dtype=np.float32)
    for k in range(3): c = np.nextafter(c, np.float32(np.inf), dtype=np.float32)
    p2 = np.exp2(rng.integers(-30, 30, n)).astype(np.float32)
    lo = np.nextafter(p2, np.float32(0), dtype=np.float32)
    hi = np.nextafter(p2, np.float32(np.inf), dtype=np.float32)
    for x, y in ((a, b), (a, c), (lo, hi), (lo, p2), (-a, b), (a, np.float32(2.0 ** -31) * b)):
        mid = ((x.astype(np.float64) + y.astype(np.float64)) * 0.5).astype(np.float32)
        half = np.float32(0.5)
        summed = (half * x) + (half * y)                       # binary32 throughout
        assert summed.dtype == np.float32 and np.array_equal(mid.view(np.uint32), summed.view(np.uint32))
