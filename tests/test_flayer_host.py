"""Host side of the library's per-layer scale shift (sop_layer_shift on an exponent histogram)
against the oracle's brute force over every shift."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import flayer as FL


@pytest.mark.parametrize("x,y,mc", [(4, 4, -1), (4, 3, 0x7E), (5, 7, -1), (8, 7, 244 * 128 + 127)])
def test_histogram_route_equals_the_definition(x, y, mc):
    # the library decides from a histogram of binary exponents (plus a count of mantissas above the
    # format's top mantissa); the oracle's brute force over k is the definition
    rng = np.random.default_rng(x * 10 + y)
    bias = 119 if x == 8 else -1
    sc = np.exp(rng.normal(-4.0, 3.0, size=5000)).astype(np.float32)
    sc[:50] = 0.0
    lo, hi, _, _ = FL.format_range(x, y, bias, mc)
    sc[50:80] = np.float32(hi) * np.float32(2.0) ** rng.integers(-20, 3, size=30)       # exactly on the top value
    sc[80:110] = np.nextafter(np.float32(hi), np.float32(np.inf)) * np.float32(2.0) ** rng.integers(-20, 3, size=30)
    sc[110:140] = np.float32(lo) * np.float32(2.0) ** rng.integers(-10, 10, size=30)    # exactly on the bottom value
    sc[140:150] = np.float32(1e-42)                                   # binary32 subnormals
    k_ref, f_ref = FL.layer_shift(sc, x, y, bias, mc)
    h = FL.exponent_histogram(sc, x, y, bias, mc)
    k, frac = sop.sop_layer_shift(h, sc.size, sop.ScaleFmt(0, x, y, 16, bias, mc))
    assert (k, frac) == (k_ref, f_ref)
