"""Pins of the oracle's per-layer scale shift (oracle/flayer.py)."""
import numpy as np
import pytest

from oracle import flayer as FL, pairsearch as ps, atoms as OA
import sop_inputs as si


def test_format_range_landmarks():
    # UE4M4: smallest normal 2^-6, largest value 496 (the landmarks the scale codec tests also pin)
    lo, hi, bias, mc = FL.format_range(4, 4)
    assert (lo, hi, bias, mc) == (2.0 ** -6, 496.0, 7, 255)
    lo, hi, _, _ = FL.format_range(4, 3)                             # E4M3 magnitudes
    assert (lo, hi) == (2.0 ** -6, 480.0)
    lo, hi, _, _ = FL.format_range(5, 6)
    assert lo == 2.0 ** -14 and hi == (2 - 2.0 ** -6) * 2.0 ** 16
    f = ps.make_fmt(0, 4, 4)
    assert ps.scale_value(f, 255) == 496.0 and ps.scale_value(f, 16) == 2.0 ** -6   # same numbers from the codec


def test_in_capacity_layer_gets_zero_shift():
    # the paper: scales that fit the normal range without a shift give k* = 0 (a no-op)
    rng = np.random.default_rng(1)
    sc = np.exp(rng.uniform(np.log(2.0 ** -5), np.log(400.0), size=4096)).astype(np.float32)
    k, frac = FL.layer_shift(sc, 4, 4)
    assert k == 0 and frac == 1.0


def test_shift_centres_small_scales_and_breaks_ties_towards_zero():
    sc = np.full(1000, 2.0 ** -9, dtype=np.float32)
    # UE4M4 normal range [2^-6, 496]: k = 3 .. 17 all reach every block; the smallest |k| wins
    k, frac = FL.layer_shift(sc, 4, 4)
    assert (k, frac) == (3, 1.0)
    k, frac = FL.layer_shift(np.full(10, 2.0 ** 12, dtype=np.float32), 4, 4)
    assert (k, frac) == (-4, 1.0)                                     # 2^12 * 2^-4 = 256 <= 496 < 512
    # a symmetric choice: +1 and -1 equally good -> the non-negative one
    sc = np.array([2.0 ** -7] * 5 + [600.0] * 5, dtype=np.float32)    # k=+1 rescues the low half, k=-1 the high half
    k, frac = FL.layer_shift(sc, 4, 4)
    assert (k, frac) == (1, 0.5)
    assert FL.fraction_in_range(sc, -1, *FL.format_range(4, 4)[:2]) == 0.5


def test_zero_scales_count_in_the_denominator_only():
    sc = np.array([0.0, 0.0, 2.0 ** -8, 2.0 ** -8], dtype=np.float32)
    k, frac = FL.layer_shift(sc, 4, 4)
    assert (k, frac) == (2, 0.5)


def test_wide_exponent_formats_need_no_shift_narrow_ones_do():
    # the paper: mean k* is about zero for 5-exponent-bit formats and several units for 4-exponent-bit
    # formats on real layers; LLM-like weight magnitudes (block scales around 2^-6 .. 2^-3) show the same split
    W = si.bf16_round(si.student_t_weights(64, 2048, 4.0, 7, row_sigma=0.5, scale=0.02))
    sc = FL.block_scales(W, 16, 1.0, 1.0)
    k5, f5 = FL.layer_shift(sc, 5, 6)
    k4, f4 = FL.layer_shift(sc, 4, 4)
    assert k5 == 0 and f5 > 0.999
    assert k4 >= 1 and f4 > FL.fraction_in_range(sc, 0, *FL.format_range(4, 4)[:2])


def test_block_scales_follow_the_two_sided_absmax_rule():
    W = np.array([[0.5, -1.0, 0.25, 0.0, 0.98139, -0.1, 0.0, 0.0]], dtype=np.float32)
    sc = FL.block_scales(W, 4, 0.98139, 1.0)                          # a sinh-grid-like atom: t+ = 0.98139, t- = -1
    assert sc[0] == np.float32(1.0)                                   # max(0.5/0.98139, 1.0/1) = 1
    assert sc[1] == np.float32(np.float32(0.98139) / np.float32(0.98139))
    # agrees with the scale the pair search rounds: representable scales are found again
    L = np.array([-1.0, -0.5, 0.0, 0.5, 0.98139], dtype=np.float32)
    f = ps.make_fmt(0, 5, 10)                                         # binary16-like magnitudes: 1.0 is a code
    r = ps.pair_search(np.tile(W, (1, 2)), np.ones(16, dtype=np.float32), [L], 4, f)
    assert ps.scale_value(f, int(r.scale_code[0][0])) == 1.0
