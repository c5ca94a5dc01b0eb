"""Per-layer scale shift ("F_layer") of the oracle.  numpy, binary64 / exact.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

Followed passage: Section "Scale Format and Metabit Allocation", paragraph "Per-layer scale shift":
the per-block scale magnitudes sc_p = |w|max,p / LUT_max of a layer are multiplied by 2^k before
they are rounded into the scale word, and k* is the integer that maximises the fraction of block
scales landing in the scale format's normal range; in-capacity layers get k* = 0.

Readings where the paper is silent:
  - sc_p is the ideal scale of the absmax rule against the codebook's two endpoints,
    max(pmax / t+, nmax / -t-), each quotient one binary32 division (as in the pair search);
  - "normal range" = [2^(1-bias), value(max_code)], both ends included; zero scales are in no range
    but count in the denominator;
  - candidates are -64 <= k <= 64 restricted to the shifts the pair search accepts for the format
    (every scale value, its subnormal quantum and its reciprocal stay normal binary32 numbers);
  - ties: the smallest |k| wins, then the non-negative one.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


def block_scales(W: np.ndarray, g: int, t_pos: float, t_neg: float) -> np.ndarray:
    """sc_p of every block, binary32: max(pmax / t+, nmax / t-) with t- given as a magnitude."""
    W = np.ascontiguousarray(W, dtype=F32)
    M, K = W.shape
    blk = W.reshape(M, K // g, g)
    pmax = np.maximum(blk.max(axis=2), F32(0))
    nmax = np.maximum((-blk).max(axis=2), F32(0))
    return np.maximum((pmax / F32(t_pos)).astype(F32), (nmax / F32(t_neg)).astype(F32)).reshape(-1)


def format_range(exp_bits: int, man_bits: int, bias: int = -1, max_code: int = -1):
    """(smallest normal value, largest value) of the scale word's magnitudes, binary64 (exact)."""
    bias = 2 ** (exp_bits - 1) - 1 if bias < 0 else bias
    max_code = 2 ** (exp_bits + man_bits) - 1 if max_code < 0 else max_code
    e, f = max_code >> man_bits, max_code & (2 ** man_bits - 1)
    vmax = (f / 2 ** man_bits) * 2.0 ** (1 - bias) if e == 0 else (1 + f / 2 ** man_bits) * 2.0 ** (e - bias)
    return 2.0 ** (1 - bias), vmax, bias, max_code


def valid_shifts(exp_bits: int, man_bits: int, bias: int = -1, max_code: int = -1):
    """Shifts k within [-64, 64] for which every scale value * 2^-k, the subnormal quantum and every
    reciprocal are normal binary32 numbers."""
    _, _, bias, max_code = format_range(exp_bits, man_bits, bias, max_code)
    emax = max(max_code >> man_bits, 1)
    return [k for k in range(-64, 65)
            if 1 - bias - man_bits - k >= -126 and 1 - bias - k <= 126 and emax - bias - k <= 125]


def fraction_in_range(sc: np.ndarray, k: int, lo: float, hi: float) -> float:
    """Fraction of block scales with lo <= sc * 2^k <= hi (exact: ldexp in binary64)."""
    s = np.ldexp(np.asarray(sc, dtype=np.float64), k)
    return float(np.count_nonzero((s >= lo) & (s <= hi))) / s.size


def layer_shift(sc: np.ndarray, exp_bits: int, man_bits: int, bias: int = -1, max_code: int = -1):
    """k* and the fraction it reaches, by trying every admissible k (the definition)."""
    lo, hi, _, _ = format_range(exp_bits, man_bits, bias, max_code)
    best_k, best_count = None, -1
    s64 = np.asarray(sc, dtype=np.float64)
    for k in sorted(valid_shifts(exp_bits, man_bits, bias, max_code), key=lambda k: (abs(k), k < 0)):
        s = np.ldexp(s64, k)
        count = int(np.count_nonzero((s >= lo) & (s <= hi)))
        if count > best_count:                                       # earlier candidates win ties
            best_k, best_count = k, count
    return best_k, best_count / s64.size


def exponent_histogram(sc: np.ndarray, exp_bits: int, man_bits: int, bias: int = -1, max_code: int = -1) -> np.ndarray:
    """[2, 320] int64: row 0 counts the block scales by binary exponent e (sc = m * 2^e, 1/2 <= m < 1,
    index e + 160); row 1 counts those whose m exceeds the m of the format's largest value."""
    _, hi, _, _ = format_range(exp_bits, man_bits, bias, max_code)
    mv, _ = np.frexp(F32(hi))
    m, e = np.frexp(np.asarray(sc, dtype=F32))
    live = np.asarray(sc) > 0
    h = np.zeros((2, 320), dtype=np.int64)
    np.add.at(h[0], e[live] + 160, 1)
    np.add.at(h[1], e[live & (m > mv)] + 160, 1)
    return h
