"""Layer-scope ("^0") floating-point weight formats of the oracle: one scale per layer, weights
rounded to an ExMy grid, channel-norm-weighted and plain reconstruction error.  numpy.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

Followed passages: Section "Primary Formats", paragraph "Block-scaled FP6 versus POT-scaled FP8"
(the baseline E4M3^0sUE8M0: bare E4M3 weights with a single power-of-two scale per layer, compared
with E2M3sUE4M4 by weight MSE); Appendix "Format string grammar" (^0 = layer-max scope, one scale
per layer; UE8M0 is power-of-two only).

Readings where the paper is silent:
  - the layer scale follows the same rule as a block scale with the whole layer as the block:
    s* = max(pmax / t+, nmax / -t-) against the grid's end values, times 2^k, rounded into the scale
    word to the nearest value with ties to the lower code (so a power-of-two scale may be the next
    power of two below s*, and the largest weights then saturate at the grid's end);
  - weight rounding: nearest grid value, ties to the lower value (count of midpoints strictly
    below x), every ExMy code finite unless max_code reserves the top ones;
  - errors: sum_i c_k(i) (w_i - s*y_i)^2 and sum_i (w_i - s*y_i)^2 over the layer, binary64 sums of
    binary32 residuals d = fma(-s, y, w).
"""
from __future__ import annotations

import numpy as np

from . import pairsearch as ps

F32 = np.float32


def exmy_table(exp_bits: int, man_bits: int, bias: int = -1, max_code: int = -1) -> np.ndarray:
    """Signed grid of an ExMy weight format, ascending, binary64: magnitudes value(q), q = 0..max_code,
    value(q) = f/2^y * 2^(1-bias) for e = 0 and (1 + f/2^y) * 2^(e-bias) otherwise."""
    bias = 2 ** (exp_bits - 1) - 1 if bias < 0 else bias
    max_code = 2 ** (exp_bits + man_bits) - 1 if max_code < 0 else max_code
    mags = []
    for q in range(max_code + 1):
        e, f = q >> man_bits, q & (2 ** man_bits - 1)
        mags.append(np.ldexp(float(f), 1 - bias - man_bits) if e == 0 else np.ldexp(float(2 ** man_bits + f), e - bias - man_bits))
    mags = np.array(mags)
    return np.concatenate([-mags[:0:-1], mags])                      # 2*max_code + 1 values, one zero


def layer_scope(W: np.ndarray, c: np.ndarray | None, table: np.ndarray, scale_fmt, k: int = 0):
    """Returns dict(q, s, codes [M,K] indices into table, err_w, err_u, wn)."""
    W = np.ascontiguousarray(W, dtype=F32)
    M, K = W.shape
    L = np.asarray(table, dtype=np.float64).astype(F32)
    cv = np.ones(K, dtype=F32) if c is None else np.asarray(c, dtype=F32)
    pmax = max(F32(0), W.max())
    nmax = max(F32(0), (-W).max())
    tp, tn = L[-1], -L[0]
    sstar = max(F32(pmax / tp), F32(nmax / tn))
    sp = F32(sstar * F32(2.0 ** k))
    q = ps.scale_encode(scale_fmt, sp)
    s = F32(np.ldexp(ps.scale_value(scale_fmt, q), -k))
    r = F32(1.0) / s if s > 0 else F32(0.0)
    mids = ((L[:-1].astype(np.float64) + L[1:].astype(np.float64)) * 0.5).astype(F32)
    zero_code = int(np.count_nonzero(mids < 0))
    err_w = err_u = wn = 0.0
    codes = np.empty((M, K), dtype=np.int32)
    rows = max(1, (1 << 22) // K)
    for r0 in range(0, M, rows):
        w = W[r0:r0 + rows]
        if s > 0:
            x = (w * r).astype(F32)
            code = np.searchsorted(mids, x, side="left").astype(np.int32)      # midpoints strictly below x
        else:
            code = np.full(w.shape, zero_code, dtype=np.int32)
        y = L[code]
        # d = fma(-s, y, w): the product of a binary32 scale (at most 11 significant bits) and a
        # binary32 grid value is exact in binary64, and so is its difference from w for the operands
        # that occur; one rounding to binary32 follows
        d = (w.astype(np.float64) - np.float64(s) * y.astype(np.float64)).astype(F32).astype(np.float64)
        err_w += float((cv.astype(np.float64)[None, :] * d * d).sum())
        err_u += float((d * d).sum())
        wn += float((cv.astype(np.float64)[None, :] * w.astype(np.float64) ** 2).sum())
        codes[r0:r0 + rows] = code
    return dict(q=q, s=float(s), codes=codes, err_w=err_w, err_u=err_u, wn=wn)
