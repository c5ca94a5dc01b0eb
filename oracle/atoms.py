"""Codebook ("atom") builders and format arithmetic of the oracle (numpy / scipy, binary64).

TEST INFRASTRUCTURE ONLY; independent of the HIP library's own builders.

Followed passages: Section "Per-Layer Pair Search" (alphabet list: NF4 = Gaussian-quantile
inverse-CDF grid; BOF4 = Lloyd iteration on the per-block-max-normalised distribution; SH4 =
sinh grid; each atom and its sign negation are separate candidates), Section "Primary Formats"
(sinh companding g = sinh(alpha t) + c with alpha = 1.50, c = -0.02, t uniform on [-1, 1];
hosting ratio max(LUT)/min nonzero |LUT|), Section "Block Scaling" (bits per weight s/g + b; NF4
has equal endpoints, seven negative and eight positive entries).

Parity unpinned: bof() and lloyd_1d() (the paper gives one line for BOF4; only Lloyd's fixed-point
invariants are checked).
"""
from __future__ import annotations

import numpy as np
from scipy.stats import norm


def nf(n_bits: int) -> np.ndarray:
    """NormalFloat grid with 2^n entries: 2^(n-1) positive and 2^(n-1)-1 negative Gaussian
    quantiles plus an exact zero, normalised to [-1, 1].

    The outermost probability is the mean of 1 - 1/32 and 1 - 1/30 for every n (the n = 5 hosting
    ratio the paper prints, 25.2, is only reproduced with the n = 4 constant kept)."""
    npos = 2 ** (n_bits - 1)
    nneg = npos - 1
    delta = 0.5 * ((1.0 - 1.0 / 32.0) + (1.0 - 1.0 / 30.0))
    pos = norm.ppf(np.linspace(delta, 0.5, npos + 1)[:-1])
    neg = -norm.ppf(np.linspace(delta, 0.5, nneg + 1)[:-1])
    v = np.concatenate([neg, [0.0], pos])
    v = np.sort(v / np.max(np.abs(v)))
    return v


def sh(n_bits: int, alpha: float = 1.5, c: float = -0.02) -> np.ndarray:
    """Sinh grid: sinh(alpha t) + c on 2^n uniform t in [-1, 1], divided by the largest magnitude."""
    t = np.linspace(-1.0, 1.0, 2 ** n_bits)
    v = np.sinh(alpha * t) + c
    return np.sort(v / np.max(np.abs(v)))


def negate(L: np.ndarray) -> np.ndarray:
    """Sign-negated atom, re-sorted ascending."""
    return -np.asarray(L, dtype=np.float64)[::-1]


def lloyd_1d(samples: np.ndarray, weights: np.ndarray | None, init: np.ndarray, iters: int,
             pinned: np.ndarray | None = None) -> np.ndarray:
    """Weighted 1-D Lloyd iteration: assign each sample to its nearest centroid (ties to the lower
    one), move every non-pinned centroid to the weighted mean of its cell; empty cells stay."""
    x = np.asarray(samples, dtype=np.float64)
    w = np.ones_like(x) if weights is None else np.asarray(weights, dtype=np.float64)
    cent = np.sort(np.asarray(init, dtype=np.float64)).copy()
    pin = np.zeros(cent.size, dtype=bool) if pinned is None else np.asarray(pinned, dtype=bool)
    for _ in range(iters):
        mids = 0.5 * (cent[:-1] + cent[1:])
        cell = np.searchsorted(mids, x, side="left")        # count of midpoints strictly below x
        sw = np.bincount(cell, weights=w, minlength=cent.size)
        swx = np.bincount(cell, weights=w * x, minlength=cent.size)
        upd = (sw > 0) & ~pin
        cent[upd] = swx[upd] / sw[upd]
        cent = np.sort(cent)
    return cent


def block_normalise(draws: np.ndarray, g: int) -> np.ndarray:
    """Cut draws into blocks of g and divide each block by its signed absmax element, so that the
    largest-magnitude element of every block becomes +1."""
    b = np.asarray(draws, dtype=np.float64)
    b = b[: (b.size // g) * g].reshape(-1, g)
    idx = np.argmax(np.abs(b), axis=1)
    piv = b[np.arange(b.shape[0]), idx]
    return (b / piv[:, None]).reshape(-1)


def bof(n_bits: int, draws: np.ndarray, g: int = 16, iters: int = 50) -> np.ndarray:
    """Block-optimum-fitted grid: Lloyd on N(0,1) blocks normalised by their signed absmax,
    started from the NormalFloat grid; afterwards the endpoints are set to exactly -1 and +1 and
    the entry nearest zero to exactly 0."""
    x = block_normalise(draws, g)
    cent = lloyd_1d(x, None, nf(n_bits), iters)
    cent[0], cent[-1] = -1.0, 1.0
    cent[np.argmin(np.abs(cent))] = 0.0
    return np.sort(cent)


def exmy_magnitudes(x: int, y: int, bias: int | None = None, reserve_top: bool = False) -> np.ndarray:
    """All magnitudes of an ExMy floating-point grid with every code finite (subnormals included);
    reserve_top drops the top exponent."""
    bias = 2 ** (x - 1) - 1 if bias is None else bias
    vals = []
    emax = 2 ** x - (2 if reserve_top else 1)
    for e in range(0, emax + 1):
        for m in range(2 ** y):
            vals.append(m / 2 ** y * 2.0 ** (1 - bias) if e == 0 else (1 + m / 2 ** y) * 2.0 ** (e - bias))
    return np.array(sorted(set(vals)))


def exmy_grid(x: int, y: int, **kw) -> np.ndarray:
    """Signed ExMy grid (distinct values, ascending)."""
    m = exmy_magnitudes(x, y, **kw)
    return np.array(sorted(set(np.concatenate([-m, m]).tolist())))


def hosting_ratio(L: np.ndarray) -> float:
    """max|L| / min nonzero |L| (the dynamic range an LUT value format must host)."""
    a = np.abs(np.asarray(L, dtype=np.float64))
    return float(a.max() / a[a > 0].min())


def bits_per_weight(scale_bits: int, g: int, elem_bits: int) -> float:
    """Average storage: s/g + b."""
    return scale_bits / g + elem_bits


def to_f32(L: np.ndarray) -> np.ndarray:
    """Table as the kernels receive it: one rounding to binary32."""
    return np.asarray(L, dtype=np.float64).astype(np.float32)
