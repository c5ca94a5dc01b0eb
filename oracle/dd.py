"""Data-derived codebook ("DD" atom) of the oracle: weighted histogram of block-normalised weights
and the weighted Lloyd fit on it.  numpy, plain loops for the small-case variant.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

Followed passages: Section "Per-Layer Pair Search", steps 1 and 3 (a data-adaptive atom is built
per layer from a histogram of the layer's weights by cluster selection) and design axis (iii)
(the Lloyd updates are uniform or channel-norm weighted); the alphabet list (DD4: data-derived
grid trained per layer).  The paper gives no recipe beyond that; the reading taken here:
  - every block of g weights is normalised by its largest magnitude, x = w / max|w|, so that x
    lies in [-1, 1] whatever the block's scale (the codebooks are used on scaled weights);
  - weight i counts with its channel norm c_i (or 1);
  - the samples are collected into a histogram of H uniform bins over [-1, 1] (the paper builds
    its data-adaptive atoms from a histogram), each bin holding the summed weight of its samples as
    an exact integer (units of 2^-20 max(c)), every binary32 operation rounded once;
  - Lloyd on the histogram: a bin stands for its centre; it goes, whole, to the cell of that
    centre, and a cell's entry moves to the weighted mean of its bins' centres; number of entries,
    start grid and number of rounds are given by the caller.
Parity unpinned for the choice of recipe (the paper prints no DD4 table); the arithmetic of the
recipe is pinned against scikit-learn's weighted k-means on the raw samples, against the plain
Lloyd iteration of oracle/atoms.py and by exact-recovery cases (tests/test_oracle_dd.py).

Grid-constrained construction (Section "Per-Layer Pair Search", step 1: a data-adaptive codebook
is selected from the grid points of the deployed LUT value format by a dynamic programme on the
histogram, so that no snap-to-grid displacement is paid afterwards): fit_grid() below.  The problem
has a plain definition, which grid_cost() writes out: among all ways to pick n_entries of the given
candidate values, the one whose nearest-entry quantisation of the histogram (a bin stands for its
centre) has the least summed mass * squared distance.  Pinned by exhaustive search over all
subsets on small cases and by the comparison with "free Lloyd fit, then snap to the grid".
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


def histogram(W: np.ndarray, c: np.ndarray | None, g: int, n_bins: int, block_mask: np.ndarray | None = None) -> np.ndarray:
    """[H] int64: summed integer weights of the samples of every bin.  block_mask ([M*K/g], non-zero =
    take the block) restricts the samples to a pool of blocks (step 3 of the pair search fits the
    second codebook on the blocks the first one serves worst)."""
    W = np.ascontiguousarray(W, dtype=F32)
    M, K = W.shape
    assert K % g == 0
    cv = np.ones(K, dtype=F32) if c is None else np.ascontiguousarray(c, dtype=F32)
    cmax = cv.max()
    cs = F32(1048576.0) / cmax if cmax > 0 else F32(0.0)             # binary32 division
    mass_col = np.rint((cv * cs).astype(F32)).astype(np.int64)       # rint(fl(c * cs)), half to even
    half = F32(0.5 * n_bins)
    hist = np.zeros(n_bins, dtype=np.int64)
    rows = max(1, (1 << 22) // K)
    for r0 in range(0, M, rows):                                     # chunks bound the temporaries
        blk = W[r0:r0 + rows].reshape(-1, K // g, g)
        a = np.abs(blk).max(axis=2)                                  # exact
        live = a > 0
        if block_mask is not None:
            live &= np.asarray(block_mask).reshape(M, K // g)[r0:r0 + rows] != 0
        r = np.zeros_like(a)
        r[live] = F32(1.0) / a[live]                                 # fl(1 / a)
        x = (blk * r[:, :, None]).astype(F32)                        # fl(w * r)
        b = np.floor(((x * half).astype(F32) + half).astype(F32)).astype(np.int64)
        b = np.clip(b, 0, n_bins - 1)
        sel = np.broadcast_to(live[:, :, None], x.shape)
        mass = np.broadcast_to(mass_col.reshape(1, K // g, g), x.shape)
        np.add.at(hist, b[sel], mass[sel])
    return hist


def histogram_loops(W: np.ndarray, c: np.ndarray | None, g: int, n_bins: int) -> np.ndarray:
    """The same histogram, one weight at a time with Python integers (tiny inputs only)."""
    W = np.ascontiguousarray(W, dtype=F32)
    M, K = W.shape
    cv = [F32(1.0)] * K if c is None else [F32(v) for v in c]
    cmax = max(cv)
    cs = F32(1048576.0) / cmax if cmax > 0 else F32(0.0)
    half = F32(0.5 * n_bins)
    mass = [0] * n_bins
    for m in range(M):
        for j in range(K // g):
            w = [F32(v) for v in W[m, j * g:(j + 1) * g]]
            a = max(abs(v) for v in w)
            if not a > 0:
                continue
            r = F32(1.0) / a
            for i, wi in enumerate(w):
                x = F32(wi * r)
                b = int(np.floor(F32(F32(x * half) + half)))
                b = min(max(b, 0), n_bins - 1)
                mass[b] += int(np.rint(F32(cv[j * g + i] * cs)))
    return np.array(mass, dtype=np.int64)


def fit(hist: np.ndarray, n_entries: int, iters: int, init: np.ndarray) -> np.ndarray:
    """Weighted Lloyd rounds on the histogram, binary64; returns the ascending grid (float64).
    Bin b stands for its centre -1 + (2b+1)/H; a cell's mean is formed from exact integer sums."""
    h = [int(v) for v in np.asarray(hist, dtype=np.int64).reshape(-1)]
    H = len(h)
    cent = np.array(init, dtype=np.float64).copy()
    assert cent.size == n_entries and np.all(np.diff(cent) > 0)
    centres = -1.0 + (2.0 * np.arange(H, dtype=np.float64) + 1.0) / H
    for _ in range(iters):
        mids = 0.5 * (cent[:-1] + cent[1:])
        cell = np.searchsorted(mids, centres, side="left")           # midpoints strictly below the centre
        for j in range(n_entries):
            bins = np.flatnonzero(cell == j)
            mass = sum(h[b] for b in bins)
            if mass > 0:
                first = sum(h[b] * (2 * int(b) + 1) for b in bins)    # exact
                cent[j] = (float(first) / float(mass)) / H - 1.0
        cent = np.sort(cent)
    return cent


def samples(W: np.ndarray, c: np.ndarray | None, g: int):
    """Raw samples behind the histogram: (x, weight) of every weight of a non-zero block, in
    binary64 from the binary32 x (for checks against sample-based clustering)."""
    W = np.ascontiguousarray(W, dtype=F32)
    M, K = W.shape
    blk = W.reshape(M, K // g, g)
    a = np.abs(blk).max(axis=2)
    live = a > 0
    r = np.zeros_like(a)
    r[live] = F32(1.0) / a[live]
    x = (blk * r[:, :, None]).astype(F32)
    cv = np.ones(K, dtype=F32) if c is None else np.asarray(c, dtype=F32)
    wt = np.broadcast_to(cv.reshape(1, K // g, g), x.shape)
    sel = np.broadcast_to(live[:, :, None], x.shape)
    return x[sel].astype(np.float64), wt[sel].astype(np.float64)


def bin_centres(n_bins: int) -> np.ndarray:
    """Centre of bin b of the histogram over [-1, 1]: -1 + (2b+1)/H."""
    return -1.0 + (2.0 * np.arange(n_bins, dtype=np.float64) + 1.0) / n_bins


def grid_cost(hist: np.ndarray, values: np.ndarray) -> float:
    """Distortion of a codebook on the histogram, by definition: every bin goes, whole, to the entry
    nearest its centre (ties to the lower entry, which does not change the sum), and pays its mass
    times the squared distance.  Units: histogram mass times squared domain units."""
    h = np.asarray(hist, dtype=np.float64).reshape(-1)
    x = bin_centres(h.size)
    L = np.sort(np.asarray(values, dtype=np.float64).reshape(-1))
    d2 = (x[:, None] - L[None, :]) ** 2
    return float((h * d2.min(axis=1)).sum())


def fit_grid(hist: np.ndarray, cand: np.ndarray, n_entries: int):
    """Best n_entries-subset of the ascending candidate values `cand` for the histogram:
    returns (indices into cand, ascending; distortion as grid_cost() defines it).

    Dynamic programme over "the k-th chosen entry is candidate c".  With entries chosen in ascending
    order, the bins at or below the first entry pay to the first entry, the bins above the last pay to
    the last, and the bins between two neighbouring chosen entries a < b pay to the nearer one (centre
    <= (a+b)/2: the lower).  Hence
        best[1][c] = below(c),   best[k][c] = min over c' < c of best[k-1][c'] + between(c', c),
        answer     = min over c of best[n][c] + above(c),
    every term a plain sum over the bins concerned.  Equal sums: the lower candidate index wins."""
    h = np.asarray(hist, dtype=np.float64).reshape(-1)
    x = bin_centres(h.size)
    G = np.asarray(cand, dtype=np.float64).reshape(-1)
    n = int(n_entries)
    assert 1 <= n <= G.size and np.all(np.diff(G) > 0)
    nG = G.size
    below = np.array([(h[x <= G[c]] * (x[x <= G[c]] - G[c]) ** 2).sum() for c in range(nG)])
    above = np.array([(h[x > G[c]] * (x[x > G[c]] - G[c]) ** 2).sum() for c in range(nG)])
    between = np.full((nG, nG), np.inf)
    for a in range(nG):
        for b in range(a + 1, nG):
            sel = (x > G[a]) & (x <= G[b])
            xs, hs = x[sel], h[sel]
            to_a = xs <= 0.5 * (G[a] + G[b])
            between[a, b] = (hs * np.where(to_a, (xs - G[a]) ** 2, (xs - G[b]) ** 2)).sum()
    best = np.full((n + 1, nG), np.inf)
    prev = np.full((n + 1, nG), -1, dtype=np.int64)
    best[1] = below
    for k in range(2, n + 1):
        for c in range(k - 1, nG):
            for cp in range(k - 2, c):
                v = best[k - 1][cp] + between[cp, c]
                if v < best[k][c]:
                    best[k][c], prev[k][c] = v, cp
    total = best[n] + above
    total[: n - 1] = np.inf
    c = int(np.argmin(total))                                        # first minimum: lowest index
    cost = float(total[c])
    chosen = []
    for k in range(n, 0, -1):
        chosen.append(c)
        c = int(prev[k][c])
    return np.array(chosen[::-1], dtype=np.int64), cost
