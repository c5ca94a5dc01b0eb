"""Step 2 of the per-layer pair search in the oracle: rank the blocks by a per-block score and split
them into the pool the first codebook keeps and the pool the second codebook is fitted on.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

Followed passages: Section "Per-Layer Pair Search", step 2 (every block is scored against L_a under
its own scale; the best-ranked p% form the first pool) and step 3 (the rest is the fitting pool of
L_b); design axes (i) (the ranking score is the block cosine or the unweighted block error) and
(iv) (the pool is defined by a rank: top-k / quantile threshold).

The paper leaves open how p% becomes a count and what happens to equal scores.  Reading taken:
  - the caller states the size of the first pool as a number of blocks n_top (0 .. N_b);
    top_count() turns a percentage into that number (nearest integer, halves up);
  - tau is the score of the block of rank n_top (ranks count from the best score, 1-based); every
    block whose score is at least as good as tau stays in the first pool, so blocks that tie with
    tau all stay and the first pool can exceed n_top by the ties;
  - n_top = 0 sends every block to the fitting pool (tau is +inf for "higher is better", -inf
    otherwise); +0 and -0 are the same score; scores are never NaN.
"""
from __future__ import annotations

import numpy as np


def top_count(p_percent: float, n_blocks: int) -> int:
    """Number of blocks in the first pool for a percentage p (nearest integer, halves up)."""
    if not 0.0 <= p_percent <= 100.0:
        raise ValueError("p must lie in [0, 100]")
    return min(n_blocks, int(np.floor(p_percent * n_blocks / 100.0 + 0.5)))


def partition(score: np.ndarray, n_top: int, higher_is_better: bool = True):
    """Returns (tau, pool_b, n_a): the threshold score, a [N_b] uint8 mask that is 1 for the blocks
    of the fitting pool (those ranked strictly worse than tau), and the size of the first pool."""
    s = np.asarray(score, dtype=np.float32).reshape(-1)
    N = s.size
    if not 0 <= n_top <= N:
        raise ValueError("n_top out of range")
    if np.isnan(s).any():
        raise ValueError("scores must not be NaN")
    if n_top == 0:
        tau = np.float32(np.inf if higher_is_better else -np.inf)
        return tau, np.ones(N, dtype=np.uint8), 0
    asc = np.sort(s)                                   # ascending, equal zeros compare equal
    tau = asc[N - n_top] if higher_is_better else asc[n_top - 1]
    in_a = (s >= tau) if higher_is_better else (s <= tau)
    return np.float32(tau), (~in_a).astype(np.uint8), int(in_a.sum())
