"""The per-layer pair search of the paper, steps 1 to 4 with the sweep over the partition parameter p,
driven through the library (Section "Per-Layer Pair Search").

Every pass over the weights runs in the HIP kernels: scoring every block against L_a and the
finishing reassignment (sop_pair_search), ranking the blocks and splitting the pools (sop_partition),
the histogram of the fitting pool (sop_dd_histogram with a block mask), packing the result
(sop_pack_blocks).  The host does what the paper leaves to the host: the loop over candidates, the
fit on the 1024-bin histogram (sop_dd_fit: free Lloyd rounds, microseconds; or sop_dd_fit_grid: the
selection among the grid points of an LUT value format) and the comparison of layer ACos values.

Candidates examined for a layer:
  (1) every pair of fixed atoms of the alphabet (one search call);
  (2) for every fixed atom a and every p of the sweep: L_b fitted on the (100-p) % of blocks that a
      serves worst (steps 2 and 3), then the pair (a, L_b) scored by step 4.  The fitted codebooks of
      one atom's sweep are scored together, as pairs (a, L_b(p)) of one alphabet.
The winner is the candidate with the largest layer ACos (the first one among equals).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import binding as B


@dataclass
class LayerResult:
    kind: str                 # "fixed": both atoms from the alphabet; "fitted": L_b fitted on the pool
    a: int                    # index of L_a in the alphabet
    b: int                    # index of L_b in the alphabet ("fixed"), -1 otherwise
    p_percent: float          # partition parameter of the winner (nan for "fixed")
    table_a: np.ndarray
    table_b: np.ndarray
    acos: float
    acos_fixed: np.ndarray    # [P] ACos of every pair of fixed atoms
    acos_fitted: dict = field(default_factory=dict)   # (a, p) -> ACos of (a, L_b(a, p))
    words: object = None      # packed scale words (device tensor) when asked for
    payload: object = None    # packed codes (device tensor)
    n_bits: int = 0


def top_count(p_percent: float, n_blocks: int) -> int:
    """Blocks in the first pool for a percentage p: nearest integer, halves up."""
    return min(n_blocks, int(np.floor(p_percent * n_blocks / 100.0 + 0.5)))


def search_layer(ctx: B.Context, W, c, g: int, fmt: B.ScaleFmt, atoms: list, p_grid=(50.0, 70.0, 85.0, 95.0),
                 k: int = 0, metric: int = B.SEL_WSE, fit_entries: int = 16, fit_iters: int = 20, fit_bins: int = 1024,
                 fit_init: np.ndarray | None = None, weighted_fit: bool = True, pack: bool = False,
                 fit_grid: np.ndarray | None = None) -> LayerResult:
    """Run the search on one layer (W [M,K] bf16/fp32 and c [K] fp32 on the GPU).

    fit_grid: ascending candidate values in the atoms' units (largest magnitude 1, e.g. the E2M3 grid
    divided by 7.5): the second codebook is then selected among them (grid-constrained construction)
    instead of being fitted freely; fit_iters and fit_init are not used."""
    import torch
    M, K = W.shape
    Nb = M * K // g
    atoms = [np.ascontiguousarray(t, dtype=np.float32) for t in atoms]
    A = len(atoms)
    init = np.asarray(atoms[0] if fit_init is None else fit_init, dtype=np.float32)
    if init.size != fit_entries:
        raise ValueError("the start grid of the fit must have fit_entries values")

    # (1) fixed pairs, and the block cosines of every fixed atom for step 2
    ctx.set_alphabet(atoms)
    ctx.set_pairs(None)
    out = ctx.alloc_outputs(M, K, g, emit=False, sel=False)
    out.blk_rank = torch.empty((A, Nb), dtype=torch.float32, device=W.device)   # the only per-block plane step 2 needs
    ctx.pair_search(W, c, g, fmt, k=k, metric=metric, out=out)
    torch.cuda.synchronize()
    acos_fixed = out.acos_pair.cpu().numpy()[:ctx.n_pairs].copy()
    pairs = [(i, j) for i in range(A) for j in range(i + 1, A)]
    best = None
    if pairs:
        q = int(np.argmax(acos_fixed))
        best = ("fixed", pairs[q][0], pairs[q][1], float("nan"), float(acos_fixed[q]), None)
    blk_rank = out.blk_rank                            # [A, Nb]

    # (2) fitted second codebooks: steps 2 and 3 per (a, p), step 4 for one atom's whole sweep at once
    acos_fitted = {}
    p_list = list(p_grid)
    # steps 2 and 3 of every (a, p): rankings and masked histograms queued back to back (the stream orders
    # them); one copy to the host then waits for all of them, and the fits follow on the host
    hists = []
    for a in range(A):
        for p in p_list:
            pool_b, _, _ = ctx.partition(blk_rank[a], top_count(p, Nb), True)
            hists.append(ctx.dd_histogram(W, c if weighted_fit else None, g, fit_bins, 1, block_mask=pool_b))
    hs = torch.stack(hists).cpu().numpy().reshape(A, len(p_list), fit_bins)       # synchronises: 8 KB per (a, p)
    if fit_grid is None:
        def fit(h):
            return B.sop_dd_fit(h, fit_entries, fit_iters, init)
    else:
        cand = np.ascontiguousarray(fit_grid, dtype=np.float64)

        def fit(h):
            return cand[B.sop_dd_fit_grid(h, cand, fit_entries)[0]].astype(np.float32)
    fitted_all = [[fit(h) if h.sum() > 0 else init.copy() for h in hs[a]] for a in range(A)]
    # step 4: one atom's whole sweep is scored by one call; the calls are queued, their tables read at the end
    pending = []
    for a in range(A):
        fitted = fitted_all[a]
        for s0 in range(0, len(p_list), 7):            # at most eight atoms in an alphabet
            chunk = fitted[s0:s0 + 7]
            torch.cuda.synchronize()                   # the alphabet's tables are replaced: nothing may still read them
            ctx.set_alphabet([atoms[a]] + chunk)
            ctx.set_pairs([(0, 1 + i) for i in range(len(chunk))])
            o = ctx.pair_search(W, c, g, fmt, k=k, metric=metric)
            pending.append((a, s0, chunk, o))
    torch.cuda.synchronize()
    for a, s0, chunk, o in pending:
        ac = o.acos_pair.cpu().numpy()[:len(chunk)]
        for i, v in enumerate(ac):
            p = p_list[s0 + i]
            acos_fitted[(a, p)] = float(v)
            if best is None or v > best[4]:
                best = ("fitted", a, -1, p, float(v), chunk[i])
    kind, a, b, p, acos, tb = best
    table_b = atoms[b] if kind == "fixed" else tb
    res = LayerResult(kind, a, b, p, atoms[a], table_b, acos, acos_fixed, acos_fitted)
    if pack:
        ctx.set_alphabet([atoms[a], table_b])
        ctx.set_pairs(None)
        o = ctx.pair_search(W, c, g, fmt, k=k, metric=metric, emit=True)
        res.words, res.payload, res.n_bits = ctx.pack_blocks(o, M, K, g, fmt, 0, 1, 0)
        torch.cuda.synchronize()
    return res
