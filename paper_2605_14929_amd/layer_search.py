"""The per-layer pair search of the paper, steps 1 to 4 with the sweep over the partition parameter p
(Section "Per-Layer Pair Search"), as the library runs it: sop_search_layer.

Nothing of the procedure lives here: the loop over candidates, the count a percentage p stands for, the fits
and the choice of the winner are the library's (include/sop.h).  This module only gives the result a Python
shape.
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
    acos_fitted: dict = field(default_factory=dict)   # (a, p) -> ACos of (a, L_b(a, p)); dropped candidates are absent
    words: object = None      # packed scale words (device tensor) when asked for
    payload: object = None    # packed codes (device tensor)
    n_bits: int = 0


def search_layer(ctx: B.Context, W, c, g: int, fmt: B.ScaleFmt, atoms: list, p_grid=(50.0, 70.0, 85.0, 95.0),
                 k: int = 0, metric: int = B.SEL_WSE, fit_entries: int = 16, fit_iters: int = 20, fit_bins: int = 1024,
                 fit_init: np.ndarray | None = None, weighted_fit: bool = True, pack: bool = False,
                 fit_grid: np.ndarray | None = None) -> LayerResult:
    """One sop_search_layer call on a layer (W [M,K] bf16/fp32 and c [K] fp32 on the GPU).

    fit_grid: ascending candidate values in the atoms' units (largest magnitude 1, e.g. the E2M3 grid divided
    by 7.5): the second codebook is then selected among them instead of being fitted freely."""
    atoms = [np.ascontiguousarray(t, dtype=np.float32) for t in atoms]
    r, words, payload = ctx.search_layer(W, c, g, fmt, atoms, p_grid=p_grid, k=k, metric=metric, fit_entries=fit_entries,
                                         fit_iters=fit_iters, fit_bins=fit_bins, fit_init=fit_init, weighted_fit=weighted_fit,
                                         fit_grid=fit_grid, pack=pack)
    A = len(atoms)
    fixed = np.array(r.acos_fixed[:A * (A - 1) // 2], dtype=np.float64)
    fitted = {}
    for a in range(A):
        for j, p in enumerate(p_grid):
            if r.acos_fitted[a][j] == r.acos_fitted[a][j]:
                fitted[(a, p)] = float(r.acos_fitted[a][j])
    table_b = np.array(r.table_b[:r.n_entries_b], dtype=np.float32)
    return LayerResult("fixed" if r.kind == 0 else "fitted", r.a, r.b, float("nan") if r.kind == 0 else r.p_percent,
                       atoms[r.a], table_b, r.acos, fixed, fitted, words, payload, r.n_bits)
