"""The whole per-layer search (fixed pairs, and for every atom a sweep over p with a refit second
codebook) driven through the library, against the same procedure written with the oracle's parts."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from paper_2605_14929_amd import layer_search as LSR
from oracle import atoms as OA, dd as DD, pack as PK, partition as PT, pairsearch as ops
import sop_inputs as si
from gpu_util import oracle_fmt, ctx

pytestmark = pytest.mark.gpu


def oracle_search(W, c, g, fmt, atoms, p_grid, entries, iters, bins, grid=None):
    A = len(atoms)
    r = ops.pair_search(W, c, atoms, g, fmt, want_codes=False)
    fixed = r.acos_pair.copy()
    fitted = {}
    Nb = W.size // g
    for a in range(A):
        for p in p_grid:
            _, pool_b, _ = PT.partition(r.blk_rank[a], PT.top_count(p, Nb), True)
            h = DD.histogram(W, c, g, bins, block_mask=pool_b)
            if grid is None:
                Lb = OA.to_f32(DD.fit(h, entries, iters, atoms[0].astype(np.float64)))
            else:
                Lb = OA.to_f32(grid[DD.fit_grid(h, grid, entries)[0]])
            rr = ops.pair_search(W, c, [atoms[a], Lb], g, fmt, want_codes=False)
            fitted[(a, p)] = (float(rr.acos_pair[0]), Lb)
    return fixed, fitted


def test_search_of_one_layer_matches_the_oracle_procedure():
    import torch
    M, K, g = 128, 2048, 16
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 6100, row_sigma=0.5, outlier_frac=0.001))
    c = si.channel_norms(K, 1.0, 6101)
    atoms = [OA.to_f32(OA.nf(4)), OA.to_f32(OA.sh(4)), OA.to_f32(OA.negate(OA.sh(4)))]
    fmt = sop.fmt_by_name("UE4M3")
    p_grid = (50.0, 75.0, 90.0)
    Wt = torch.from_numpy(W).cuda().to(torch.bfloat16)
    ct = torch.from_numpy(c).cuda()
    res = LSR.search_layer(ctx(), Wt, ct, g, fmt, atoms, p_grid=p_grid, fit_iters=12, pack=True)
    fixed, fitted = oracle_search(W, c, g, oracle_fmt(fmt), atoms, p_grid, 16, 12, 1024)
    assert np.max(np.abs(res.acos_fixed - fixed)) <= 1e-6
    # both sides rank the same binary32 scores: pools, histograms and fitted codebooks are equal, and
    # every pair's ACos agrees to the tolerance of a single search
    for key, (v, Lb) in fitted.items():
        assert abs(res.acos_fitted[key] - v) <= 1e-6, key
    ref_best = max([("fixed", float(v)) for v in fixed] + [("fitted", v) for v, _ in fitted.values()], key=lambda t: t[1])
    assert abs(res.acos - ref_best[1]) <= 1e-6 and res.kind == ref_best[0]
    if res.kind == "fitted":
        assert np.array_equal(res.table_b, fitted[(res.a, res.p_percent)][1])
    # a second codebook fitted on the worst blocks beats every fixed pair on this layer, and more so
    # than any single atom
    assert res.kind == "fitted" and res.acos > fixed.max()
    # the packed result decodes to a layer whose cosine is the reported one
    w_, x_, y_, b_ = 0, 4, 3, 8
    What = PK.reconstruct(res.words.cpu().numpy().view(np.uint16), res.payload.cpu().numpy(), res.n_bits, g, M, K,
                          res.table_a, res.table_b, oracle_fmt(fmt), 0, w_, x_, y_, b_)
    cw = np.tile(c.astype(np.float64), M).reshape(-1, g)
    wb, hb = W.astype(np.float64).reshape(-1, g), What.astype(np.float64).reshape(-1, g)
    num = (cw * wb * hb).sum(1); den = np.sqrt((cw * wb * wb).sum(1) * (cw * hb * hb).sum(1))
    cosv = np.where(den > 0, num / np.where(den > 0, den, 1), 1.0)
    assert abs(cosv.mean() - res.acos) <= 1e-6


def test_search_with_the_second_codebook_selected_on_an_lut_grid():
    """Step 3 with the grid-constrained construction: L_b is chosen among the E2M3 grid's values."""
    import torch
    M, K, g = 96, 1024, 16
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 6200, row_sigma=0.5, outlier_frac=0.001))
    c = si.channel_norms(K, 1.0, 6201)
    atoms = [OA.to_f32(OA.nf(4)), OA.to_f32(OA.sh(4))]
    fmt = sop.fmt_by_name("UE4M3")
    p_grid = (60.0, 90.0)
    grid = OA.exmy_grid(2, 3) / 7.5
    assert np.array_equal(grid, sop.sop_weight_grid(sop.WeightFmt(2, 3, -1, -1)) / 7.5)
    Wt = torch.from_numpy(W).cuda().to(torch.bfloat16)
    ct = torch.from_numpy(c).cuda()
    res = LSR.search_layer(ctx(), Wt, ct, g, fmt, atoms, p_grid=p_grid, fit_grid=grid)
    fixed, fitted = oracle_search(W, c, g, oracle_fmt(fmt), atoms, p_grid, 16, 0, 1024, grid=grid)
    assert np.max(np.abs(res.acos_fixed - fixed)) <= 1e-6
    for key, (v, Lb) in fitted.items():
        assert abs(res.acos_fitted[key] - v) <= 1e-6, key
    ref_best = max([("fixed", float(v)) for v in fixed] + [("fitted", v) for v, _ in fitted.values()], key=lambda t: t[1])
    assert abs(res.acos - ref_best[1]) <= 1e-6 and res.kind == ref_best[0]
    if res.kind == "fitted":
        assert np.all(np.isin(res.table_b.astype(np.float64), grid.astype(np.float32).astype(np.float64)))   # every entry is a grid value


@pytest.mark.parametrize("A", [9, 10, 16])
def test_alphabets_of_more_than_eight_atoms(A):
    """Alphabets above the kernel's eight atoms are covered by several searches inside the one call: every pair of
    atoms, every atom alone and the sweep over p against the oracle (which takes sixteen atoms at once)."""
    import torch
    M, K, g = 64, 2048, 16
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 6300 + A, row_sigma=0.5, outlier_frac=0.001))
    c = si.channel_norms(K, 1.0, 6301)
    draws = si.normal_draws(1 << 16, 4242)
    base = [OA.nf(4), OA.sh(4), OA.bof(4, draws), OA.sh(4, 1.2, 0.01), OA.sh(4, 2.0, -0.03), OA.nf(3), OA.sh(5), OA.nf(5)]
    atoms = [OA.to_f32(t) for t in base] + [OA.to_f32(OA.negate(t)) for t in base]
    order = [0, 8, 1, 9, 2, 10, 3, 11, 4, 12, 5, 13, 6, 14, 7, 15][:A]
    atoms = [atoms[i] for i in order]
    fmt = sop.fmt_by_name("UE4M3")
    p_grid = (60.0, 90.0)
    Wt = torch.from_numpy(W).cuda().to(torch.bfloat16)
    ct = torch.from_numpy(c).cuda()
    res = LSR.search_layer(ctx(), Wt, ct, g, fmt, atoms, p_grid=p_grid, fit_iters=8, fit_init=atoms[0])
    ofmt = oracle_fmt(fmt)
    pairs = np.array([(a, b) for a in range(A) for b in range(a + 1, A)], dtype=np.int32)
    fixed = np.zeros(len(pairs))
    r = None
    for i0 in range(0, len(pairs), 28):                                   # the oracle's selector word holds 32 pairs
        r = ops.pair_search(W, c, atoms, g, ofmt, pairs=pairs[i0:i0 + 28], want_codes=False)
        fixed[i0:i0 + 28] = r.acos_pair[:len(pairs[i0:i0 + 28])]
    assert res.acos_fixed.shape == fixed.shape and np.max(np.abs(res.acos_fixed - fixed)) <= 1e-6
    Nb = W.size // g
    best = ("fixed", fixed.max())
    for a in range(A):
        for p in p_grid:
            _, pool_b, _ = PT.partition(r.blk_rank[a], PT.top_count(p, Nb), True)
            h = DD.histogram(W, c, g, 1024, block_mask=pool_b)
            Lb = OA.to_f32(DD.fit(h, 16, 8, atoms[0].astype(np.float64)))
            v = float(ops.pair_search(W, c, [atoms[a], Lb], g, ofmt, want_codes=False).acos_pair[0])
            assert abs(res.acos_fitted[(a, p)] - v) <= 1e-6, (a, p)
            if v > best[1]: best = ("fitted", v)
    assert abs(res.acos - best[1]) <= 1e-6 and res.kind == best[0]
    if A == 10:
        # pairs of atoms only, the winner packed: the packed layer decodes to the reported cosine
        r2 = LSR.search_layer(ctx(), Wt, ct, g, fmt, atoms, p_grid=(), pack=True)
        assert r2.kind == "fixed" and np.array_equal(r2.acos_fixed, res.acos_fixed) and abs(r2.acos - fixed.max()) <= 1e-6
        assert (r2.a, r2.b) == tuple(pairs[int(np.argmax(fixed))])
        What = PK.reconstruct(r2.words.cpu().numpy().view(np.uint16), r2.payload.cpu().numpy(), r2.n_bits, g, M, K,
                              r2.table_a, r2.table_b, ofmt, 0, 0, 4, 3, 8)
        cw = np.tile(c.astype(np.float64), M).reshape(-1, g)
        wb, hb = W.astype(np.float64).reshape(-1, g), What.astype(np.float64).reshape(-1, g)
        num = (cw * wb * hb).sum(1); den = np.sqrt((cw * wb * wb).sum(1) * (cw * hb * hb).sum(1))
        assert abs(np.where(den > 0, num / np.where(den > 0, den, 1), 1.0).mean() - r2.acos) <= 1e-6


def test_calls_with_fewer_and_then_more_atoms_leave_no_state():
    """The batched ranking keeps digit counts per score plane in the context: a call over fewer planes between
    two calls over more must leave nothing behind (the third call equals the first bit for bit)."""
    import torch
    M, K, g = 64, 1024, 16
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 6400, row_sigma=0.5))
    c = si.channel_norms(K, 1.0, 6401)
    atoms = [OA.to_f32(OA.nf(4)), OA.to_f32(OA.sh(4)), OA.to_f32(OA.negate(OA.sh(4))), OA.to_f32(OA.negate(OA.nf(4)))]
    fmt = sop.fmt_by_name("UE4M3")
    Wt = torch.from_numpy(W).cuda().to(torch.bfloat16)
    ct = torch.from_numpy(c).cuda()
    cx = sop.Context(0)
    run = lambda n: LSR.search_layer(cx, Wt, ct, g, fmt, atoms[:n], p_grid=(50.0, 80.0), fit_iters=6)
    first = run(4)
    for n in (2, 4, 3, 1, 4):
        r = run(n)
        if n == 4:
            assert r.acos_fitted == first.acos_fitted and np.array_equal(r.acos_fixed, first.acos_fixed) and r.acos == first.acos


@pytest.mark.parametrize("seed", range(int(__import__("os").environ.get("SOP_RANDOM_LAYER_SEARCHES", "8"))))
def test_random_layer_searches_on_one_context(seed):
    """Random shapes, alphabets (1 to 12 atoms), sweeps, block sizes and scale words through sop_search_layer on the shared
    context, each against the oracle's parts chained."""
    import torch
    rng = np.random.default_rng(6500 + seed)
    g = int(rng.choice([8, 16, 32]))
    M, K = int(rng.integers(4, 40)), g * int(rng.integers(8, 80))
    if (M * (K // g)) % 4: M += 4 - M % 4                      # (whole float4s of scores: the batched ranking)
    W = si.bf16_round(si.student_t_weights(M, K, float(rng.uniform(3, 8)), 6600 + seed, row_sigma=0.5, outlier_frac=0.001))
    c = si.channel_norms(K, 1.0, 6700 + seed)
    pool = [OA.nf(4), OA.sh(4), OA.sh(4, 1.2, 0.01), OA.nf(3), OA.sh(5), OA.negate(OA.nf(4)), OA.negate(OA.sh(4)), OA.sh(4, 2.0, -0.03),
            OA.nf(5), OA.negate(OA.sh(5)), OA.negate(OA.nf(3)), OA.sh(3)]
    A = int(rng.choice([1, 2, 3, 4, 6, 8, 9, 12]))
    atoms = [OA.to_f32(pool[i]) for i in rng.permutation(len(pool))[:A]]
    fmt = sop.fmt_by_name(str(rng.choice(["UE4M3", "S1E5M5", "E4M5", "UE5M7"])))
    n_p = int(rng.integers(1 if A == 1 else 0, 4))
    p_grid = tuple(sorted(float(x) for x in rng.choice([0.0, 30.0, 50.0, 70.0, 85.0, 95.0, 100.0], size=n_p, replace=False)))
    bins = int(rng.choice([256, 1024]))
    init = OA.to_f32(OA.nf(4))
    metric = int(rng.choice([0, 0, 1, 2]))
    weighted = bool(rng.random() < 0.7)
    grid = None
    if rng.random() < 0.35:
        gv = OA.exmy_grid(*[(2, 3), (3, 3), (3, 2)][int(rng.integers(0, 3))])
        grid = gv / np.abs(gv).max()
    Wt = torch.from_numpy(W).cuda().to(torch.bfloat16)
    ct = torch.from_numpy(c).cuda()
    res = LSR.search_layer(ctx(), Wt, ct, g, fmt, atoms, p_grid=p_grid, fit_iters=5, fit_bins=bins, fit_init=init, metric=metric,
                           weighted_fit=weighted, fit_grid=grid)
    ofmt = oracle_fmt(fmt)
    pairs = np.array([(a, b) for a in range(A) for b in range(a + 1, A)], dtype=np.int32).reshape(-1, 2)
    fixed = np.zeros(len(pairs))
    r = ops.pair_search(W, c, atoms, g, ofmt, metric=metric, pairs=pairs[:1] if len(pairs) else None, want_codes=False)
    for i0 in range(0, len(pairs), 28):
        rr = ops.pair_search(W, c, atoms, g, ofmt, metric=metric, pairs=pairs[i0:i0 + 28], want_codes=False)
        fixed[i0:i0 + 28] = rr.acos_pair[:len(pairs[i0:i0 + 28])]
    assert np.max(np.abs(res.acos_fixed - fixed), initial=0.0) <= 1e-6
    Nb = W.size // g
    cands = [("fixed", float(v)) for v in fixed]
    for a in range(A):
        for p in p_grid:
            _, pool_b, _ = PT.partition(r.blk_rank[a], PT.top_count(p, Nb), True)
            h = DD.histogram(W, c if weighted else None, g, bins, block_mask=pool_b)
            if not h.any(): Lb = init
            elif grid is None: Lb = OA.to_f32(DD.fit(h, 16, 5, init.astype(np.float64)))
            else: Lb = OA.to_f32(grid[DD.fit_grid(h, grid, 16)[0]])
            if (a, p) not in res.acos_fitted:                  # dropped: the fitted codebook cannot serve as an atom
                continue
            v = float(ops.pair_search(W, c, [atoms[a], Lb], g, ofmt, metric=metric, want_codes=False).acos_pair[0])
            assert abs(res.acos_fitted[(a, p)] - v) <= 1e-6, (a, p)
            cands.append(("fitted", v))
    best = max(cands, key=lambda t: t[1])
    assert abs(res.acos - best[1]) <= 1e-6
