"""Seeded random sweeps of the widened rows against the oracle, on the shared context: levelled ranking and levelled
histograms, the data-derived histogram (row steps, masks, row strides), the static entry point against the ordinary one,
the scale-shift statistics and the layer-scope formats on small layers, and the packing.  The number of cases per sweep
can be raised through SOP_RANDOM_WIDENED for a longer hunt."""
import os

import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, dd as DD, flayer as FL, pack as PK, partition as PT, pairsearch as ops
import sop_inputs as si
from gpu_util import oracle_fmt, ctx
import test_gpu_dd as TD, test_gpu_flayer as TF, test_gpu_layerscope as TL, test_gpu_pack as TP

pytestmark = pytest.mark.gpu
N = int(os.environ.get("SOP_RANDOM_WIDENED", "12"))


def _layer(rng, seed, scale=1.0, row_sigma=0.5):
    g = int(rng.choice([8, 16, 32, 64]))
    M, K = int(rng.integers(1, 60)), g * int(rng.integers(1, 60))
    while K % 8: K += g
    bf16 = bool(rng.random() < 0.5)
    W = si.student_t_weights(M, K, 4.0, seed, row_sigma=row_sigma, outlier_frac=0.002, scale=scale)
    if rng.random() < 0.3: W.reshape(-1, g)[rng.integers(0, M * K // g, 4)] = 0
    if rng.random() < 0.2: W[rng.integers(0, M)] = 0
    if bf16: W = si.bf16_round(W)
    return g, M, K, bf16, W


@pytest.mark.parametrize("seed", range(N))
def test_levelled_ranking_and_histograms(seed):
    import torch
    rng = np.random.default_rng(8800 + seed)
    g, M, K, bf16, W = _layer(rng, 8900 + seed)
    Nb = M * K // g
    c = si.channel_norms(K, 1.0, 9000 + seed) if rng.random() < 0.8 else None
    kind = rng.integers(0, 3)
    score = ((1 - np.abs(rng.standard_normal(Nb)) * 0.01) if kind == 0 else (rng.integers(-3, 4, Nb) * 0.5) if kind == 1 else rng.standard_normal(Nb)).astype(np.float32)
    L = int(rng.integers(1, 9))
    tops = sorted(int(x) for x in rng.integers(0, Nb + 1, L))
    higher = bool(rng.random() < 0.7)
    level, tau, n_a = ctx().partition_levels(torch.from_numpy(score).cuda(), tops, higher)
    torch.cuda.synchronize()
    level, tau, n_a = level.cpu().numpy(), tau.cpu().numpy(), n_a.cpu().numpy()
    ref_level = np.zeros(Nb, np.uint8)
    for j, t in enumerate(tops):
        rt, rp, rn = PT.partition(score, t, higher)
        ref_level += rp.astype(np.uint8)
        assert n_a[j] == rn and (t == 0 or tau[j] == rt or (tau[j] == 0 and rt == 0)), (j, t)
    assert np.array_equal(level, ref_level)
    bins = int(rng.choice([64, 256, 1024]))
    if L * bins > 8192: bins = 64
    Wt = torch.from_numpy(W).cuda()
    if bf16: Wt = Wt.to(torch.bfloat16)
    h = ctx().dd_histogram_levels(Wt, None if c is None else torch.from_numpy(c).cuda(), g, torch.from_numpy(level).cuda(), L, n_bins=bins)
    torch.cuda.synchronize()
    h = h.cpu().numpy()
    for j in range(L):
        assert np.array_equal(h[j], DD.histogram(W, c, g, bins, block_mask=(level > j).astype(np.uint8))), j


@pytest.mark.parametrize("seed", range(N))
def test_histogram_and_static_entry_point(seed):
    import torch
    rng = np.random.default_rng(13000 + seed)
    g, M, K, bf16, W = _layer(rng, 13100 + seed)
    c = si.channel_norms(K, 1.0, 13200 + seed) if rng.random() < 0.8 else None
    if c is not None and rng.random() < 0.3: c[rng.integers(0, K, 4)] = 0
    H = int(rng.choice([64, 128, 1024, 4096, 8192]))
    step = int(rng.choice([1, 1, 2, 3, 7]))
    mask = (rng.random(M * K // g) < 0.5).astype(np.uint8) if (rng.random() < 0.5 and step == 1) else None
    ldw = K + 8 * int(rng.integers(1, 4)) if rng.random() < 0.3 else None
    got = TD.gpu_hist(W, c, g, H, bf16, ldw=ldw, row_step=step, mask=mask)
    assert np.array_equal(got, DD.histogram(W[::step], c, g, H, block_mask=mask))
    pool = [OA.to_f32(t) for t in (OA.nf(4), OA.sh(4), OA.negate(OA.nf(4)), OA.nf(3), OA.nf(5), OA.sh(5), OA.negate(OA.sh(4)))]
    A = int(rng.integers(1, 7))
    tabs = [pool[i] for i in rng.permutation(len(pool))[:A]]
    fmt = sop.fmt_by_name(str(rng.choice(["UE4M4", "E4M3", "UE4M6", "S1E5M5", "E4M7"])))
    cx = ctx(); cx.set_alphabet(tabs); cx.set_pairs(None)
    Wt = torch.from_numpy(W).cuda()
    if bf16: Wt = Wt.to(torch.bfloat16)
    ct = torch.from_numpy(si.channel_norms(K, 1.0, 13300 + seed)).cuda()
    emit = bool(rng.random() < 0.5)
    o1 = cx.pair_search(Wt, ct, g, fmt, emit=emit)
    o2 = cx.alloc_outputs(M, K, g, emit=emit)
    cx.pair_search(Wt, ct, g, fmt, out=o2, emit=emit, static=True)
    torch.cuda.synchronize()
    P = A * (A - 1) // 2
    assert torch.equal(o1.acos_atom, o2.acos_atom)
    if P: assert torch.equal(o1.acos_pair[:P], o2.acos_pair[:P]) and torch.equal(o1.sel_words, o2.sel_words)
    if emit:
        for nm in ("scale_code", "codes", "blk_err", "blk_cos", "blk_rank"):
            assert torch.equal(getattr(o1, nm), getattr(o2, nm)), nm


@pytest.mark.parametrize("seed", range(N))
def test_scale_shift_statistics_and_layer_scope(seed):
    rng = np.random.default_rng(9900 + seed)
    g, M, K, bf16, W = _layer(rng, 9950 + seed, scale=float(2.0 ** rng.integers(-12, 6)), row_sigma=float(rng.choice([0.5, 1.5])))
    f = sop.fmt_by_name(str(rng.choice(["UE4M4", "E4M3", "S1E5M5", "UE5M7", "E4M7", "E5M6"])))
    tp, tn = [(1.0, 1.0), (0.98139, 1.0), (1.0, 0.98139), (0.75, 0.5)][int(rng.integers(0, 4))]
    sc = FL.block_scales(W, g, tp, tn)
    got = TF.gpu_hist(W, g, tp, tn, f, bf16)
    assert np.array_equal(got, FL.exponent_histogram(sc, f.exp_bits, f.man_bits, f.bias, f.max_code))
    assert sop.sop_layer_shift(got, sc.size, f) == FL.layer_shift(sc, f.exp_bits, f.man_bits, f.bias, f.max_code)
    c = si.channel_norms(K, 1.0, 9960 + seed) if rng.random() < 0.7 else None
    wf = [(4, 3, -1, -1), (4, 3, -1, 0x7E), (2, 3, -1, -1), (5, 6, -1, -1), (3, 4, -1, -1), (5, 2, -1, -1)][int(rng.integers(0, 6))]
    sf = [TL.UE8M0, sop.fmt_by_name("UE4M4"), sop.fmt_by_name("E8M7"), sop.fmt_by_name("UE5M3")][int(rng.integers(0, 4))]
    TL.check(W, c, wf, sf, k=int(rng.integers(0, 6)) if sf.exp_bits < 8 else 0, bf16=bf16)


@pytest.mark.parametrize("seed", range(N))
def test_packing(seed):
    import torch
    rng = np.random.default_rng(12000 + seed)
    g = int(rng.choice([8, 16, 32, 64]))
    M, K = 2 * int(rng.integers(1, 20)), g * int(rng.integers(1, 50))          # (code planes back to back stay 8-byte aligned)
    while K % 16: K += g
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 12100 + seed, row_sigma=0.5, outlier_frac=0.002))
    if rng.random() < 0.3: W[rng.integers(0, M)] = 0
    c = si.channel_norms(K, 1.0, 12200 + seed)
    pool = [OA.to_f32(t) for t in (OA.nf(4), OA.sh(4), OA.negate(OA.nf(4)), OA.nf(3), OA.nf(5), OA.sh(5), OA.exmy_grid(2, 3), np.array([-1.0, 1.0]), OA.sh(3))]
    A = int(rng.integers(1, 7))
    tabs = [pool[i] for i in rng.permutation(len(pool))[:A]]
    fmt, (w, x, y, b) = TP.make_fmt(str(rng.choice(["UE4M3", "S1E5M5", "S0E6M5", "S1E5M4", "S0E5M5", "E4M3", "UE4M4"])))
    k = int(rng.integers(-1, 4))
    out = TP.search(W, c, tabs, g, fmt, k=k)
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), k=k)
    pairs = ops.all_pairs(A).tolist()
    trials = [(int(rng.integers(0, A)), None, None)]
    if pairs and b - w - x - y > 0:
        q = int(rng.integers(0, len(pairs))); trials.append((pairs[q][0], pairs[q][1], q))
    for (a, bb, q) in trials:
        words, payload, n = ctx().pack_blocks(out, M, K, g, fmt, a, bb, q if q is not None else 0)
        torch.cuda.synchronize()
        rw, rp, rn = PK.materialise(ref, tabs, M, K, g, a, bb, q, w, x, y, b)
        assert n == rn and np.array_equal(words.cpu().numpy().view(np.uint16), rw) and np.array_equal(payload.cpu().numpy(), rp)
