"""GPU parity of the block ranking (step 2 of the pair search) and of steps 1-4 chained: threshold,
pool mask and pool size bit-exact against the oracle; the refit on the pool and the final search
equal to the oracle's chain."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, dd as DD, partition as PT, pairsearch as ops
import sop_inputs as si
from gpu_util import run_gpu, compare, oracle_fmt, ctx

pytestmark = pytest.mark.gpu


def gpu_partition(score, n_top, higher=True):
    import torch
    st = torch.from_numpy(np.ascontiguousarray(score, dtype=np.float32)).cuda()
    pool_b, tau, n_a = ctx().partition(st, n_top, higher)
    torch.cuda.synchronize()
    return tau.cpu().numpy()[0], pool_b.cpu().numpy(), int(n_a.cpu().numpy()[0])


def check(score, n_top, higher=True):
    tau, pool_b, n_a = gpu_partition(score, n_top, higher)
    rt, rp, rn = PT.partition(score, n_top, higher)
    assert tau == rt or (tau == 0.0 and rt == 0.0), (tau, rt)
    assert n_a == rn
    assert np.array_equal(pool_b, rp)


@pytest.mark.parametrize("higher", [True, False])
def test_ranks_sizes_and_ties(higher):
    rng = np.random.default_rng(11)
    for N in (1, 2, 3, 5, 1023, 1024, 4099, 70001):                  # ragged tails, one and many workgroups
        cosv = (1.0 - np.abs(rng.standard_normal(N)) * 0.01).astype(np.float32)     # block cosines crowd below 1
        for n_top in sorted({0, 1, N // 3, N - 1, N} & set(range(N + 1))):
            check(cosv, n_top, higher)
    # heavy ties, both zeros, negative and huge values, subnormals
    s = rng.integers(-4, 5, 50000).astype(np.float32) * np.float32(0.25)
    s[::7] = -0.0
    s[1::11] = np.float32(1e-42)
    s[2::13] = np.float32(-3e38)
    s[3::17] = np.float32(3e38)
    for n_top in (1, 100, 25000, 49999, 50000):
        check(s, n_top, higher)
    # all equal
    check(np.full(777, 0.5, np.float32), 5, higher)


def test_calls_in_a_row_leave_no_state():
    rng = np.random.default_rng(12)
    a = rng.standard_normal(30000).astype(np.float32)
    b = rng.standard_normal(999).astype(np.float32)
    for _ in range(2):
        check(a, 12345)
        check(b, 17, False)
        check(b, 0)


def test_argument_validation():
    import torch
    cx = ctx()
    s = torch.zeros(16, dtype=torch.float32, device="cuda")
    with pytest.raises(sop.SopError):
        cx.partition(s, 17)
    with pytest.raises(sop.SopError):
        cx.partition(s, -1)
    with pytest.raises(sop.SopError):
        cx.partition(s[1:], 2)                                        # misaligned
    with pytest.raises(sop.SopError):
        cx.partition(s.double(), 2)


def test_steps_one_to_four_chained():
    import torch
    M, K, g = 96, 2048, 16
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 2100, row_sigma=0.4, outlier_frac=0.001))
    c = si.channel_norms(K, 1.0, 2101)
    fmt = sop.fmt_by_name("UE4M3")                                   # one metabit: the selector fits
    La = OA.to_f32(OA.nf(4))
    cx = ctx()
    Wt = torch.from_numpy(W).cuda().to(torch.bfloat16)
    ct = torch.from_numpy(c).cuda()
    # steps 1 and 2 on the GPU
    cx.set_alphabet([La]); cx.set_pairs(None)
    o1 = cx.pair_search(Wt, ct, g, fmt, emit=True)
    Nb = M * K // g
    n_top = PT.top_count(70.0, Nb)
    pool_b, tau, n_a = cx.partition(o1.blk_rank[0], n_top, True)
    # step 3 on the GPU: histogram of the pool, fit on the host side of the library
    hist = cx.dd_histogram(Wt, ct, g, 1024, 1, block_mask=pool_b)
    torch.cuda.synchronize()
    Lb = sop.sop_dd_fit(hist.cpu().numpy(), 16, 12, La)
    # the oracle's chain
    r1 = ops.pair_search(W, c, [La], g, oracle_fmt(fmt))
    assert np.max(np.abs(o1.blk_cos[0].cpu().numpy() - r1.blk_cos[0])) < 2e-5
    # the ranking score is a binary32 decision quantity: both sides hold the same bits, and the oracle
    # ranks its own plane
    assert np.array_equal(o1.blk_rank[0].cpu().numpy().view(np.uint32), r1.blk_rank[0].view(np.uint32))
    rt, rp, rn = PT.partition(r1.blk_rank[0], n_top, True)
    assert tau.cpu().numpy()[0] == rt and int(n_a.cpu().numpy()[0]) == rn and np.array_equal(pool_b.cpu().numpy(), rp)
    rh = DD.histogram(W, c, g, 1024, block_mask=rp)
    assert np.array_equal(hist.cpu().numpy(), rh)
    rLb = OA.to_f32(DD.fit(rh, 16, 12, OA.nf(4)))
    assert np.array_equal(Lb, rLb)
    # step 4: the search over (L_a, L_b) on both sides
    gpu = run_gpu(W, c, [La, Lb], g, fmt, bf16=True)
    ref = ops.pair_search(W, c, [La, rLb], g, oracle_fmt(fmt))
    compare(gpu, ref, 1)
    assert ref.acos_pair[0] > ref.acos_atom.max()


def test_block_counts_of_the_large_configurations():
    # 2 818 048 blocks (4096 x 11008, g = 16) and 14 680 064 blocks (28672 x 8192, g = 16): scores shaped
    # like block cosines (crowded just below 1), both directions
    rng = np.random.default_rng(13)
    for N in (4096 * 11008 // 16, 28672 * 8192 // 16):
        s = (1.0 - np.abs(rng.standard_normal(N)).astype(np.float32) * np.float32(0.004)).astype(np.float32)
        for p_percent, higher in ((70.0, True), (12.5, False)):
            check(s, PT.top_count(p_percent, N), higher)


@pytest.mark.parametrize("higher", [True, False])
def test_several_thresholds_at_once_equal_single_rankings(higher):
    """sop_partition_levels / sop_dd_histogram_levels (the sweep over p from one ranking and one pass over the
    weights) against the oracle's ranking and masked histogram, threshold by threshold."""
    import torch
    M, K, g = 96, 2048, 16
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 7700, row_sigma=0.5))
    c = si.channel_norms(K, 1.0, 7701)
    Nb = M * K // g
    rng = np.random.default_rng(77)
    # scores crowded like block cosines, with ties, zeros of both signs and a ragged length for the pure ranking
    s = (1.0 - np.abs(rng.standard_normal(Nb)).astype(np.float32) * np.float32(0.004)).astype(np.float32)
    s[rng.integers(0, Nb, 500)] = s[7]
    s[:5] = [0.0, -0.0, 1.0, 1.0, -1.0]
    cx = ctx()
    for tops in ([PT.top_count(p, Nb) for p in (50.0, 70.0, 85.0, 95.0)], [0, 0, 17, Nb // 3, Nb // 3, Nb - 1, Nb, Nb], [Nb // 2], [0]):
        level, tau, n_a = cx.partition_levels(torch.from_numpy(s).cuda(), tops, higher)
        hist = cx.dd_histogram_levels(torch.from_numpy(W).cuda().to(torch.bfloat16), torch.from_numpy(c).cuda(), g, level, len(tops), 512)
        torch.cuda.synchronize()
        level, tau, n_a, hist = level.cpu().numpy(), tau.cpu().numpy(), n_a.cpu().numpy(), hist.cpu().numpy()
        want_level = np.zeros(Nb, dtype=np.int64)
        for j, t in enumerate(tops):
            rt, rp, rn = PT.partition(s, t, higher)
            assert tau[j] == rt and n_a[j] == rn, (tops, j)
            assert np.array_equal((level > j).astype(np.uint8), rp), (tops, j)
            assert np.array_equal(hist[j], DD.histogram(W, c, g, 512, block_mask=rp)), (tops, j)
            want_level += rp
        assert np.array_equal(level, want_level)
    # a ragged number of scores (not a multiple of four), ranking only
    s2 = s[:Nb - 3]
    tops = [10, 1000, Nb // 2]
    level, tau, n_a = cx.partition_levels(torch.from_numpy(s2).cuda(), tops, higher)
    torch.cuda.synchronize()
    for j, t in enumerate(tops):
        rt, rp, rn = PT.partition(s2, t, higher)
        assert tau.cpu().numpy()[j] == rt and int(n_a.cpu().numpy()[j]) == rn
        assert np.array_equal((level.cpu().numpy() > j).astype(np.uint8), rp)
    with pytest.raises(sop.SopError):
        cx.partition_levels(torch.from_numpy(s).cuda(), [100, 50], higher)          # pools must be nested
