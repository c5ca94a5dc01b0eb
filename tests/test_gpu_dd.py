"""GPU parity of the data-derived codebook: the integer histogram of the HIP path against the
oracle's (bit-exact), the fitted table, and the pair search with the fitted atom appended."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, dd as DD, pairsearch as ops
import sop_inputs as si
from gpu_util import run_gpu, compare, oracle_fmt, ctx, cached_config

pytestmark = pytest.mark.gpu


def gpu_hist(W, c, g, H, bf16, ldw=None, row_step=1, mask=None):
    import torch
    Wt = torch.from_numpy(W).cuda()
    if bf16:
        Wt = Wt.to(torch.bfloat16)
    if ldw is not None:
        buf = torch.zeros((W.shape[0], ldw), dtype=Wt.dtype, device="cuda")
        buf[:, :W.shape[1]] = Wt
        Wt = buf[:, :W.shape[1]]
    ct = None if c is None else torch.from_numpy(c).cuda()
    mt = None if mask is None else torch.from_numpy(mask).cuda()
    h = ctx().dd_histogram(Wt, ct, g, H, row_step, block_mask=mt)
    torch.cuda.synchronize()
    return h.cpu().numpy()


@pytest.mark.parametrize("g", [8, 16, 32, 64])
@pytest.mark.parametrize("bf16", [False, True])
def test_histogram_block_sizes_dtypes_ragged(g, bf16):
    M, K = 37, 1088                                                   # ragged last strip, uneven row ranges
    W = si.student_t_weights(M, K, 4.0, 900 + g, row_sigma=0.5, outlier_frac=0.002)
    if bf16:
        W = si.bf16_round(W)
    W[3, :] = 0.0                                                     # zero blocks are skipped
    W[5, 64:128] = -np.abs(W[5, 64:128])
    c = si.channel_norms(K, 1.0, 901)
    c[200:216] = 0.0
    for H in (256, 1024):
        assert np.array_equal(gpu_hist(W, c, g, H, bf16), DD.histogram(W, c, g, H))
    assert np.array_equal(gpu_hist(W, None, g, 512, bf16), DD.histogram(W, None, g, 512))
    for step in (2, 5, 64):                                           # a sample of the rows: 0, step, 2*step, ...
        assert np.array_equal(gpu_hist(W, c, g, 256, bf16, row_step=step), DD.histogram(W[::step], c, g, 256))


def test_histogram_row_stride_and_bin_counts():
    M, K = 16, 512
    W = si.student_t_weights(M, K, 4.0, 911)
    c = si.channel_norms(K, 1.0, 912)
    assert np.array_equal(gpu_hist(W, c, 16, 64, False, ldw=K + 64), DD.histogram(W, c, 16, 64))
    assert np.array_equal(gpu_hist(W, c, 16, 8192, False), DD.histogram(W, c, 16, 8192))
    import torch
    with pytest.raises(sop.SopError) as e:
        ctx().dd_histogram(torch.from_numpy(W).cuda(), torch.from_numpy(c).cuda(), 16, 1000)
    assert e.value.status == 1
    with pytest.raises(sop.SopError) as e:
        ctx().dd_histogram(torch.from_numpy(W).cuda(), torch.from_numpy(c).cuda(), 12, 1024)
    assert e.value.status == 2


def test_histogram_is_reproducible_and_full_layer():
    W, c, cfg = cached_config("C3_down")
    a = gpu_hist(W, c, 16, 1024, True)
    b = gpu_hist(W, c, 16, 1024, True)
    assert np.array_equal(a, b)
    assert np.array_equal(a, DD.histogram(W, c, 16, 1024))


def test_dd4_joins_the_alphabet_config5_shape():
    # 70B-shaped MLP layer 28672 x 8192: histogram and fit on the whole layer, then the seven-atom
    # search (21 pairs, 32-bit selector words) against the oracle on the whole layer
    W, c, cfg = cached_config("C5")
    g, H = 16, 4096
    hist = gpu_hist(W, c, g, H, True)
    assert np.array_equal(hist, DD.histogram(W, c, g, H))
    init = sop.sop_atom_nf(4)
    dd4 = sop.sop_dd_fit(hist, 16, 20, init)                          # 16 centroids, 20 rounds, from NF4
    assert np.array_equal(dd4, DD.fit(hist, 16, 20, OA.to_f32(OA.nf(4)).astype(np.float64)).astype(np.float32))
    tabs = sop.build_alphabet(cfg["atoms"], bof_draws=si.normal_draws(1 << 20, 4242)) + [dd4]
    fmt = sop.fmt_by_name(cfg["fmt"])
    gpu = run_gpu(W, c, tabs, g, fmt, bf16=True, emit=False)
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), want_codes=False)
    compare(gpu, ref, 21, emit=False)
    # the atom fitted to this layer beats every fixed atom on it
    assert gpu["acos_atom"][6] > gpu["acos_atom"][:6].max()
    # a fit from every 16th row is the same grid to within two histogram bins
    h16 = gpu_hist(W, c, g, H, True, row_step=16)
    assert np.array_equal(h16, DD.histogram(W[::16], c, g, H))
    assert np.max(np.abs(sop.sop_dd_fit(h16, 16, 20, init) - dd4)) < 4e-3


@pytest.mark.parametrize("g", [8, 16, 32, 64])
def test_histogram_of_a_pool_of_blocks(g):
    M, K = 41, 1088
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 950 + g, row_sigma=0.5))
    c = si.channel_norms(K, 1.0, 951)
    rng = np.random.default_rng(952 + g)
    mask = (rng.random(M * K // g) < 0.35).astype(np.uint8)
    mask[mask == 1] = rng.integers(1, 256, int(mask.sum())).astype(np.uint8)      # any non-zero byte counts
    for row_step in (1, 3):
        ref_mask = mask.copy().reshape(M, K // g)
        keep = np.zeros(M, bool); keep[::row_step] = True
        ref_mask[~keep] = 0
        ref = DD.histogram(W, c, g, 512, block_mask=ref_mask.reshape(-1))
        got = gpu_hist(W, c, g, 512, True, row_step=row_step, mask=mask)
        assert np.array_equal(got, ref)
    assert gpu_hist(W, c, g, 512, True, mask=np.zeros_like(mask)).sum() == 0


def test_grid_constrained_dd4_joins_the_alphabet():
    # the codebook selected among the E4M3 grid's values (step 1 of the pair search, data-adaptive atom)
    # from the GPU's histogram: same selection as the oracle's, and as an atom it serves the layer better
    # than the free fit or NF4 snapped to the same grid
    M, K, g, H = 512, 4096, 16, 1024
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 7300, row_sigma=0.5, outlier_frac=0.001))
    c = si.channel_norms(K, 1.0, 7301)
    hist = gpu_hist(W, c, g, H, True)
    assert np.array_equal(hist, DD.histogram(W, c, g, H))
    grid = sop.sop_weight_grid(sop.WeightFmt(4, 3, -1, -1))
    cand = grid / grid[-1]
    idx, cost = sop.sop_dd_fit_grid(hist, cand, 16)
    ridx, rcost = DD.fit_grid(hist, cand, 16)
    assert abs(cost - rcost) <= 1e-11 * rcost and np.array_equal(idx, ridx)
    dd_grid = cand[idx].astype(np.float32)
    free = sop.sop_dd_fit(hist, 16, 20, sop.sop_atom_nf(4)).astype(np.float64)
    snapped = np.unique(cand[np.abs(cand[None, :] - free[:, None]).argmin(axis=1)]).astype(np.float32)
    nf = sop.sop_atom_nf(4).astype(np.float64)
    nf_snapped = np.unique(cand[np.abs(cand[None, :] - nf[:, None]).argmin(axis=1)]).astype(np.float32)
    assert snapped.size == 16 and nf_snapped.size == 16
    tabs = [sop.sop_atom_nf(4), dd_grid, snapped, nf_snapped]
    fmt = sop.fmt_by_name("UE4M4")
    gpu = run_gpu(W, c, tabs, g, fmt, bf16=True, emit=True)
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt))
    assert np.array_equal(gpu["sel_words"], ref.sel_words) and np.array_equal(gpu["scale_code"], ref.scale_code)
    for a in range(4):
        assert np.array_equal(gpu["codes"][a], ref.codes[a])
    assert np.max(np.abs(gpu["acos_atom"] - ref.acos_atom)) <= 1e-6
    # among codebooks that live on the E4M3 grid, the one selected on the grid serves the layer best
    # (the unconstrained NF4 table, which no E4M3 LUT can hold, is better still)
    assert gpu["acos_atom"][1] > gpu["acos_atom"][2] and gpu["acos_atom"][1] > gpu["acos_atom"][3]
