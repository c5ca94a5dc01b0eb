"""GPU parity of the layer-scope weight formats and of the FP6-block versus FP8-layer comparison:
scale code and every weight's grid index bit-exact against the oracle, error sums to 1e-6 relative
(the kernel forms the products and the sums of one step in binary32, the oracle everything in binary64)."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import layerscope as LS, pairsearch as ops
import sop_inputs as si
from gpu_util import run_gpu, oracle_fmt, ctx, cached_config

pytestmark = pytest.mark.gpu

# power-of-two scales 2^-126 .. 2^125 (the top two exponents are left out: their reciprocals are not normal binary32 numbers)
UE8M0 = sop.ScaleFmt(0, 8, 0, 8, 127, 252)


def run(W, c, wfmt, sfmt, k=0, bf16=True):
    import torch
    Wt = torch.from_numpy(W).cuda()
    if bf16:
        Wt = Wt.to(torch.bfloat16)
    ct = None if c is None else torch.from_numpy(c).cuda()
    out, codes = ctx().layer_scope_error(Wt, ct, wfmt, sfmt, k, want_codes=True)
    torch.cuda.synchronize()
    return out.cpu().numpy(), codes.cpu().numpy().view(np.uint16).astype(np.int32)


def check(W, c, wf, sf, k=0, bf16=True):
    out, codes = run(W, c, sop.WeightFmt(*wf), sf, k, bf16)
    tab = LS.exmy_table(*wf)
    ref = LS.layer_scope(W, c, tab, oracle_fmt(sf), k)
    assert int(out[3]) == ref["q"], (out[3], ref["q"])
    assert np.array_equal(codes, ref["codes"])
    for got, want in ((out[0], ref["err_w"]), (out[1], ref["err_u"]), (out[2], ref["wn"])):
        assert abs(got - want) <= 1e-6 * abs(want) + 1e-300, (got, want)
    return out, ref


@pytest.mark.parametrize("bf16", [False, True])
def test_formats_and_scales(bf16):
    M, K = 37, 1096                                                   # ragged last strip
    W = si.student_t_weights(M, K, 4.0, 970, row_sigma=0.5, outlier_frac=0.002, scale=0.03)
    if bf16:
        W = si.bf16_round(W)
    c = si.channel_norms(K, 1.0, 971)
    check(W, c, (4, 3, -1, -1), UE8M0, bf16=bf16)                     # E4M3^0sUE8M0
    check(W, c, (4, 3, -1, 0x7E), UE8M0, bf16=bf16)                   # top code reserved
    check(W, None, (2, 3, -1, -1), sop.fmt_by_name("UE4M4"), k=5, bf16=bf16)
    check(W, c, (5, 6, -1, -1), sop.fmt_by_name("E8M7"), bf16=bf16)   # E5M6^ with a 16-bit layer scale
    check(W, c, (3, 4, -1, -1), sop.fmt_by_name("UE5M3"), bf16=bf16)
    out, _ = check(W * np.float32(0.0), c, (4, 3, -1, -1), UE8M0, bf16=bf16)   # all-zero layer
    assert out[0] == 0.0 and out[3] == 0.0


def test_ties_saturation_and_bf16_identity():
    tab = LS.exmy_table(4, 3)
    mids = ((tab[:-1] + tab[1:]) / 2).astype(np.float32)
    rng = np.random.default_rng(8)
    W = rng.choice(np.concatenate([mids, tab.astype(np.float32)]), size=(16, 256)).astype(np.float32)
    W[0, 0] = 480.0                                                   # pins the scale to 1
    out, ref = check(W, None, (4, 3, -1, -1), UE8M0, bf16=False)
    assert ref["s"] == 1.0
    W2 = W * np.float32(1.4)                                          # ideal scale 1.4 -> 1: the top values saturate
    check(W2, None, (4, 3, -1, -1), UE8M0, bf16=False)
    # (the grid's top value is about 2^126: weights of the order 2^40 keep the layer scale inside UE8M0's range)
    Wb = si.bf16_round(si.student_t_weights(32, 512, 4.0, 972, scale=2.0 ** 40))
    Wb[0, 0] = np.float32(2.0 ** 46) * np.float32(LS.exmy_table(8, 7, 119, 244 * 128 + 127)[-1] / 2.0 ** 125)   # layer scale exactly 2^-79
    out, _ = check(Wb, si.channel_norms(512, 1.0, 973), (8, 7, 119, 244 * 128 + 127), UE8M0)
    assert out[0] == 0.0 and out[1] == 0.0                            # bf16 weights sit on the E8M7 grid: no error


def test_sum_kernel():
    import torch
    rng = np.random.default_rng(9)
    for n in (1, 255, 4097, 3_000_001):
        x = (rng.standard_normal(n) * 10.0 ** rng.uniform(-6, 6, size=n)).astype(np.float32)
        got = ctx().sum_f32(torch.from_numpy(x).cuda())
        torch.cuda.synchronize()
        ref = float(x.astype(np.float64).sum())
        assert abs(got.item() - ref) <= 1e-12 * float(np.abs(x).astype(np.float64).sum())


def test_fp6_block_scaled_versus_fp8_layer_scaled_full_layer():
    # the paper's operating-point comparison on the 70B-shaped layer of configuration 5:
    # E2M3sUE4M4 (g = 16, 6.5 bpw) against E4M3^0sUE8M0 (8.0 bpw), weighted reconstruction error
    import torch
    W, c, cfg = cached_config("C5")
    g = 16
    e2m3 = LS.exmy_table(2, 3).astype(np.float32)
    ue4m4 = sop.fmt_by_name("UE4M4")
    cx = ctx()
    Wt = torch.from_numpy(W).cuda().to(torch.bfloat16)
    ct = torch.from_numpy(c).cuda()
    # per-layer shift for the 4-exponent-bit block scale, then the block-scaled search with the FP6 grid as the atom
    h = cx.scale_histogram(Wt, g, 7.5, 7.5, ue4m4)
    torch.cuda.synchronize()
    k, _ = sop.sop_layer_shift(h.cpu().numpy(), W.size // g, ue4m4)
    cx.set_alphabet([e2m3])
    cx.set_pairs(None)
    o = cx.alloc_outputs(W.shape[0], W.shape[1], g, emit=True)
    cx.pair_search(Wt, ct, g, ue4m4, k=k, out=o)
    fp6 = cx.sum_f32(o.blk_err.reshape(-1))
    fp8, _ = cx.layer_scope_error(Wt, ct, sop.WeightFmt(4, 3, -1, -1), UE8M0)
    torch.cuda.synchronize()
    fp6, fp8 = fp6.item(), fp8.cpu().numpy()
    rows = np.sort(np.random.default_rng(11).choice(W.shape[0], 128, replace=False))
    ref6 = ops.pair_search(W[rows], c, [e2m3], g, oracle_fmt(ue4m4), k=k, want_codes=False)
    Bk = W.shape[1] // g
    assert np.array_equal(o.blk_err.cpu().numpy().reshape(W.shape[0], Bk)[rows].reshape(-1), ref6.blk_err[0])
    ref8 = LS.layer_scope(W, c, LS.exmy_table(4, 3), oracle_fmt(UE8M0))
    assert int(fp8[3]) == ref8["q"] and abs(fp8[0] - ref8["err_w"]) <= 1e-6 * ref8["err_w"]
    full6 = float(o.blk_err.cpu().numpy().astype(np.float64).sum())
    assert abs(fp6 - full6) <= 1e-12 * full6
    assert fp6 < fp8[0]                                               # block-scaled FP6 wins at 1.5 bpw less


@pytest.mark.parametrize("bf16", [False, True])
def test_one_negative_weight_in_a_small_layer(bf16):
    """A layer so small that many wavefronts of the maxima pass have no work, and whose weights are all positive but one:
    the largest negative magnitude must reach the layer's scale wherever that weight sits (a wavefront without negative
    weights once handed on -0, whose bit pattern erased the running maximum it was joined with)."""
    M, K = 27, 1408
    base = np.full((M, K), 1.0 / 1024, np.float32)
    for r, c0 in ((0, 0), (5, 700), (13, 64), (26, 933), (26, 1407), (20, 3)):
        W = base.copy(); W[r, c0] = -0.5
        check(W, None, (3, 4, -1, -1), sop.fmt_by_name("UE4M4"), k=3, bf16=bf16)
        check(-W, None, (4, 3, -1, -1), UE8M0, bf16=bf16)
    check(base, None, (3, 4, -1, -1), sop.fmt_by_name("UE4M4"), k=3, bf16=bf16)          # no negative weight at all
