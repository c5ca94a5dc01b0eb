"""GPU parity of the per-layer scale shift: exponent histogram of the block scales (bit-exact), the
chosen shift, and the pair search run with it."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import flayer as FL, pairsearch as ops
import sop_inputs as si
from gpu_util import run_gpu, compare, oracle_fmt, ctx, cached_config

pytestmark = pytest.mark.gpu


def gpu_hist(W, g, tp, tn, fmt, bf16):
    import torch
    Wt = torch.from_numpy(W).cuda()
    if bf16:
        Wt = Wt.to(torch.bfloat16)
    h = ctx().scale_histogram(Wt, g, tp, tn, fmt)
    torch.cuda.synchronize()
    return h.cpu().numpy()


@pytest.mark.parametrize("g", [8, 16, 32, 64])
@pytest.mark.parametrize("bf16", [False, True])
def test_exponent_histogram(g, bf16):
    M, K = 37, 1088
    W = si.student_t_weights(M, K, 4.0, 950 + g, row_sigma=1.5, scale=2.0 ** -8)
    W[3, :] = 0.0                                                     # zero scales are not counted
    W[4, :64] = np.float32(1e-41)                                     # binary32 subnormals
    W[5, :] *= np.float32(1e30)
    if bf16:
        W = si.bf16_round(W)
    for name, tp, tn in (("UE4M4", 1.0, 1.0), ("E4M3", 0.98139, 1.0), ("S1E5M5", 1.0, 0.98139)):
        f = sop.fmt_by_name(name)
        sc = FL.block_scales(W, g, tp, tn)
        ref = FL.exponent_histogram(sc, f.exp_bits, f.man_bits, f.bias, f.max_code)
        got = gpu_hist(W, g, tp, tn, f, bf16)
        assert np.array_equal(got, ref)
        k, frac = sop.sop_layer_shift(got, sc.size, f)
        assert (k, frac) == FL.layer_shift(sc, f.exp_bits, f.man_bits, f.bias, f.max_code)


def test_shift_feeds_the_pair_search():
    # small-magnitude weights: UE4M4 without a shift stores most block scales as subnormals
    M, K, g = 64, 2048, 16
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 961, row_sigma=0.5, scale=2.0 ** -9))
    c = si.channel_norms(K, 1.0, 962)
    f = sop.fmt_by_name("UE4M4")
    tabs = sop.build_alphabet(["NF4", "SH4", "-NF4", "-SH4"])
    h = gpu_hist(W, g, 1.0, 1.0, f, True)
    k, frac = sop.sop_layer_shift(h, M * K // g, f)
    assert k >= 3 and frac > 0.99
    with_shift = run_gpu(W, c, tabs, g, f, k=k, bf16=True)
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(f), k=k)
    compare(with_shift, ref, 6)
    without = run_gpu(W, c, tabs, g, f, k=0, bf16=True)
    assert np.all(with_shift["acos_atom"] > without["acos_atom"] + 1e-4)


def test_full_layer_and_errors():
    import torch
    W, c, cfg = cached_config("C3_down")
    f = sop.fmt_by_name("UE4M4")
    sc = FL.block_scales(W, 16, 1.0, 1.0)
    got = gpu_hist(W, 16, 1.0, 1.0, f, True)
    assert np.array_equal(got, FL.exponent_histogram(sc, 4, 4))
    assert np.array_equal(got, gpu_hist(W, 16, 1.0, 1.0, f, True))
    assert sop.sop_layer_shift(got, sc.size, f) == FL.layer_shift(sc, 4, 4)
    Wt = torch.zeros((4, 128), device="cuda")
    with pytest.raises(sop.SopError) as e:
        ctx().scale_histogram(Wt, 16, 0.0, 1.0, f)
    assert e.value.status == 3
    with pytest.raises(sop.SopError) as e:
        ctx().scale_histogram(Wt, 16, 1.0, 1.0, sop.ScaleFmt(0, 9, 4, 16, -1, -1))
    assert e.value.status == 4
