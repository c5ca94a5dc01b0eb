"""GPU parity of the argmax scale rule against the oracle: every integer output bit for bit, ACos
within 1e-6."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, pairsearch as ops
import sop_inputs as si
from gpu_util import run_gpu, compare, oracle_fmt, ctx

pytestmark = pytest.mark.gpu


def alphabet():
    lop = np.array([-0.4, -0.3, -0.2, -0.1, -0.05, 0.0, 0.04, 0.1, 0.17, 0.25, 0.35, 0.47, 0.6, 0.75, 0.9, 1.0])
    return [OA.to_f32(OA.nf(4)), OA.to_f32(OA.sh(4)), OA.to_f32(OA.negate(OA.sh(4))), OA.to_f32(lop),
            OA.to_f32(OA.negate(lop)), OA.to_f32(OA.nf(5))]


@pytest.mark.parametrize("g", [8, 16, 32, 64])
@pytest.mark.parametrize("bf16", [False, True])
def test_block_sizes_dtypes_ragged(g, bf16):
    M, K = 37, 1088
    W = si.student_t_weights(M, K, 4.0, 4100 + g, row_sigma=0.5, outlier_frac=0.002)
    if bf16:
        W = si.bf16_round(W)
    W[3, :] = 0.0
    W[5, :64] = np.abs(W[5, :64])                                     # one-sided blocks
    W[6, :64] = -np.abs(W[6, :64])
    W[7, 0], W[7, 1] = 0.75, -0.75                                    # the dominant element ties in magnitude
    c = si.channel_norms(K, 1.0, 4101)
    tabs = alphabet()
    fmt = sop.fmt_by_name("S1E5M5")
    gpu = run_gpu(W, c, tabs, g, fmt, k=1, bf16=bf16, scale_rule=sop.SCALE_ARGMAX)
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), k=1, scale_rule=ops.ARGMAX)
    compare(gpu, ref, 15)
    # the rule does something: signs both ways, and results that differ from absmax with both signs
    sgn = ref.scale_code[1] >> 15
    assert 0.2 < sgn.mean() < 0.8
    both = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), k=1)
    assert not np.array_equal(both.blk_err[3], ref.blk_err[3])


@pytest.mark.parametrize("metric", [sop.SEL_WSE, sop.SEL_COS, sop.SEL_MSE])
@pytest.mark.parametrize("fmtname", ["E4M3", "E8M7"])
def test_metrics_and_scale_words(metric, fmtname):
    M, K, g = 48, 512, 16
    W = si.bf16_round(si.student_t_weights(M, K, 5.0, 4200, row_sigma=0.8))
    c = si.channel_norms(K, 1.2, 4201)
    tabs = alphabet()
    fmt = sop.fmt_by_name(fmtname)
    for emit in (True, False):
        gpu = run_gpu(W, c, tabs, g, fmt, metric=metric, bf16=True, emit=emit, scale_rule=sop.SCALE_ARGMAX)
        ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), metric=metric, scale_rule=ops.ARGMAX)
        compare(gpu, ref, 15, emit=emit)


def test_eight_atoms_and_saturating_scale():
    M, K, g = 24, 1024, 16
    W = si.student_t_weights(M, K, 3.0, 4300, row_sigma=1.5, outlier_frac=0.01)
    W[:4] *= np.float32(300.0)                                        # beyond E4M3's largest scale: the word saturates
    W[4:8] *= np.float32(1e-4)                                        # subnormal scale words
    W = si.bf16_round(W)
    c = si.channel_norms(K, 1.0, 4301)
    tabs = alphabet() + [OA.to_f32(OA.negate(OA.nf(4))), OA.to_f32(OA.exmy_grid(2, 1))]
    fmt = sop.fmt_by_name("E4M3")
    gpu = run_gpu(W, c, tabs, g, fmt, bf16=True, scale_rule=sop.SCALE_ARGMAX)
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), scale_rule=ops.ARGMAX)
    compare(gpu, ref, 28)


def test_unsigned_scale_word_is_refused_and_rule_resets():
    import torch
    cx = ctx()
    cx.set_alphabet(alphabet()[:2]); cx.set_pairs(None)
    W = torch.zeros((8, 256), dtype=torch.bfloat16, device="cuda")
    c = torch.ones(256, dtype=torch.float32, device="cuda")
    cx.set_scale_rule(sop.SCALE_ARGMAX)
    try:
        with pytest.raises(sop.SopError) as ei:
            cx.pair_search(W, c, 16, sop.fmt_by_name("UE4M4"))
        assert ei.value.status == 4
        with pytest.raises(sop.SopError):
            cx.set_scale_rule(7)
    finally:
        cx.set_scale_rule(sop.SCALE_ABSMAX)
    cx.pair_search(W, c, 16, sop.fmt_by_name("UE4M4"))
    torch.cuda.synchronize()
