"""GPU parity of the kernel variants built for alphabets of one or two atoms (the scoring call of step 2,
the two-atom search of step 4 and the materialisation): every block size, both weight types, unsigned,
signed and argmax scales, all metrics, with and without the per-block outputs."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, pairsearch as ops
import sop_inputs as si
from gpu_util import run_gpu, compare, oracle_fmt

pytestmark = pytest.mark.gpu


def layer(M, K, seed, bf16):
    W = si.student_t_weights(M, K, 4.0, seed, row_sigma=0.5, outlier_frac=0.002)
    if bf16:
        W = si.bf16_round(W)
    W[1, :] = 0.0
    W[2, :64] = np.abs(W[2, :64])
    return W, si.channel_norms(K, 1.0, seed + 1)


@pytest.mark.parametrize("g", [8, 16, 32, 64])
@pytest.mark.parametrize("bf16", [False, True])
def test_one_and_two_atoms(g, bf16):
    M, K = 33, 1088
    W, c = layer(M, K, 7100 + g, bf16)
    sets = ([OA.to_f32(OA.sh(4))], [OA.to_f32(OA.nf(4)), OA.to_f32(OA.negate(OA.sh(4)))], [OA.to_f32(OA.nf(5)), OA.to_f32(OA.nf(4))])
    for tabs in sets:
        for fmtname, rule in (("UE4M4", 0), ("E4M3", 0), ("S1E5M5", 1)):
            fmt = sop.fmt_by_name(fmtname)
            for emit in (True, False):
                gpu = run_gpu(W, c, tabs, g, fmt, k=1, bf16=bf16, emit=emit, scale_rule=rule)
                ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), k=1, scale_rule=rule)
                compare(gpu, ref, len(tabs) * (len(tabs) - 1) // 2, emit=emit)


@pytest.mark.parametrize("metric", [sop.SEL_COS, sop.SEL_MSE])
def test_metrics(metric):
    M, K, g = 40, 512, 16
    W, c = layer(M, K, 7200, True)
    tabs = [OA.to_f32(OA.nf(4)), OA.to_f32(OA.sh(4))]
    for fmtname in ("UE4M4", "E4M3"):
        fmt = sop.fmt_by_name(fmtname)
        for emit in (True, False):
            gpu = run_gpu(W, c, tabs, g, fmt, metric=metric, bf16=True, emit=emit)
            ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), metric=metric)
            compare(gpu, ref, 1, emit=emit)
