"""GPU parity: the HIP path against the CPU oracle on the same seeded tensors, through the C ABI.

Bar: codes, scale codes (with sign), selector bits and block scores bit-exact; every ACos within
1e-6 absolute (the tolerance the benchmark spec fixes)."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, pairsearch as ops
import sop_inputs as si
from gpu_util import run_gpu, compare, oracle_fmt, ctx

pytestmark = pytest.mark.gpu


def tabs_for(names, draws_seed=4242):
    draws = si.normal_draws(1 << 18, draws_seed) if any("BOF" in n for n in names) else None
    return sop.build_alphabet(names, bof_draws=draws)


def check(W, c, tabs, g, fmt, *, k=0, metric=0, pairs=None, bf16=False, ldw=None):
    gpu = run_gpu(W, c, tabs, g, fmt, k=k, metric=metric, pairs=pairs, bf16=bf16, ldw=ldw)
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), k=k, metric=metric,
                          pairs=None if pairs is None else np.asarray(pairs, dtype=np.int32))
    P = len(tabs) * (len(tabs) - 1) // 2 if pairs is None else len(pairs)
    compare(gpu, ref, P)
    return gpu, ref


def test_config1_full():
    W, c, cfg = si.make_config("C1")
    gpu, ref = check(W, c, tabs_for(cfg["atoms"]), cfg["g"], sop.fmt_by_name(cfg["fmt"]))
    assert 0.99 < gpu["acos_pair"].min() < 1.0


@pytest.mark.parametrize("g", [8, 16, 32, 64])
@pytest.mark.parametrize("fmt", ["UE4M4", "E4M3", "S1E5M5"])
@pytest.mark.parametrize("bf16", [False, True])
def test_block_sizes_formats_dtypes_ragged(g, fmt, bf16):
    # K = 1088 = 17*64: a ragged last strip for every block size; 37 rows: ranges that split rows unevenly
    M, K = 37, 1088
    W = si.student_t_weights(M, K, 4.0, 100 + g, row_sigma=0.5, outlier_frac=0.002)
    if bf16:
        W = si.bf16_round(W)
    c = si.channel_norms(K, 1.0, 200 + g)
    check(W, c, tabs_for(["NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4"]), g, sop.fmt_by_name(fmt), bf16=bf16)


@pytest.mark.parametrize("fmt", ["UE4M6", "E4M5", "UE5M7", "E5M6", "E4M7", "E8M7", "UE4M3", "S0E6M5"])
def test_scale_format_sweep(fmt):
    M, K = 64, 2048
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 301, row_sigma=1.0))
    c = si.channel_norms(K, 1.0, 302)
    check(W, c, tabs_for(["NF4", "SH4", "-SH4"]), 16, sop.fmt_by_name(fmt), bf16=True)


def test_five_bit_and_mixed_alphabets():
    M, K = 48, 1536
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 401))
    c = si.channel_norms(K, 1.0, 402)
    check(W, c, tabs_for(["NF5", "SH5", "-NF5", "-SH5"]), 16, sop.fmt_by_name("UE4M4"), bf16=True)
    check(W, c, tabs_for(["NF4", "SH5", "BOF4", "-NF5"]), 32, sop.fmt_by_name("E4M3"), bf16=True)
    e2m3 = OA.to_f32(OA.exmy_grid(2, 3))                             # 63-entry FP6 grid as an atom
    check(W, c, [e2m3, sop.sop_atom_nf(4)], 16, sop.fmt_by_name("UE4M4"), bf16=True)
    three = np.array([-1.0, 0.0, 0.5], dtype=np.float32)             # tiny asymmetric atom
    check(W, c, [three, sop.sop_atom_negate(three)], 8, sop.fmt_by_name("E4M3"), bf16=True)


def test_eight_atoms_and_pair_subset():
    M, K = 32, 1024
    W = si.student_t_weights(M, K, 5.0, 501, row_sigma=0.5)
    c = si.channel_norms(K, 1.0, 502)
    names = ["NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4", "NF5", "SH5"]
    check(W, c, tabs_for(names), 16, sop.fmt_by_name("UE4M4"))
    check(W, c, tabs_for(names), 16, sop.fmt_by_name("UE4M4"), pairs=[(2, 5), (0, 7), (0, 1)])
    check(W, c, tabs_for(names[:1]), 16, sop.fmt_by_name("UE4M4"))   # one atom, no pair


def test_unweighted_metric_and_layer_shift():
    M, K = 40, 1024
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 601, row_sigma=0.5, scale=2.0 ** -9))
    c = si.channel_norms(K, 1.0, 602)
    t = tabs_for(["NF4", "SH4", "-NF4", "-SH4"])
    check(W, c, t, 16, sop.fmt_by_name("UE4M4"), metric=sop.SEL_MSE, bf16=True)
    check(W, c, t, 16, sop.fmt_by_name("UE4M4"), k=9, bf16=True)       # shifted into the normal range
    check(W, c, t, 16, sop.fmt_by_name("UE4M4"), k=0, bf16=True)       # subnormal scale codes
    check(W, c, t, 32, sop.fmt_by_name("E4M3"), k=-3, metric=sop.SEL_MSE, bf16=True)


@pytest.mark.parametrize("g,fmt", [(8, "UE4M4"), (16, "UE4M4"), (16, "E4M3"), (32, "E4M3"), (64, "UE4M6")])
def test_cosine_metric(g, fmt):
    # finishing reassignment by per-block cosine: decisions from the binary32 numerator / denominator sums
    M, K = 33, 1088
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 650 + g, row_sigma=0.5, outlier_frac=0.002))
    W[3, 64:96] = 0.0
    c = si.channel_norms(K, 1.0, 651)
    c[128:160] = 0.0
    t = tabs_for(["NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4"])
    gpu, ref = check(W, c, t, g, sop.fmt_by_name(fmt), metric=sop.SEL_COS, bf16=True)
    # selecting by cosine, a pair is never worse than either of its atoms
    pairs = [(a, b) for a in range(6) for b in range(a + 1, 6)]
    for p, (a, b) in enumerate(pairs):
        assert gpu["acos_pair"][p] >= max(gpu["acos_atom"][a], gpu["acos_atom"][b]) - 1e-6


def test_row_stride():
    M, K = 16, 512
    W = si.student_t_weights(M, K, 4.0, 701)
    c = si.channel_norms(K, 1.0, 702)
    check(W, c, tabs_for(["NF4", "SH4"]), 16, sop.fmt_by_name("UE4M4"), ldw=K + 64)


@pytest.mark.parametrize("M,K,g,bf16", [(192, 1040, 16, True),    # 65 lanes a row: 64 rows walked as one fill 65 strips
                                         (6, 1040, 16, False),     # 6 rows: two rows at a time at most
                                         (7, 1040, 16, True),      # an odd number of rows: no folding
                                         (48, 1032, 8, False),     # lanes of 8 elements, 129 a row
                                         (40, 2112, 32, True),     # two lanes a block, 132 lanes a row
                                         (16, 4160, 64, True)])    # four lanes a block, 260 lanes a row
def test_rows_walked_as_one(M, K, g, bf16):
    """Rows that lie back to back are walked several at a time where that fills the last 64-lane strip of a row better;
    every per-block output keeps its place and the channel norm of a column is the one of its index within the true row."""
    W = si.student_t_weights(M, K, 4.0, 9100 + M)
    if bf16:
        W = si.bf16_round(W)
    c = si.channel_norms(K, 1.0, 9200 + K)
    tabs = tabs_for(["NF4", "SH4", "-NF4"])
    check(W, c, tabs, g, sop.fmt_by_name("UE4M4"), bf16=bf16)
    check(W, c, tabs, g, sop.fmt_by_name("E4M3"), bf16=bf16)
    check(W, c, tabs, g, sop.fmt_by_name("UE4M4"), bf16=bf16, ldw=K + 32)      # rows apart: no folding, same results


def test_degenerate_blocks():
    rng = np.random.default_rng(9)
    M, K, g = 8, 512, 16
    W = si.student_t_weights(M, K, 4.0, 801)
    W[0, :] = 0.0                                   # all-zero row
    W[1, 16:32] = 0.0
    W[1, 20] = 3.0                                  # single non-zero in a block
    W[2, :] = 1e-15                                 # underflows the scale formats: code 0, cosine 0
    W[3, :] *= 1e6                                  # saturates UE4M4's largest scale
    W[5, 32:48] = -W[5, 32:48].__abs__()            # one-signed block
    c = si.channel_norms(K, 1.0, 802)
    c[64:80] = 0.0                                  # a block with zero channel norms
    c[100] = 0.0
    t = tabs_for(["NF4", "SH4", "-NF4", "-SH4"])
    for fmt in ("UE4M4", "E4M3"):
        check(W, c, t, g, sop.fmt_by_name(fmt))
    # exactly representable weights: ACos is 1 and every score is 0
    L = si.bf16_round(sop.sop_atom_nf(4))
    f = sop.fmt_by_name("UE4M4")
    of = oracle_fmt(f)
    q = rng.integers(20, 250, size=(M, K // g))
    s = np.array([[ops.scale_value(of, int(v)) for v in row] for row in q])
    kk = rng.integers(0, 16, size=(M, K // g, g))
    kk[:, :, 0], kk[:, :, 1] = 15, 0
    Wx = (s[:, :, None] * L[kk].astype(np.float64)).reshape(M, K).astype(np.float32)
    gpu, ref = check(Wx, c, [L, sop.sop_atom_sh(4)], g, f)
    assert np.all(gpu["blk_err"][0] == 0.0) and abs(gpu["acos_atom"][0] - 1.0) < 1e-7


def test_vanishing_weights_integer_outputs():
    # Weights so small that c*w^2 leaves binary32's range: the cosine VALUE of such blocks is outside
    # the library's contract (its fp32 norm underflows), every integer output is still exact.
    M, K, g = 4, 256, 16
    W = si.student_t_weights(M, K, 4.0, 811)
    W[0, :] = 1e-30
    W[1, :64] = np.float32(1e-41)                   # binary32 subnormals
    W[2, :] *= np.float32(1e-38)
    c = si.channel_norms(K, 1.0, 812)
    t = tabs_for(["NF4", "SH4", "-NF4", "-SH4"])
    for fmt, k in (("UE4M4", 0), ("E8M7", 0), ("E4M3", 60)):
        f = sop.fmt_by_name(fmt)
        gpu = run_gpu(W, c, t, g, f, k=k)
        ref = ops.pair_search(W, c, t, g, oracle_fmt(f), k=k)
        assert np.array_equal(gpu["scale_code"], ref.scale_code)
        assert all(np.array_equal(x, y) for x, y in zip(gpu["codes"], ref.codes))
        assert np.array_equal(gpu["blk_err"], ref.blk_err) and np.array_equal(gpu["sel_words"], ref.sel_words)


def test_midpoint_ties():
    # weights placed exactly on code midpoints after scaling by a power-of-two scale
    L = np.array([-1, -0.5, 0, 0.25, 0.5, 1], dtype=np.float32)
    mids = (L[:-1] + L[1:]) / 2
    M, K, g = 4, 256, 16
    rng = np.random.default_rng(2)
    W = np.empty((M, K), dtype=np.float32)
    for b in range(M * K // g):
        s = 2.0 ** rng.integers(-3, 4)
        blk = rng.choice(np.concatenate([mids, L]), size=g) * s
        blk[0] = s                                   # absmax element pins the scale
        W.reshape(-1, g)[b] = blk
    c = np.ones(K, dtype=np.float32)
    check(W, c, [L, sop.sop_atom_negate(L)], g, sop.fmt_by_name("E4M3"))
    check(W, c, [L, sop.sop_atom_negate(L)], g, sop.fmt_by_name("UE4M4"))


def test_deterministic():
    W, c, cfg = si.make_config("C1")
    t = tabs_for(cfg["atoms"])
    a = run_gpu(W, c, t, 16, sop.fmt_by_name("UE4M4"))
    b = run_gpu(W, c, t, 16, sop.fmt_by_name("UE4M4"))
    assert np.array_equal(a["acos_pair"], b["acos_pair"]) and np.array_equal(a["sel_words"], b["sel_words"])
    assert np.array_equal(a["blk_cos"], b["blk_cos"])


def test_argument_errors():
    import torch
    cx = ctx()
    cx.set_alphabet(tabs_for(["NF4", "SH4"]))
    W = torch.zeros((4, 128), device="cuda")
    c = torch.ones(128, device="cuda")
    f = sop.fmt_by_name("UE4M4")
    for g in (12, 128):
        with pytest.raises(sop.SopError) as e:
            cx.pair_search(W, c, g, f)
        assert e.value.status == 2
    with pytest.raises(sop.SopError) as e:
        cx.pair_search(W[:, :120], c[:120], 16, f)                   # g does not divide K
    assert e.value.status == 2
    with pytest.raises(sop.SopError) as e:
        cx.pair_search(W, c, 16, sop.ScaleFmt(0, 9, 4, 16, -1, -1))
    assert e.value.status == 4
    with pytest.raises(sop.SopError) as e:
        cx.pair_search(W, c, 16, sop.fmt_by_name("UE4M4"), k=100)
    assert e.value.status == 4
    with pytest.raises(sop.SopError) as e:
        cx.pair_search(W, c, 16, f, metric=7)
    assert e.value.status == 1
    with pytest.raises(sop.SopError) as e:
        cx.set_alphabet([np.array([0.5, -0.5], dtype=np.float32)])
    assert e.value.status == 3
    with pytest.raises(sop.SopError) as e:
        cx.set_pairs([(1, 0)])
    assert e.value.status == 1
    with pytest.raises(sop.SopError) as e:
        cx.pair_search(W.cpu(), c.cpu(), 16, f)
    assert e.value.status == 1
