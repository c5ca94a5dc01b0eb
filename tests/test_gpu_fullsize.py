"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py
times (search mode, no per-block outputs) and in emit mode on row samples."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import pairsearch as ops
import sop_inputs as si
from gpu_util import run_gpu, compare, oracle_fmt

pytestmark = pytest.mark.gpu


def _alphabet(names):
    return sop.build_alphabet(names, bof_draws=si.normal_draws(1 << 20, 4242))


def _sample_rows_check(W, c, tabs, g, fmt, gpu_full, rows, bf16):
    """Oracle on a row sample; the full-layer GPU outputs of those rows must match bit for bit."""
    M, K = W.shape
    Bk = K // g
    ref = ops.pair_search(W[rows], c, tabs, g, oracle_fmt(fmt))
    assert np.array_equal(gpu_full["sel_words"].reshape(M, Bk)[rows].reshape(-1), ref.sel_words)
    if "scale_code" in gpu_full:
        sc = gpu_full["scale_code"].reshape(len(tabs), M, Bk)[:, rows].reshape(len(tabs), -1)
        assert np.array_equal(sc, ref.scale_code)
        be = gpu_full["blk_err"].reshape(len(tabs), M, Bk)[:, rows].reshape(len(tabs), -1)
        assert np.array_equal(be, ref.blk_err)
        for a in range(len(tabs)):
            per_row = K // 2 if tabs[a].size <= 16 else K
            assert np.array_equal(gpu_full["codes"][a].reshape(M, per_row)[rows].reshape(-1), ref.codes[a])


def test_config2_full_signed():
    W, c, cfg = si.make_config("C2")
    tabs = _alphabet(cfg["atoms"])
    fmt = sop.fmt_by_name(cfg["fmt"])
    gpu = run_gpu(W, c, tabs, 16, fmt, bf16=True, emit=False)
    ref = ops.pair_search(W, c, tabs, 16, oracle_fmt(fmt), want_codes=False)
    compare(gpu, ref, 15, emit=False)
    # signed scale: an atom and its negation reach the same candidates
    assert np.max(np.abs(gpu["acos_atom"][:3] - gpu["acos_atom"][3:])) < 1e-6
    rows = np.sort(np.random.default_rng(1).choice(W.shape[0], 96, replace=False))
    gpu_e = run_gpu(W, c, tabs, 16, fmt, bf16=True, emit=True)
    _sample_rows_check(W, c, tabs, 16, fmt, gpu_e, rows, True)


@pytest.mark.parametrize("name", ["C3_down", "C3_up"])
def test_config3_headline_full(name):
    W, c, cfg = si.make_config(name)
    tabs = _alphabet(cfg["atoms"])
    fmt = sop.fmt_by_name(cfg["fmt"])
    gpu = run_gpu(W, c, tabs, 16, fmt, bf16=True, emit=False)        # the configuration bench.py times
    ref = ops.pair_search(W, c, tabs, 16, oracle_fmt(fmt), want_codes=False)
    compare(gpu, ref, 15, emit=False)


@pytest.mark.parametrize("g,fmt", [(8, "E4M5"), (32, "UE5M7"), (64, "S1E5M5")])
def test_config3_sweep_samples(g, fmt):
    W, c, cfg = si.make_config("C3_down", rows=512)
    tabs = _alphabet(["NF5", "SH5", "BOF5", "-NF5", "-SH5", "-BOF5"])
    f = sop.fmt_by_name(fmt)
    gpu = run_gpu(W, c, tabs, g, f, bf16=True, emit=True)
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(f))
    compare(gpu, ref, 15)


def test_config5_shape_row_sample():
    # 70B-shaped MLP layer 28672 x 8192: search mode on the full layer, oracle on sampled rows and
    # on the layer mean through the property  mean over rows of sampled per-row results
    W, c, cfg = si.make_config("C5", rows=28672)
    tabs = _alphabet(cfg["atoms"])
    fmt = sop.fmt_by_name(cfg["fmt"])
    gpu = run_gpu(W, c, tabs, 16, fmt, bf16=True, emit=False)
    rows = np.sort(np.random.default_rng(5).choice(W.shape[0], 256, replace=False))
    _sample_rows_check(W, c, tabs, 16, fmt, gpu, rows, True)
    # the sampled rows' ACos is an unbiased estimate of the layer's: agree to sampling accuracy
    ref = ops.pair_search(W[rows], c, tabs, 16, oracle_fmt(fmt), want_codes=False)
    assert np.max(np.abs(gpu["acos_pair"] - ref.acos_pair)) < 2e-4
    assert np.all((gpu["acos_pair"] > 0.99) & (gpu["acos_pair"] <= 1.0))


def test_config4_one_block_full_size_through_the_model_wide_call():
    """The seven layers of a 7B-shaped block at their full sizes in one model-wide call (the launch
    bench.py --workload model times, on one block): the ACos table equals the single calls' bit for bit,
    the selector words of sampled rows equal the oracle's, the ACos of one layer the oracle's."""
    import torch
    host = list(si.model_7b_layers(1))
    tabs = _alphabet(["NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4"])
    fmt = sop.fmt_by_name("UE4M4")
    cx = sop.Context(0)
    cx.set_alphabet(tabs); cx.set_pairs(None)
    layers = [(torch.from_numpy(W).cuda().to(torch.bfloat16), torch.from_numpy(c).cuda()) for _, W, c, _ in host]
    tp, ta, sels = cx.pair_search_layers(layers, 16, fmt, want_sel=True)
    torch.cuda.synchronize()
    tp, ta = tp.cpu().numpy(), ta.cpu().numpy()
    rng = np.random.default_rng(9)
    for i, (name, W, c, _) in enumerate(host):
        o = cx.pair_search(layers[i][0], layers[i][1], 16, fmt)
        torch.cuda.synchronize()
        assert np.array_equal(o.acos_pair.cpu().numpy()[:15], tp[i]) and np.array_equal(o.acos_atom.cpu().numpy(), ta[i]), name
        assert torch.equal(o.sel_words, sels[i]), name
        M, K = W.shape
        rows = np.sort(rng.choice(M, size=24, replace=False))
        ref = ops.pair_search(W[rows], c, tabs, 16, oracle_fmt(fmt), want_codes=False)
        got = sels[i].cpu().numpy().view(np.uint16).astype(np.uint32).reshape(M, K // 16)[rows].reshape(-1)
        assert np.array_equal(got, ref.sel_words), name
    name, W, c, _ = host[0]                                          # 4096 x 4096: the oracle on the whole layer
    ref = ops.pair_search(W, c, tabs, 16, oracle_fmt(fmt), want_codes=False)
    assert np.max(np.abs(tp[0] - ref.acos_pair)) <= 1e-6 and np.max(np.abs(ta[0] - ref.acos_atom)) <= 1e-6
