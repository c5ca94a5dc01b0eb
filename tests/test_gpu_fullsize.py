"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py
times (search mode, no per-block outputs) and in emit mode on row samples."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import pairsearch as ops
import sop_inputs as si
from gpu_util import run_gpu, compare, oracle_fmt, cached_config, ctx

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
    W, c, cfg = cached_config(name)
    tabs = _alphabet(cfg["atoms"])
    fmt = sop.fmt_by_name(cfg["fmt"])
    gpu = run_gpu(W, c, tabs, 16, fmt, bf16=True, emit=False)        # the configuration bench.py times
    ref = ops.pair_search(W, c, tabs, 16, oracle_fmt(fmt), want_codes=False)
    compare(gpu, ref, 15, emit=False)


def test_config5_whole_layer_against_the_oracle():
    # 70B-shaped MLP layer 28672 x 8192 in the launch configuration bench.py times (search mode): every
    # selector word and every ACos against the oracle on the whole layer
    W, c, cfg = cached_config("C5")
    tabs = _alphabet(cfg["atoms"])
    fmt = sop.fmt_by_name(cfg["fmt"])
    gpu = run_gpu(W, c, tabs, 16, fmt, bf16=True, emit=False)
    ref = ops.pair_search(W, c, tabs, 16, oracle_fmt(fmt), want_codes=False)
    compare(gpu, ref, 15, emit=False)
    assert np.all((gpu["acos_pair"] > 0.99) & (gpu["acos_pair"] <= 1.0))


def test_headline_layer_repeat_runs_are_bit_equal():
    # the sums of the layer reduction are integers: which wavefront took which step, and in what order
    # the workgroups finished, cannot change a bit of the result
    import torch
    W, c, cfg = cached_config("C3_down")
    tabs = _alphabet(cfg["atoms"])
    fmt = sop.fmt_by_name(cfg["fmt"])
    cx = sop.Context(0)
    cx.set_alphabet(tabs)
    Wt = torch.from_numpy(W).cuda().to(torch.bfloat16)
    ct = torch.from_numpy(c).cuda()
    runs = []
    for i in range(4):
        o = cx.pair_search(Wt, ct, 16, fmt, static=(i == 3), out=cx.alloc_outputs(W.shape[0], W.shape[1], 16))
        torch.cuda.synchronize()
        runs.append((o.acos_pair.cpu().numpy().copy(), o.acos_atom.cpu().numpy().copy(), o.sel_words.cpu().numpy().copy()))
    for r in runs[1:]:
        assert all(np.array_equal(x.view(np.uint8), y.view(np.uint8)) for x, y in zip(runs[0], r))


# the scale words of the sweep: the 8-, 10-, 12- and 16-bit formats of the paper's scale-format tables
SWEEP_FORMATS = ["UE4M4", "E4M3", "UE4M6", "E4M5", "UE5M7", "E5M6", "E4M7", "S1E5M5", "E8M7"]


@pytest.mark.parametrize("layer", ["C3_down", "C3_up"])
@pytest.mark.parametrize("n", [4, 5])
def test_config3_sweep_block_sizes_by_scale_formats(layer, n):
    """The sweep of configuration 3 on the first 256 rows of both MLP layers: block sizes 8, 16, 32, 64 by
    nine scale words, for the six four-bit atoms and the six five-bit atoms; every output against the oracle
    (codes, scale codes, selector words, block errors and ranking scores bit for bit, ACos at 1e-6)."""
    W, c, cfg = cached_config(layer)
    W = W[:256]
    tabs = _alphabet([f"NF{n}", f"SH{n}", f"BOF{n}", f"-NF{n}", f"-SH{n}", f"-BOF{n}"])
    for g in (8, 16, 32, 64):
        for name in SWEEP_FORMATS:
            f = sop.fmt_by_name(name)
            gpu = run_gpu(W, c, tabs, g, f, bf16=True, emit=True)
            ref = ops.pair_search(W, c, tabs, g, oracle_fmt(f))
            try:
                compare(gpu, ref, 15)
            except AssertionError as e:
                raise AssertionError(f"{layer} n={n} g={g} {name}: {e}") from e


def test_config4_fourteen_layers_full_size_through_the_model_wide_call():
    """Fourteen layers of the 7B-shaped model at their full sizes in one model-wide call (the launch
    bench.py --workload model times): the seven layers of block 0 and one layer of each type from seven
    other blocks.  Every row of the ACos tables and every selector word against the oracle on the whole
    layer; the tables also equal the single calls' bit for bit."""
    import torch
    picks = [(0, i) for i in range(7)] + [(3, 4), (7, 0), (12, 6), (18, 2), (21, 5), (27, 1), (31, 3)]
    tabs = _alphabet(["NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4"])
    fmt = sop.fmt_by_name("UE4M4")
    cx = sop.Context(0)
    cx.set_alphabet(tabs); cx.set_pairs(None)
    host = [si.model_7b_layer(b, i) for b, i in picks]
    assert len({nu for _, _, _, nu in host}) == 14
    layers = [(torch.from_numpy(W).cuda().to(torch.bfloat16), torch.from_numpy(c).cuda()) for _, W, c, _ in host]
    tp, ta, sels = cx.pair_search_layers(layers, 16, fmt, want_sel=True)
    torch.cuda.synchronize()
    tp, ta = tp.cpu().numpy(), ta.cpu().numpy()
    for i, (name, W, c, _) in enumerate(host):
        ref = ops.pair_search(W, c, tabs, 16, oracle_fmt(fmt), want_codes=False)
        assert np.max(np.abs(tp[i] - ref.acos_pair)) <= 1e-6 and np.max(np.abs(ta[i] - ref.acos_atom)) <= 1e-6, name
        assert np.array_equal(sels[i].cpu().numpy().view(np.uint16).astype(np.uint32), ref.sel_words), name
        if i < 7:
            o = cx.pair_search(layers[i][0], layers[i][1], 16, fmt)
            torch.cuda.synchronize()
            assert np.array_equal(o.acos_pair.cpu().numpy()[:15], tp[i]) and np.array_equal(o.acos_atom.cpu().numpy(), ta[i]), name
            assert torch.equal(o.sel_words, sels[i]), name


def test_layer_of_more_than_128_steps_per_wavefront():
    """A wavefront adds its lanes' sums to the workgroup's every 128 steps (a lane's 32-bit sums would overflow beyond);
    no layer of the configurations is large enough to get there (it takes more than 403 M weights).  805 M weights
    (49152 x 16384: twelve row-rotated, rescaled copies of one drawn block): every selector word and ACos against the oracle."""
    import torch
    K, Mb, reps = 16384, 4096, 12
    base = si.bf16_round(si.student_t_weights(Mb, K, 4.0, 15001, row_sigma=0.5))
    W = np.concatenate([np.roll(base, 7 * r, axis=0) * np.float32(2.0 ** (r % 3 - 1)) for r in range(reps)], axis=0)
    c = si.channel_norms(K, 1.0, 15002)
    tabs = sop.build_alphabet(["NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4"], bof_draws=si.normal_draws(1 << 18, 4242))
    cx = ctx()
    cx.set_alphabet(tabs); cx.set_pairs(None)
    fmt = sop.fmt_by_name("UE4M4")
    out = cx.pair_search(torch.from_numpy(W).cuda().to(torch.bfloat16), torch.from_numpy(c).cuda(), 16, fmt)
    torch.cuda.synchronize()
    assert W.size / 1024 / (torch.cuda.get_device_properties(0).multi_processor_count * 12) > 128
    ref = ops.pair_search(W, c, tabs, 16, oracle_fmt(fmt), want_codes=False)
    assert np.array_equal(out.sel_words.cpu().numpy().view(np.uint16).astype(np.uint32), ref.sel_words)
    assert np.max(np.abs(out.acos_pair.cpu().numpy()[:15] - ref.acos_pair)) <= 1e-6
    assert np.max(np.abs(out.acos_atom.cpu().numpy() - ref.acos_atom)) <= 1e-6
