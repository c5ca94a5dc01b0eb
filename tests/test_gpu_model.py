"""GPU parity of the model-wide search (configuration 4: every linear layer of 7B-shaped blocks in one
call, a per-layer ACos table out): the table and the selector words against the oracle, layer by layer."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, pairsearch as ops
import sop_inputs as si
from gpu_util import oracle_fmt, ctx

pytestmark = pytest.mark.gpu


def _alphabet():
    draws = si.normal_draws(1 << 18, 4242)
    nf4, sh4, bof4 = OA.nf(4), OA.sh(4), OA.bof(4, draws)
    return [OA.to_f32(t) for t in (nf4, sh4, bof4, OA.negate(nf4), OA.negate(sh4), OA.negate(bof4))]


@pytest.mark.parametrize("fmtname", ["UE4M4", "E4M3"])
def test_two_blocks_of_seven_layers(fmtname):
    import torch
    tabs = _alphabet()
    fmt = sop.fmt_by_name(fmtname)
    cx = ctx()
    cx.set_alphabet(tabs); cx.set_pairs(None)
    host = list(si.model_7b_layers(2, rows=96))                       # 14 layers, three different shapes
    layers = [(torch.from_numpy(W).cuda().to(torch.bfloat16), torch.from_numpy(c).cuda()) for _, W, c, _ in host]
    shifts = [(-1, 0, 2)[i % 3] for i in range(len(host))]
    tp, ta, sels = cx.pair_search_layers(layers, 16, fmt, shifts=shifts, want_sel=True)
    torch.cuda.synchronize()
    tp, ta = tp.cpu().numpy(), ta.cpu().numpy()
    assert tp.shape == (14, 15) and ta.shape == (14, 6)
    nus = []
    for i, (name, W, c, nu) in enumerate(host):
        ref = ops.pair_search(W, c, tabs, 16, oracle_fmt(fmt), k=shifts[i], want_codes=False)
        assert np.max(np.abs(tp[i] - ref.acos_pair)) <= 1e-6, name
        assert np.max(np.abs(ta[i] - ref.acos_atom)) <= 1e-6, name
        assert np.array_equal(sels[i].cpu().numpy().view(np.uint16).astype(np.uint32), ref.sel_words), name
        nus.append(nu)
    assert len(set(nus)) == 14 and 3.0 <= min(nus) and max(nus) <= 8.0
    # a single call per layer gives the same table bit for bit
    for i in (0, 6, 13):
        o = cx.pair_search(layers[i][0], layers[i][1], 16, fmt, k=shifts[i])
        torch.cuda.synchronize()
        assert np.array_equal(o.acos_pair.cpu().numpy()[:15], tp[i]) and np.array_equal(o.acos_atom.cpu().numpy(), ta[i])
    # table only, no selector words
    tp2, ta2, none = cx.pair_search_layers(layers, 16, fmt, shifts=shifts)
    torch.cuda.synchronize()
    assert none is None and np.array_equal(tp2.cpu().numpy(), tp) and np.array_equal(ta2.cpu().numpy(), ta)


def test_a_bad_layer_stops_the_call_before_any_launch():
    import torch
    cx = ctx()
    cx.set_alphabet(_alphabet()[:2]); cx.set_pairs(None)
    good = (torch.zeros((8, 256), dtype=torch.bfloat16, device="cuda"), torch.ones(256, dtype=torch.float32, device="cuda"))
    bad = (torch.zeros((8, 264), dtype=torch.bfloat16, device="cuda"), torch.ones(264, dtype=torch.float32, device="cuda"))   # 16 does not divide K
    with pytest.raises(sop.SopError) as ei:
        cx.pair_search_layers([good, good, bad], 16, sop.fmt_by_name("UE4M4"))
    assert ei.value.status == 2 and "layer 2" in str(ei.value)
    with pytest.raises(sop.SopError):
        cx.pair_search_layers([good, (good[0].float(), good[1])], 16, sop.fmt_by_name("UE4M4"))


def test_more_layers_than_one_launch_takes():
    """1030 small layers (the model-wide kernel takes 1024 per launch): every row of the table equals the
    single call's, a few are checked against the oracle."""
    import torch
    tabs = _alphabet()
    fmt = sop.fmt_by_name("UE4M4")
    cx = ctx()
    cx.set_alphabet(tabs); cx.set_pairs(None)
    rng = np.random.default_rng(77)
    n = 1030
    Ws = (rng.standard_t(4.0, size=(n, 8, 256)) * 0.05).astype(np.float32)
    c = np.exp(rng.standard_normal(256)).astype(np.float32)
    big = torch.from_numpy(Ws).cuda()
    ct = torch.from_numpy(c).cuda()
    layers = [(big[i], ct) for i in range(n)]
    tp, ta, _ = cx.pair_search_layers(layers, 16, fmt)
    torch.cuda.synchronize()
    tp, ta = tp.cpu().numpy(), ta.cpu().numpy()
    assert tp.shape == (n, 15) and ta.shape == (n, 6)
    for i in (0, 1, 511, 1023, 1024, 1029):
        o = cx.pair_search(big[i], ct, 16, fmt)
        torch.cuda.synchronize()
        assert np.array_equal(o.acos_pair.cpu().numpy()[:15], tp[i]) and np.array_equal(o.acos_atom.cpu().numpy(), ta[i]), i
    for i in (3, 1027):
        ref = ops.pair_search(Ws[i], c, tabs, 16, oracle_fmt(fmt), want_codes=False)
        assert np.max(np.abs(tp[i] - ref.acos_pair)) <= 1e-6 and np.max(np.abs(ta[i] - ref.acos_atom)) <= 1e-6
    assert np.all(np.isfinite(tp)) and np.all(tp <= 1.0 + 1e-9) and np.all(tp > 0.5)


def test_two_atom_alphabet_goes_layer_by_layer():
    """Alphabets of one or two atoms have no model-wide kernel: the call runs one kernel per layer on two
    streams of its own; same table as single calls and as the oracle."""
    import torch
    tabs = _alphabet()[:2]
    fmt = sop.fmt_by_name("UE4M3")
    cx = ctx()
    cx.set_alphabet(tabs); cx.set_pairs(None)
    host = list(si.model_7b_layers(1, rows=64))[:5]
    layers = [(torch.from_numpy(W).cuda().to(torch.bfloat16), torch.from_numpy(c).cuda()) for _, W, c, _ in host]
    tp, ta, sels = cx.pair_search_layers(layers, 16, fmt, want_sel=True)
    torch.cuda.synchronize()
    tp, ta = tp.cpu().numpy(), ta.cpu().numpy()
    for i, (name, W, c, _) in enumerate(host):
        ref = ops.pair_search(W, c, tabs, 16, oracle_fmt(fmt), want_codes=False)
        assert np.max(np.abs(tp[i] - ref.acos_pair)) <= 1e-6 and np.max(np.abs(ta[i] - ref.acos_atom)) <= 1e-6, name
        assert np.array_equal(sels[i].cpu().numpy().view(np.uint16).astype(np.uint32), ref.sel_words), name
        o = cx.pair_search(layers[i][0], layers[i][1], 16, fmt)
        torch.cuda.synchronize()
        assert np.array_equal(o.acos_pair.cpu().numpy()[:1], tp[i]) and np.array_equal(o.acos_atom.cpu().numpy(), ta[i])


@pytest.mark.parametrize("seed", range(int(__import__("os").environ.get("SOP_RANDOM_MODELS", "6"))))
def test_random_lists_of_layers(seed):
    """Random lists of layers (shapes with ragged strips, row strides, 1 to 40 layers, several layer shifts), alphabets of 1 to
    8 atoms, block sizes, signed and unsigned scale words, metrics: every row of the table and every selector word against the
    oracle, and bit for bit against the single call."""
    import torch
    rng = np.random.default_rng(7700 + seed)
    pool = _alphabet() + [OA.to_f32(t) for t in (OA.nf(3), OA.sh(5), OA.negate(OA.sh(5)), OA.nf(5), np.array([-1.0, 0.0, 1.0]))]
    A = int(rng.integers(1, 9))
    tabs = [pool[i] for i in rng.permutation(len(pool))[:A]]
    g = int(rng.choice([8, 16, 16, 32, 64]))
    fmt = sop.fmt_by_name(str(rng.choice(["UE4M4", "E4M3", "UE4M6", "S1E5M5", "UE5M7"])))
    metric = int(rng.choice([0, 0, 1, 2]))
    bf16 = bool(rng.random() < 0.7)
    cx = ctx()
    cx.set_alphabet(tabs); cx.set_pairs(None)
    P = A * (A - 1) // 2
    n = int(rng.integers(1, 41))
    host, layers, shifts = [], [], []
    for l in range(n):
        M, K = int(rng.integers(1, 24)), g * int(rng.integers(1, 40))
        while K % 8: K += g
        W = si.student_t_weights(M, K, float(rng.uniform(3, 8)), 7800 + 100 * seed + l, row_sigma=0.5)
        if rng.random() < 0.1: W[:] = 0.0
        if bf16: W = si.bf16_round(W)
        c = si.channel_norms(K, 1.0, 7900 + 100 * seed + l)
        Wt = torch.from_numpy(W).cuda()
        if bf16: Wt = Wt.to(torch.bfloat16)
        if rng.random() < 0.3:                                        # a row stride larger than K
            buf = torch.zeros((M, K + 16), dtype=Wt.dtype, device="cuda")
            buf[:, :K] = Wt
            Wt = buf[:, :K]
        host.append((W, c)); layers.append((Wt, torch.from_numpy(c).cuda())); shifts.append(int(rng.choice([0, 0, 1, -2, 3])))
    tp, ta, sels = cx.pair_search_layers(layers, g, fmt, metric=metric, shifts=shifts, want_sel=P > 0)
    torch.cuda.synchronize()
    tp, ta = tp.cpu().numpy(), ta.cpu().numpy()
    for l, (W, c) in enumerate(host):
        ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), k=shifts[l], metric=metric, want_codes=False)
        assert np.max(np.abs(ta[l] - ref.acos_atom)) <= 1e-6, l
        if P:
            assert np.max(np.abs(tp[l] - ref.acos_pair)) <= 1e-6, l
            sw = sels[l].cpu().numpy()
            assert np.array_equal(sw.view(np.uint16 if sw.dtype == np.int16 else np.uint32).astype(np.uint32), ref.sel_words), l
        if l % 7 == 0:
            o = cx.pair_search(layers[l][0], layers[l][1], g, fmt, k=shifts[l], metric=metric)
            torch.cuda.synchronize()
            assert np.array_equal(o.acos_atom.cpu().numpy(), ta[l]) and (P == 0 or np.array_equal(o.acos_pair.cpu().numpy()[:P], tp[l])), l
