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
