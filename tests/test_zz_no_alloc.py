"""The entry point that allocates nothing (sop_pair_search_static) against sop_pair_search: the same
kernels with the layer sums and the scale table in the library's static device array, so every output
must agree bit for bit.  Two calls in a row, the second on a smaller layer with another scale word, so
that what the first call left in the array (sums, tickets, a longer scale table) would show."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
import sop_inputs as si

pytestmark = pytest.mark.gpu


def _both(cx, W, c, g, fmt, k, emit):
    import torch
    M, K = W.shape
    res = []
    for static in (False, True):
        out = cx.alloc_outputs(M, K, g, emit=emit)
        for t in (out.acos_pair, out.acos_atom, out.sel_words, out.scale_code, out.codes, out.blk_cos, out.blk_err, out.blk_rank):
            if t is not None:
                t.fill_(-3 if t.dtype != torch.uint8 else 0xEE)   # so that an output left unwritten differs
        cx.pair_search(W, c, g, fmt, k=k, out=out, static=static)
        torch.cuda.synchronize()
        res.append(out)
    return res


def _equal(a, b, n_pairs):
    names = ("acos_atom", "sel_words", "scale_code", "codes", "blk_cos", "blk_err", "blk_rank")
    assert np.array_equal(a.acos_pair.cpu().numpy()[:n_pairs], b.acos_pair.cpu().numpy()[:n_pairs]), "acos_pair"
    for nm in names:
        x, y = getattr(a, nm), getattr(b, nm)
        assert (x is None) == (y is None)
        if x is not None:
            xv, yv = x.cpu().numpy(), y.cpu().numpy()
            assert np.array_equal(xv.view(np.uint8), yv.view(np.uint8)), nm


def test_static_entry_point_equals_pair_search_two_calls_in_a_row():
    import torch
    cx = sop.Context(0)
    tabs = sop.build_alphabet(["NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4"], bof_draws=si.normal_draws(1 << 18, 4242))
    cx.set_alphabet(tabs)
    # first call: 300 x 3072 bf16 (three strips, ranges that split rows unevenly), signed 12-bit scale word
    # (2048 table entries: the whole static table), search + emit
    W1 = torch.from_numpy(si.bf16_round(si.student_t_weights(300, 3072, 4.0, 9101, row_sigma=0.5))).cuda().to(torch.bfloat16)
    c1 = torch.from_numpy(si.channel_norms(3072, 1.0, 9102)).cuda()
    a, b = _both(cx, W1, c1, 16, sop.fmt_by_name("E4M7"), 0, True)
    _equal(a, b, cx.n_pairs)
    # second call: smaller layer (37 x 1088 fp32, ragged last strip), 8-bit unsigned word with a layer shift
    W2 = torch.from_numpy(si.student_t_weights(37, 1088, 4.0, 9103, row_sigma=0.5, outlier_frac=0.002)).cuda()
    c2 = torch.from_numpy(si.channel_norms(1088, 1.0, 9104)).cuda()
    a, b = _both(cx, W2, c2, 8, sop.fmt_by_name("UE4M4"), 3, True)
    _equal(a, b, cx.n_pairs)
    # and search mode (no per-block planes) on the first layer again
    a, b = _both(cx, W1, c1, 32, sop.fmt_by_name("UE4M4"), 0, False)
    _equal(a, b, cx.n_pairs)
    assert 0.9 < float(b.acos_pair.cpu().numpy()[:cx.n_pairs].min()) <= 1.0


def test_static_entry_point_refuses_wide_scale_words():
    import torch
    cx = sop.Context(0)
    cx.set_alphabet(sop.build_alphabet(["NF4", "SH4"]))
    W = torch.zeros((8, 1024), dtype=torch.float32, device="cuda")
    c = torch.ones(1024, dtype=torch.float32, device="cuda")
    out = cx.alloc_outputs(8, 1024, 16)
    with pytest.raises(sop.SopError) as e:
        cx.pair_search(W, c, 16, sop.fmt_by_name("E8M7"), out=out, static=True)      # 15 magnitude bits
    assert e.value.status == 4 and "static" in str(e.value)
    cx.pair_search(W, c, 16, sop.fmt_by_name("E8M7"), out=out)                        # the allocating call takes it
    torch.cuda.synchronize()
