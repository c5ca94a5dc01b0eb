"""GPU parity of the materialisation: scale words and code payloads byte for byte against the oracle."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, pack as PK, pairsearch as ops
import sop_inputs as si
from gpu_util import oracle_fmt, ctx

pytestmark = pytest.mark.gpu

FMTS = {"UE4M3": (0, 4, 3, 8), "S1E5M5": (1, 5, 5, 12), "S0E6M5": (0, 6, 5, 12), "S1E5M4": (1, 5, 4, 12), "S0E5M5": (0, 5, 5, 12),
        "E4M3": (1, 4, 3, 8), "UE4M4": (0, 4, 4, 8)}


def search(W, c, tabs, g, fmt, k=0):
    import torch
    cx = ctx()
    cx.set_alphabet(tabs); cx.set_pairs(None)
    Wt = torch.from_numpy(W).cuda().to(torch.bfloat16)
    ct = torch.from_numpy(c).cuda()
    out = cx.pair_search(Wt, ct, g, fmt, k=k, emit=True)
    torch.cuda.synchronize()
    return out


def make_fmt(name):
    w, x, y, b = FMTS[name]
    return sop.ScaleFmt(w, x, y, b, -1, -1), (w, x, y, b)


@pytest.mark.parametrize("name", ["UE4M3", "S1E5M5", "S0E6M5", "S1E5M4", "S0E5M5"])
@pytest.mark.parametrize("g", [8, 16, 32, 64])
def test_pair_packing_n4(name, g):
    import torch
    fmt, (w, x, y, b) = make_fmt(name)
    M, K = 29, 1088
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 3100 + g, row_sigma=0.5, outlier_frac=0.002))
    W[2, :] = 0.0
    c = si.channel_norms(K, 1.0, 3101)
    tabs = [OA.to_f32(OA.nf(4)), OA.to_f32(OA.sh(4)), OA.to_f32(OA.negate(OA.nf(4)))]
    out = search(W, c, tabs, g, fmt, k=2)
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), k=2)
    for (a, bb, q) in ((0, 1, 0), (1, 2, 2), (0, 2, 1)):
        words, payload, n = ctx().pack_blocks(out, M, K, g, fmt, a, bb, q)
        torch.cuda.synchronize()
        rw, rp, rn = PK.materialise(ref, tabs, M, K, g, a, bb, q, w, x, y, b)
        assert n == rn == 4
        assert np.array_equal(words.cpu().numpy().view(np.uint16), rw)
        assert np.array_equal(payload.cpu().numpy(), rp)
    # one codebook alone
    words, payload, n = ctx().pack_blocks(out, M, K, g, fmt, 1)
    rw, rp, rn = PK.materialise(ref, tabs, M, K, g, 1, None, None, w, x, y, b)
    assert np.array_equal(words.cpu().numpy().view(np.uint16), rw) and np.array_equal(payload.cpu().numpy(), rp)


@pytest.mark.parametrize("g", [8, 16, 32])
def test_wider_and_narrower_codes(g):
    import torch
    fmt, (w, x, y, b) = make_fmt("S1E5M5")
    M, K = 17, 576
    W = si.bf16_round(si.student_t_weights(M, K, 5.0, 3200 + g, row_sigma=0.3))
    c = si.channel_norms(K, 0.7, 3201)
    e2m3 = OA.to_f32(OA.exmy_grid(2, 3))                             # 63 values: n = 6
    nf3 = OA.to_f32(OA.nf(3))                                       # 8 values: n = 3
    tabs = [OA.to_f32(OA.nf(5)), OA.to_f32(OA.nf(4)), e2m3, nf3]
    out = search(W, c, tabs, g, fmt)
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt))
    pairs = ops.all_pairs(4).tolist()
    for (a, bb, n_want) in ((0, 1, 5), (1, 2, 6), (0, 2, 6), (1, 3, 4)):
        q = pairs.index([a, bb])
        words, payload, n = ctx().pack_blocks(out, M, K, g, fmt, a, bb, q)
        torch.cuda.synchronize()
        rw, rp, rn = PK.materialise(ref, tabs, M, K, g, a, bb, q, w, x, y, b)
        assert n == rn == n_want and payload.shape[1] == g * n // 8
        assert np.array_equal(words.cpu().numpy().view(np.uint16), rw)
        assert np.array_equal(payload.cpu().numpy(), rp)
    for a, n_want in ((2, 6), (3, 3), (0, 5)):
        words, payload, n = ctx().pack_blocks(out, M, K, g, fmt, a)
        rw, rp, rn = PK.materialise(ref, tabs, M, K, g, a, None, None, w, x, y, b)
        assert n == rn == n_want
        assert np.array_equal(words.cpu().numpy().view(np.uint16), rw) and np.array_equal(payload.cpu().numpy(), rp)


def test_formats_without_a_metabit():
    import torch
    M, K, g = 8, 256, 16
    W = si.bf16_round(si.student_t_weights(M, K, 5.0, 3300))
    c = si.channel_norms(K, 0.7, 3301)
    tabs = [OA.to_f32(OA.nf(4)), OA.to_f32(OA.sh(4))]
    for name in ("E4M3", "UE4M4"):
        fmt, (w, x, y, b) = make_fmt(name)
        out = search(W, c, tabs, g, fmt)
        ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt))
        with pytest.raises(sop.SopError) as ei:
            ctx().pack_blocks(out, M, K, g, fmt, 0, 1, 0)
        assert ei.value.status == 4
        words, payload, n = ctx().pack_blocks(out, M, K, g, fmt, 0)
        rw, rp, rn = PK.materialise(ref, tabs, M, K, g, 0, None, None, w, x, y, b)
        assert np.array_equal(words.cpu().numpy().view(np.uint16), rw) and np.array_equal(payload.cpu().numpy(), rp)


def test_decoding_the_gpu_arrays_reproduces_the_layer():
    import torch
    fmt, (w, x, y, b) = make_fmt("UE4M3")
    M, K, g = 32, 512, 16
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 3400, row_sigma=0.4))
    c = si.channel_norms(K, 1.0, 3401)
    tabs = [OA.to_f32(OA.nf(4)), OA.to_f32(OA.sh(4))]
    out = search(W, c, tabs, g, fmt, k=1)
    words, payload, n = ctx().pack_blocks(out, M, K, g, fmt, 0, 1, 0)
    torch.cuda.synchronize()
    What = PK.reconstruct(words.cpu().numpy().view(np.uint16), payload.cpu().numpy(), n, g, M, K, tabs[0], tabs[1],
                          oracle_fmt(fmt), 1, w, x, y, b)
    d = (W.astype(np.float64) - What.astype(np.float64)).reshape(-1, g)
    err = (np.tile(c.astype(np.float64), M).reshape(-1, g) * d * d).sum(axis=1)
    be = out.blk_err.cpu().numpy()
    sel = (out.sel_words.cpu().numpy().view(np.uint16) & 1).astype(bool)
    assert np.allclose(err, np.where(sel, be[1], be[0]).astype(np.float64), rtol=2e-5, atol=1e-12)
