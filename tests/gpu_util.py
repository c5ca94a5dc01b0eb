"""Helpers of the GPU parity tests: run the HIP path and the oracle on the same tensors."""
import numpy as np

import paper_2605_14929_amd as sop
from oracle import pairsearch as ops

_ctx = None
_cfg_cache = {}


def cached_config(name):
    """A benchmark configuration's tensors, drawn once per test session (the 70B-shaped layer takes a
    while to draw and several tests use it)."""
    import sop_inputs as si
    if name not in _cfg_cache:
        _cfg_cache[name] = si.make_config(name)
    return _cfg_cache[name]


def ctx():
    global _ctx
    if _ctx is None:
        _ctx = sop.Context(0)
    return _ctx


def oracle_fmt(f: sop.ScaleFmt):
    return ops.make_fmt(f.sign_bits, f.exp_bits, f.man_bits, f.container_bits, f.bias, f.max_code)


def run_gpu(W, c, tabs, g, fmt, k=0, metric=0, pairs=None, bf16=False, emit=True, ldw=None, scale_rule=0):
    """W fp32 numpy (already on the bf16 grid when bf16=True).  Returns dict of numpy arrays."""
    import torch
    cx = ctx()
    cx.set_alphabet(tabs)
    cx.set_pairs(pairs)
    Wt = torch.from_numpy(W).cuda()
    if bf16:
        Wt = Wt.to(torch.bfloat16)
    if ldw is not None:
        buf = torch.zeros((W.shape[0], ldw), dtype=Wt.dtype, device="cuda")
        buf[:, :W.shape[1]] = Wt
        Wt = buf[:, :W.shape[1]]
    ct = torch.from_numpy(c).cuda()
    cx.set_scale_rule(scale_rule)
    try:
        out = cx.pair_search(Wt, ct, g, fmt, k=k, metric=metric, emit=emit)
        torch.cuda.synchronize()
    finally:
        cx.set_scale_rule(0)
    r = dict(acos_pair=out.acos_pair.cpu().numpy()[:cx.n_pairs], acos_atom=out.acos_atom.cpu().numpy())
    if out.sel_words is not None:
        sw = out.sel_words.cpu().numpy()
        r["sel_words"] = sw.view(np.uint16 if sw.dtype == np.int16 else np.uint32).astype(np.uint32)
    if emit:
        r["scale_code"] = out.scale_code.cpu().numpy().view(np.uint16)
        r["codes"] = [p.cpu().numpy() for p in out.code_planes]
        r["blk_err"] = out.blk_err.cpu().numpy()
        r["blk_rank"] = out.blk_rank.cpu().numpy()
        r["blk_cos"] = out.blk_cos.cpu().numpy()
    return r


def compare(gpu, ref, n_pairs, emit=True, acos_tol=1e-6, cos_tol=2e-5):
    """Bit-exact on every integer output and on the decision scores; ACos within 1e-6 absolute."""
    if n_pairs:
        assert np.array_equal(gpu["sel_words"], ref.sel_words), "selector bits differ"
        assert np.max(np.abs(gpu["acos_pair"] - ref.acos_pair)) <= acos_tol, (gpu["acos_pair"], ref.acos_pair)
    assert np.max(np.abs(gpu["acos_atom"] - ref.acos_atom)) <= acos_tol, (gpu["acos_atom"], ref.acos_atom)
    if emit:
        assert np.array_equal(gpu["scale_code"], ref.scale_code), "scale codes differ"
        for a, (x, y) in enumerate(zip(gpu["codes"], ref.codes)):
            assert np.array_equal(x, y), f"codes of atom {a} differ at {np.flatnonzero(x != y)[:8]}"
        assert np.array_equal(gpu["blk_err"], ref.blk_err), "block scores differ"
        assert np.array_equal(gpu["blk_rank"].view(np.uint32), ref.blk_rank.view(np.uint32)), "ranking scores differ"
        assert np.max(np.abs(gpu["blk_cos"] - ref.blk_cos)) <= cos_tol
