"""Signed scale words with sign-negated copies in the alphabet: the library takes a copy's candidates over
from its original (the positive sign of -a is the negative sign of a) instead of evaluating them, except
in wavefronts where a scaled weight lies exactly on a code boundary.  Every output must stay the requested
atom's, bit for bit, whichever way a wavefront went."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, pairsearch as ops
import sop_inputs as si
from gpu_util import run_gpu, compare, oracle_fmt

pytestmark = pytest.mark.gpu


def _check(W, c, tabs, g, fmt, metric=0, pairs=None, bf16=True):
    f = sop.fmt_by_name(fmt)
    gpu = run_gpu(W, c, tabs, g, f, metric=metric, pairs=pairs, bf16=bf16)
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(f), metric=metric,
                          pairs=None if pairs is None else np.asarray(pairs, dtype=np.int32))
    P = len(tabs) * (len(tabs) - 1) // 2 if pairs is None else len(pairs)
    compare(gpu, ref, P)
    return gpu


def _layer(seed, M=40, K=2048):
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, seed, row_sigma=0.5, outlier_frac=0.002))
    return W, si.channel_norms(K, 1.0, seed + 1)


@pytest.mark.parametrize("metric", [0, 1, 2])
@pytest.mark.parametrize("g", [8, 16, 32, 64])
def test_copies_in_every_order_of_the_alphabet(metric, g):
    W, c = _layer(8100 + g)
    nf, sh = sop.sop_atom_nf(4), sop.sop_atom_sh(4)
    bof = sop.sop_atom_bof(4, si.normal_draws(1 << 16, 4242))
    neg = sop.sop_atom_negate
    sh2 = (sh * np.float32(0.75)).astype(np.float32); sh2[0], sh2[-1] = sh[0], sh[-1]    # a second atom with SH4's endpoints
    for tabs in ([nf, sh, bof, neg(nf), neg(sh), neg(bof)],            # the usual order: copies far from their originals
                 [neg(sh), neg(nf), sh, nf],                           # copies first
                 [sh, sh2, neg(sh2), neg(sh)],                         # two atoms per endpoint pair, both with copies
                 [sh, nf],                                             # no copy at all under a signed word
                 [neg(bof), bof]):
        _check(W, c, tabs, g, "E4M3", metric=metric)
    gpu = _check(W, c, [nf, sh, bof, neg(nf), neg(sh), neg(bof)], g, "S1E5M5", metric=metric)
    # an atom and its copy reach the same candidates; only blocks whose two signs score exactly the same
    # (the original keeps its positive sign, the copy its own) can separate the two layer values
    assert np.max(np.abs(gpu["acos_atom"][:3] - gpu["acos_atom"][3:])) < 1e-5


def test_self_negated_codebooks_and_wide_codes():
    W, c = _layer(8200)
    e2m3 = OA.to_f32(OA.exmy_grid(2, 3) / 7.5)                           # 63 entries, its own sign-negated copy
    three = np.array([-1.0, 0.0, 1.0], dtype=np.float32)
    nf5, sh5 = sop.sop_atom_nf(5), sop.sop_atom_sh(5)
    neg = sop.sop_atom_negate
    for fmt in ("E4M3", "E5M6"):
        _check(W, c, [e2m3, three, sop.sop_atom_nf(4)], 16, fmt)
        _check(W, c, [nf5, neg(nf5), sh5, neg(sh5)], 16, fmt)            # one byte per code: codes mirrored per byte
        _check(W, c, [e2m3, sh5, neg(sh5)], 32, fmt, metric=1)


def test_ties_on_code_boundaries_send_a_wavefront_the_long_way():
    # weights exactly on code boundaries after scaling by a power-of-two scale, in some wavefronts only:
    # rows 0..3 carry ties, the rest are ordinary weights
    L = np.array([-1, -0.5, 0, 0.25, 0.5, 1], dtype=np.float32)
    neg = sop.sop_atom_negate
    mids = (L[:-1] + L[1:]) / 2
    M, K, g = 12, 2048, 16
    rng = np.random.default_rng(2)
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 8300))
    for b in range(4 * K // g):
        s = 2.0 ** rng.integers(-3, 4)
        blk = rng.choice(np.concatenate([mids, L]), size=g) * s
        blk[0] = s
        W.reshape(-1, g)[b] = blk
    c = si.channel_norms(K, 1.0, 8301)
    sh = sop.sop_atom_sh(4)
    for fmt in ("E4M3", "E4M7"):
        for metric in (0, 1):
            _check(W, c, [L, neg(L), sh, neg(sh)], g, fmt, metric=metric)
    # zero weights on an atom with a boundary at zero: -0 and +0 tie with it
    two = np.array([-1.0, 1.0], dtype=np.float32)
    W2 = W.copy(); W2[5, 64:512] = 0.0; W2[6, 0:256] = -0.0; W2[7, 100:700:3] = -0.0
    _check(W2, c, [two, L, neg(L)], g, "E4M3")
    _check(W2, c, [two, neg(two), sh], g, "E4M3", bf16=False)


def test_degenerate_blocks_under_a_signed_word():
    M, K, g = 8, 1024, 16
    W = si.student_t_weights(M, K, 4.0, 8401)
    W[0, :] = 0.0
    W[1, 16:32] = 0.0; W[1, 20] = 3.0
    W[2, :] = 1e-15                                  # the scale underflows: nothing reconstructed under either sign
    W[3, :] *= 1e6                                   # saturates the largest scale: clamped look-ups
    W[5, 32:48] = -np.abs(W[5, 32:48])
    c = si.channel_norms(K, 1.0, 8402)
    c[64:80] = 0.0
    nf, sh = sop.sop_atom_nf(4), sop.sop_atom_sh(4)
    neg = sop.sop_atom_negate
    for fmt in ("E4M3", "E8M7"):
        _check(W, c, [nf, sh, neg(nf), neg(sh)], g, fmt, bf16=False)
