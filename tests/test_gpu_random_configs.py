"""Seeded random configurations of the pair search against the oracle: shapes with ragged strips and row strides,
block sizes, scale words, codebooks of random sizes and values beside the named ones, metrics, pair subsets, layer
shifts, both scale rules, search and emit mode, all on one context in a row (so that nothing a call leaves behind
can change the next)."""
import os

import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, pairsearch as ops
import sop_inputs as si
from gpu_util import run_gpu, compare, oracle_fmt

pytestmark = pytest.mark.gpu

_NAMED = None


def _named():
    global _NAMED
    if _NAMED is None:
        draws = si.normal_draws(1 << 16, 4242)
        t = [OA.nf(4), OA.sh(4), OA.bof(4, draws), OA.nf(3), OA.nf(5), OA.sh(5), OA.sh(3, 1.2, 0.01), OA.exmy_grid(2, 3) / 7.5,
             np.array([-1.0, 1.0]), np.array([-1.0, 0.0, 1.0]), np.array([-1.0, -1 / 3, 1 / 3, 1.0])]
        _NAMED = [OA.to_f32(x) for x in t]
    return _NAMED


def _random_codebook(rng):
    n = int(rng.choice([2, 3, 5, 8, 16, 16, 17, 32, 40, 64]))
    # entries at least 1/80 of the range apart (the table's spacing limit), two-sided, random endpoints
    gaps = rng.uniform(1.0, 3.0, n - 1)
    L = np.concatenate([[0.0], np.cumsum(gaps)])
    z = rng.uniform(0.2, 0.8) * L[-1]
    L = (L - z) / max(z, L[-1] - z) * rng.choice([1.0, 1.0, 0.75, 1.5])
    return OA.to_f32(L)


@pytest.mark.parametrize("seed", range(int(os.environ.get("SOP_RANDOM_CONFIGS", "36"))))     # (more seeds for a longer hunt)
def test_random_configuration(seed):
    rng = np.random.default_rng(9000 + seed)
    g = int(rng.choice([8, 16, 16, 32, 64]))
    K = g * int(rng.integers(1, 70)) if rng.random() < 0.5 else 64 * int(rng.integers(1, 40))
    K = max(K, g) // g * g
    if K % 8: K = (K // 8 + 1) * 8 // g * g or g
    while K % g or K % 8: K += g
    M = int(rng.integers(1, 48))
    bf16 = bool(rng.random() < 0.6)
    W = si.student_t_weights(M, K, float(rng.uniform(3, 8)), 9100 + seed, row_sigma=0.5 if rng.random() < 0.5 else None,
                             outlier_frac=0.002 if rng.random() < 0.5 else 0.0)
    W *= np.float32(2.0 ** int(rng.integers(-6, 4)))
    if rng.random() < 0.3: W[rng.integers(0, M), :] = 0.0
    if rng.random() < 0.3: W.reshape(-1, g)[rng.integers(0, M * K // g, 5)] = 0.0
    if bf16: W = si.bf16_round(W)
    c = si.channel_norms(K, 1.0, 9200 + seed)
    if rng.random() < 0.3: c[rng.integers(0, K, 3)] = 0.0
    A = int(rng.integers(1, 9))
    tabs = []
    for _ in range(A):
        t = _named()[int(rng.integers(0, len(_named())))] if rng.random() < 0.6 else _random_codebook(rng)
        if rng.random() < 0.4: t = OA.to_f32(OA.negate(t))
        tabs.append(t)
    if A >= 2 and rng.random() < 0.5: tabs[-1] = OA.to_f32(OA.negate(tabs[0]))      # a sign-negated copy in the alphabet
    fmt_name = str(rng.choice(list(si.generate.SCALE_FORMATS)))
    fmt = sop.fmt_by_name(fmt_name)
    metric = int(rng.choice([0, 0, 1, 2]))
    rule = 1 if (fmt.sign_bits and rng.random() < 0.25) else 0
    k = int(rng.integers(-2, 5)) if rng.random() < 0.5 else 0
    if fmt.exp_bits >= 8: k = 0                      # (an 8-bit exponent leaves no room for a shift inside binary32's normal range)
    all_pairs = [(a, b) for a in range(A) for b in range(a + 1, A)]
    pairs = None
    if all_pairs and rng.random() < 0.5:
        idx = rng.permutation(len(all_pairs))[: int(rng.integers(1, len(all_pairs) + 1))]
        pairs = [all_pairs[i] for i in idx]
    ldw = None
    if rng.random() < 0.3: ldw = K + 8 * int(rng.integers(1, 5))
    emit = bool(rng.random() < 0.6)
    try:
        gpu = run_gpu(W, c, tabs, g, fmt, k=k, metric=metric, pairs=pairs, bf16=bf16, emit=emit, ldw=ldw, scale_rule=rule)
    except sop.SopError as e:
        # the only refusal a configuration drawn here can meet: codebooks too closely spaced for the table
        assert e.status == 3 and "closely" in str(e), (seed, str(e))
        pytest.skip(f"refused: {e}")
    ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), k=k, metric=metric,
                          pairs=None if pairs is None else np.asarray(pairs, dtype=np.int32), scale_rule=rule, want_codes=emit)
    P = len(all_pairs) if pairs is None else len(pairs)
    compare(gpu, ref, P, emit=emit)


def test_more_scale_tables_than_the_context_keeps():
    """The context keeps the (scale, reciprocal) tables of the 160 (format, shift) pairs used last; 420 distinct pairs in a
    row, the first ones used again at the end: every search against the oracle."""
    import torch
    rng = np.random.default_rng(4711)
    M, K, g = 6, 512, 16
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 4712, row_sigma=0.5) * np.float32(0.25))
    c = si.channel_norms(K, 1.0, 4713)
    tabs = [OA.to_f32(OA.nf(4)), OA.to_f32(OA.sh(4)), OA.to_f32(OA.negate(OA.sh(4)))]
    combos = [(w, x, y, bias, k) for w in (0, 1) for x in (4, 5) for y in (3, 4, 5) for bias in (5, 6, 7, 8, 9) for k in (-2, -1, 0, 1, 2, 3, 4)]
    order = [combos[i] for i in rng.permutation(len(combos))]
    order = order + order[:25]
    assert len(set(order)) == 420
    for (w, x, y, bias, k) in order:
        fmt = sop.ScaleFmt(w, x, y, 16, bias, -1)
        gpu = run_gpu(W, c, tabs, g, fmt, k=k, bf16=True, emit=False)
        ref = ops.pair_search(W, c, tabs, g, oracle_fmt(fmt), k=k, want_codes=False)
        compare(gpu, ref, 3, emit=False)
