"""Pins for the oracle's block search: hand-worked blocks, exact-arithmetic brute force on tiny
layers, representable weights, and the symmetries the definitions imply."""
from fractions import Fraction as Fr
import math

import numpy as np
import pytest

from oracle import atoms as A, pairsearch as ps
import sop_inputs as si

WIDE = ps.make_fmt(1, 8, 7, bias=119, max_code=244 * 128 + 127)     # fine scale grid, signed
WIDE_U = ps.make_fmt(0, 8, 7, bias=119, max_code=244 * 128 + 127)
UE4M4 = ps.make_fmt(0, 4, 4)
E4M3 = ps.make_fmt(1, 4, 3)


def f32(x):
    return np.asarray(x, dtype=np.float32)


# ---------------------------------------------------------------- hand-worked blocks
def test_hand_worked_block_linear_channel_weighting():
    # L = {-1,0,1}, block (1, 0.4), c = (1, 4): s = 1, codes (2,1), w_hat = (1,0).
    # <w,w_hat>_c = 1, ||w||_c^2 = 1 + 4*0.16, ||w_hat||_c^2 = 1, error = 4*0.16.
    L = f32([-1, 0, 1])
    W = f32([[1.0, 0.4]])
    c = f32([1.0, 4.0])
    r = ps.pair_search(W, c, [L], 2, WIDE_U)
    assert ps.unpack_codes(r.codes[0], 3, 1, 2).tolist() == [[2, 1]]
    wn = 1 + 4 * float(np.float32(0.4)) ** 2
    assert abs(r.acos_atom[0] - 1 / math.sqrt(wn)) < 1e-15
    assert abs(r.blk_err[0, 0] - 4 * float(np.float32(0.4)) ** 2) < 1e-7
    # with c squared the cosine would be 1/sqrt(1+16*0.16): make sure that is NOT what we get
    assert abs(r.acos_atom[0] - 1 / math.sqrt(1 + 16 * 0.16)) > 0.1


def test_hand_worked_asymmetric_absmax_and_sign():
    # endpoints t- = -1, t+ = 0.5.  Block (0.3, -0.9): positive scale = max(0.3/0.5, 0.9/1) = 0.9.
    # Negative scale swaps the endpoints: max(0.3/1, 0.9/0.5) = 1.8.
    L = f32([-1, 0, 0.5])
    W = f32([[0.3, -0.9]])
    c = f32([1, 1])
    u = ps.pair_search(W, c, [L], 2, WIDE_U)
    q = int(u.scale_code[0, 0])
    assert abs(ps.scale_value(WIDE_U, q) - 0.9) < 0.9 * 2 ** -8
    assert ps.unpack_codes(u.codes[0], 3, 1, 2).tolist() == [[2, 0]]      # 0.33 -> 0.5 ; -1 -> -1
    # the same block under the sign-negated atom {-0.5, 0, 1} needs scale 1.8
    n = ps.pair_search(W, c, [f32(A.negate(L))], 2, WIDE_U)
    assert abs(ps.scale_value(WIDE_U, int(n.scale_code[0, 0])) - 1.8) < 1.8 * 2 ** -8
    # signed format: both signs tried, better one kept.  sigma=+ : w_hat = (0.45,-0.9), err 0.0225;
    # sigma=- : scale 1.8, -w/s = (-0.167, 0.5) -> (0, 0.5) -> w_hat = (0,-0.9), err 0.09.
    s = ps.pair_search(W, c, [L], 2, WIDE)
    assert (int(s.scale_code[0, 0]) >> 15) == 0
    assert abs(s.blk_err[0, 0] - 0.0225) < 2e-3
    # a block whose negative-sign candidate is better: (0.9, -0.3) -> sigma=+ scale 1.8: (0.5,-0.17)->(0.5,0):
    # w_hat=(0.9,0) err .09 ; sigma=-: scale max(0.9/1, 0.3/0.5)=0.9: -w/s=(-1, 0.33)->(-1,0.5): w_hat=(0.9,-0.45) err .0225
    s2 = ps.pair_search(f32([[0.9, -0.3]]), c, [L], 2, WIDE)
    assert (int(s2.scale_code[0, 0]) >> 15) == 1
    assert ps.unpack_codes(s2.codes[0], 3, 1, 2).tolist() == [[0, 2]]
    assert abs(s2.blk_err[0, 0] - 0.0225) < 2e-3


def test_acos_is_mean_of_block_cosines_not_ratio_of_sums():
    L = f32([-1, 0, 1])
    W = f32([[1.0, 0.4, 100.0, 0.0]])          # second block is exactly representable
    c = f32([1, 4, 1, 1])
    r = ps.pair_search(W, c, [L], 2, WIDE_U)
    cos0 = 1 / math.sqrt(1 + 4 * float(np.float32(0.4)) ** 2)
    assert abs(r.acos_atom[0] - 0.5 * (cos0 + 1.0)) < 1e-12
    assert abs(r.blk_cos[0, 0] - cos0) < 1e-7 and r.blk_cos[0, 1] == 1.0


def test_ties_go_to_the_lower_index_and_the_positive_sign():
    L = f32([-1, 0, 1])                                   # midpoints -0.5 and +0.5, closed under negation
    c = f32([1, 1, 1, 1])
    r = ps.pair_search(f32([[1.0, 0.5, -0.5, -1.0]]), c, [L], 4, WIDE)
    assert ps.unpack_codes(r.codes[0], 3, 1, 4).tolist() == [[2, 1, 0, 0]]
    # a codebook closed under negation reconstructs identically under both scale signs: exact tie,
    # and the tie keeps the positive sign
    W = si.student_t_weights(8, 64, 5.0, 91)
    r = ps.pair_search(W, np.ones(64, dtype=np.float32), [L], 16, WIDE)
    assert np.all(r.scale_code[0] >> 15 == 0)
    # in a pair of identical atoms the selector stays 0
    r = ps.pair_search(W, np.ones(64, dtype=np.float32), [L, L], 16, WIDE)
    assert not r.sel_words.any()


def test_zero_blocks():
    L = f32(A.nf(4))
    W = np.zeros((1, 32), dtype=np.float32)
    W[0, 16] = 1e-30                                  # second block underflows the scale format
    c = np.ones(32, dtype=np.float32)
    r = ps.pair_search(W, c, [L], 16, UE4M4)
    assert r.scale_code[0].tolist() == [0, 0]
    assert (ps.unpack_codes(r.codes[0], 16, 1, 32) == 7).all()       # entry 7 of NF4 is the zero
    assert r.blk_cos[0].tolist() == [1.0, 0.0]
    assert r.acos_atom[0] == 0.5


# ---------------------------------------------------------------- exact-arithmetic brute force
def _exact_block(w, c, L, s):
    """argmin_k |w_i - s L_k| (ties to the lower k) and the weighted sums, in rationals."""
    Ls = [Fr(float(v)) for v in L]
    codes, num, den, wn, err = [], Fr(0), Fr(0), Fr(0), Fr(0)
    for wi, ci in zip(w, c):
        wi, ci = Fr(float(wi)), Fr(float(ci))
        k = min(range(len(Ls)), key=lambda j: (abs(wi - s * Ls[j]), j))
        wh = s * Ls[k]
        codes.append(k)
        num += ci * wi * wh
        den += ci * wh * wh
        wn += ci * wi * wi
        err += ci * (wi - wh) ** 2
    return codes, num, den, wn, err


@pytest.mark.parametrize("fmt,atoms", [(UE4M4, ("nf4", "sh4")), (E4M3, ("nf4", "sh4n")), (WIDE_U, ("nf5",))])
def test_quantiser_and_sums_against_rationals(fmt, atoms):
    tabs = {"nf4": A.nf(4), "sh4": A.sh(4), "sh4n": A.negate(A.sh(4)), "nf5": A.nf(5)}
    at = [A.to_f32(tabs[a]) for a in atoms]
    M, K, g = 6, 64, 16
    W = si.student_t_weights(M, K, 5.0, 11, row_sigma=0.5)
    c = si.channel_norms(K, 1.0, 12)
    r = ps.pair_search(W, c, at, g, fmt)
    Bk = K // g
    near_tie = 0
    for a, L in enumerate(at):
        codes = ps.unpack_codes(r.codes[a], L.size, M, K)
        for m in range(M):
            for j in range(Bk):
                sc = int(r.scale_code[a, m * Bk + j])
                s = Fr(ps.scale_value(fmt, sc & 0x7FFF)) * (-1 if sc >> 15 else 1)
                w, cb = W[m, j * g:(j + 1) * g], c[j * g:(j + 1) * g]
                ex_codes, num, den, wn, err = _exact_block(w, cb, L, s)
                got = codes[m, j * g:(j + 1) * g].tolist()
                if got != ex_codes:
                    # only allowed where w/s sits within a few binary32 ulps of a midpoint
                    for i, (x, y) in enumerate(zip(got, ex_codes)):
                        if x != y:
                            assert abs(x - y) == 1
                            mid = (Fr(float(L[min(x, y)])) + Fr(float(L[max(x, y)]))) / 2
                            assert abs(Fr(float(w[i])) / s - mid) <= abs(mid) * Fr(4, 2 ** 23)
                            near_tie += 1
                    continue
                cos = float(num) / math.sqrt(float(wn) * float(den))
                assert abs(r.blk_cos[a, m * Bk + j] - cos) < 2e-7
                assert abs(r.blk_err[a, m * Bk + j] - float(err)) <= 1e-5 * float(err) + 1e-30
                # unsaturated elements are within half the widest gap of their entry, in units of s
                x = np.array([float(Fr(float(v)) / s) for v in w])
                inside = (x >= L[0]) & (x <= L[-1])
                gap = np.max(np.diff(L.astype(np.float64)))
                assert np.all(np.abs(x - L[np.array(ex_codes)])[inside] <= gap / 2 + 1e-12)
    assert near_tie <= 2


def test_scale_is_nearest_representable_to_absmax_over_endpoint():
    # brute force over every code of the format: the chosen code minimises |v(q) - absmax/t+|
    L = A.to_f32(A.nf(4))
    W = si.student_t_weights(4, 64, 5.0, 21)
    c = np.ones(64, dtype=np.float32)
    r = ps.pair_search(W, c, [L], 16, UE4M4)
    vals = [Fr(ps.scale_value(UE4M4, q)) for q in range(256)]
    for b in range(16):
        blk = W.reshape(-1, 16)[b]
        target = Fr(float(np.max(np.abs(blk))))                     # t+ = -t- = 1
        best = min(range(256), key=lambda q: (abs(vals[q] - target), q))
        assert int(r.scale_code[0, b]) == best


# ---------------------------------------------------------------- representable weights
@pytest.mark.parametrize("fmt", [UE4M4, E4M3])
def test_representable_weights_give_acos_one(fmt):
    rng = np.random.default_rng(3)
    # atoms on the bf16 grid and scales with <= 5 significant bits: s*L[k] is exact in binary32
    atoms = [si.bf16_round(A.to_f32(A.nf(4))), si.bf16_round(A.to_f32(A.sh(4)))]
    M, K, g = 8, 128, 16
    Bk = K // g
    c = si.channel_norms(K, 1.0, 5)
    for a, L in enumerate(atoms):
        q = rng.integers(20, fmt.max_code - 8, size=(M, Bk))
        s = np.array([[ps.scale_value(fmt, int(v)) for v in row] for row in q])
        k = rng.integers(0, 16, size=(M, Bk, g))
        k[:, :, 0] = 15                                           # every block holds t+ so absmax finds s
        k[:, :, 1] = 0 if L[0] == -1.0 else k[:, :, 1]
        W = (s[:, :, None] * L[k].astype(np.float64)).reshape(M, K).astype(np.float32)
        r = ps.pair_search(W, c, atoms, g, fmt)
        assert np.array_equal(ps.unpack_codes(r.codes[a], 16, M, K), k.reshape(M, K))
        assert np.array_equal(r.scale_code[a] & 0x7FFF, q.reshape(-1))
        assert np.all(r.blk_err[a] == 0.0)
        assert abs(r.acos_atom[a] - 1.0) < 1e-15
        # pairs containing this atom select it wherever the other atom is not also exact
        for p, (pa, pb) in enumerate(ps.all_pairs(2)):
            assert abs(r.acos_pair[p] - 1.0) < 1e-15


# ---------------------------------------------------------------- symmetries and invariants
def _layer(seed=31, M=16, K=256, dtype="bf16"):
    W = si.student_t_weights(M, K, 4.0, seed, row_sigma=0.5, outlier_frac=0.01)
    if dtype == "bf16":
        W = si.bf16_round(W)
    return W, si.channel_norms(K, 1.0, seed + 1)


def _alphabet():
    base = [A.nf(4), A.sh(4)]
    return [A.to_f32(t) for t in base] + [A.to_f32(A.negate(t)) for t in base]


def test_negation_symmetry():
    W, c = _layer()
    for L in (A.nf(4), A.sh(4)):
        a, an = A.to_f32(L), A.to_f32(A.negate(L))
        r1 = ps.pair_search(W, c, [a], 16, UE4M4)
        r2 = ps.pair_search(-W, c, [an], 16, UE4M4)
        assert np.array_equal(r1.scale_code, r2.scale_code)
        assert np.array_equal(r1.blk_err, r2.blk_err)
        assert r1.acos_atom[0] == r2.acos_atom[0]
        c1 = ps.unpack_codes(r1.codes[0], 16, *W.shape)
        c2 = ps.unpack_codes(r2.codes[0], 16, *W.shape)
        assert np.mean(c1 == 15 - c2) > 0.9999                     # mirrored away from exact ties


def test_signed_scale_makes_negated_atoms_redundant():
    W, c = _layer(seed=41)
    at = _alphabet()
    r = ps.pair_search(W, c, at, 16, E4M3)
    for a in (0, 1):
        assert abs(r.acos_atom[a] - r.acos_atom[a + 2]) < 1e-9
        assert np.mean(r.blk_err[a] == r.blk_err[a + 2]) > 0.999
    # and a signed scale never does worse than the unsigned scale with the same magnitude grid
    ru = ps.pair_search(W, c, at, 16, ps.make_fmt(0, 4, 3))
    assert np.all(r.blk_err <= ru.blk_err)


def test_selector_takes_the_smaller_error():
    W, c = _layer(seed=51, M=32)
    at = _alphabet()
    for metric in (ps.WSE, ps.MSE):
        r = ps.pair_search(W, c, at, 16, UE4M4, metric=metric)
        Bk = W.shape[1] // 16
        for p, (a, b) in enumerate(ps.all_pairs(4)):
            bits = (r.sel_words >> np.uint32(p)) & 1
            assert np.array_equal(bits.astype(bool), r.blk_err[b] < r.blk_err[a])
            chosen = np.where(bits.astype(bool), r.blk_err[b], r.blk_err[a])
            assert np.array_equal(chosen, np.minimum(r.blk_err[a], r.blk_err[b]))
            assert chosen.sum(dtype=np.float64) <= min(r.blk_err[a].sum(dtype=np.float64), r.blk_err[b].sum(dtype=np.float64))
            cosv = np.where(bits.astype(bool), r.blk_cos[b], r.blk_cos[a]).astype(np.float64)
            assert abs(cosv.mean() - r.acos_pair[p]) < 1e-7


def test_mse_metric_ignores_channel_norms_in_the_score():
    W, c = _layer(seed=52)
    at = _alphabet()[:2]
    r1 = ps.pair_search(W, c, at, 16, UE4M4, metric=ps.MSE)
    r2 = ps.pair_search(W, np.ones_like(c), at, 16, UE4M4, metric=ps.WSE)
    assert np.array_equal(r1.blk_err, r2.blk_err) and np.array_equal(r1.sel_words, r2.sel_words)
    assert not np.array_equal(r1.acos_pair, r2.acos_pair)          # the cosine still uses c


def test_cos_metric_pair_dominates_singles():
    W, c = _layer(seed=53, M=32)
    at = _alphabet()
    r = ps.pair_search(W, c, at, 16, UE4M4, metric=ps.COS)
    for p, (a, b) in enumerate(ps.all_pairs(4)):
        assert r.acos_pair[p] >= max(r.acos_atom[a], r.acos_atom[b]) - 1e-9
        bits = (r.sel_words >> np.uint32(p)) & 1
        agree = bits.astype(bool) == (r.blk_cos[b] > r.blk_cos[a])
        assert agree.mean() > 0.995                                 # binary32 cosines tie occasionally


def test_power_of_two_invariances():
    W, c = _layer(seed=61)
    at = _alphabet()
    r0 = ps.pair_search(W, c, at, 16, UE4M4, k=0)
    r1 = ps.pair_search(W, c * np.float32(8.0), at, 16, UE4M4, k=0)
    assert np.array_equal(r0.acos_pair, r1.acos_pair) and np.array_equal(r0.sel_words, r1.sel_words)
    assert all(np.array_equal(x, y) for x, y in zip(r0.codes, r1.codes))
    # scaling W by 2^-9 and shifting the block scales by k = +9 changes no code and no cosine
    r2 = ps.pair_search(W * np.float32(2.0 ** -9), c, at, 16, UE4M4, k=9)
    assert np.array_equal(r0.scale_code, r2.scale_code)
    assert all(np.array_equal(x, y) for x, y in zip(r0.codes, r2.codes))
    assert np.array_equal(r0.sel_words, r2.sel_words) and np.array_equal(r0.acos_pair, r2.acos_pair)
    # without the shift the small layer falls into the format's subnormal range and loses fidelity
    r3 = ps.pair_search(W * np.float32(2.0 ** -9), c, at, 16, UE4M4, k=0)
    assert r3.acos_atom[0] < r0.acos_atom[0]


def test_row_permutation_and_thread_count():
    W, c = _layer(seed=71, M=24)
    at = _alphabet()
    perm = np.random.default_rng(0).permutation(W.shape[0])
    r0 = ps.pair_search(W, c, at, 16, E4M3, n_threads=1)
    r1 = ps.pair_search(W[perm], c, at, 16, E4M3, n_threads=4)
    Bk = W.shape[1] // 16
    assert np.array_equal(r0.scale_code.reshape(4, -1, Bk)[:, perm], r1.scale_code.reshape(4, -1, Bk))
    assert np.array_equal(r0.sel_words.reshape(W.shape[0], -1)[perm].reshape(-1), r1.sel_words)
    assert np.allclose(r0.acos_pair, r1.acos_pair, rtol=0, atol=1e-13)
    r2 = ps.pair_search(W, c, at, 16, E4M3, n_threads=3)
    assert np.array_equal(r0.acos_pair, r2.acos_pair) and np.array_equal(r0.blk_err, r2.blk_err)


@pytest.mark.parametrize("g", [8, 16, 32, 64])
def test_block_sum_tree(g):
    # the block error equals the chunk-of-8 tree evaluated independently in numpy binary32 (numpy
    # has no fma, so use binary64 products, which are exact for binary32 factors, rounded once)
    W, c = _layer(seed=81, M=4, K=256, dtype="f32")
    L = A.to_f32(A.nf(4))
    r = ps.pair_search(W, c, [L], g, UE4M4)
    codes = ps.unpack_codes(r.codes[0], 16, *W.shape)
    Bk = W.shape[1] // g
    for blk in range(4 * Bk):
        m, j = divmod(blk, Bk)
        s = np.float32(ps.scale_value(UE4M4, int(r.scale_code[0, blk])))
        w, cb, y = W[m, j * g:(j + 1) * g], c[j * g:(j + 1) * g], L[codes[m, j * g:(j + 1) * g]]
        d = (w.astype(np.float64) - np.float64(s) * y.astype(np.float64)).astype(np.float32)
        cd = cb * d
        parts = []
        for p in range(g // 8):
            acc = np.float32(0)
            for i in range(8 * p, 8 * p + 8):
                acc = np.float32(np.float64(cd[i]) * np.float64(d[i]) + np.float64(acc))
            parts.append(acc)
        while len(parts) > 1:
            parts = [np.float32(parts[2 * i] + parts[2 * i + 1]) for i in range(len(parts) // 2)]
        assert parts[0] == r.blk_err[0, blk]


def test_argument_validation():
    W, c = _layer(M=2, K=64)
    L = A.to_f32(A.nf(4))
    with pytest.raises(ValueError):
        ps.pair_search(W, c, [L], 24, UE4M4)                        # g does not divide K / not a power of two
    with pytest.raises(ValueError):
        ps.pair_search(W, c, [L[::-1].copy()], 16, UE4M4)           # unsorted atom
    with pytest.raises(ValueError):
        ps.pair_search(W, c, [np.abs(L) + 1], 16, UE4M4)            # one-sided atom


# ---------------------------------------------------------------- ranking score of step 2
def test_rank_score_hand_worked_block():
    # L = {-1,0,1}, c = 1, block (1, 0.5, -1, 0.25, 0, 0, 0, 0): s = 1 (representable), x = w, midpoints
    # -0.5 / +0.5 (0.5 is a tie and goes down): w_hat = (1, 0, -1, 0, 0...).
    # num = 1 + 1 = 2, den = 2, wn = 1 + 1/4 + 1 + 1/16 = 37/16: every sum exact in binary32.
    # score = fl(fl(2 / (37/16)) * fl(2 / 2)) = fl(32/37) = cos^2 = 4 / (37/16 * 2)
    L = f32([-1, 0, 1])
    W = f32([[1.0, 0.5, -1.0, 0.25, 0, 0, 0, 0]])
    r = ps.pair_search(W, np.ones(8, dtype=np.float32), [L], 8, WIDE_U)
    assert ps.unpack_codes(r.codes[0], 3, 1, 8).tolist() == [[2, 1, 0, 1, 1, 1, 1, 1]]
    want = np.float32(Fr(32, 37))                                     # one rounding of the exact quotient
    assert r.blk_rank[0, 0] == want
    assert abs(float(r.blk_rank[0, 0]) - float(r.blk_cos[0, 0]) ** 2) < 2e-7
    # channel norms weigh linearly: c = (4,1,1,1,...) gives num = 5, den = 5, wn = 4 + 21/16 = 85/16
    c = np.ones(8, dtype=np.float32); c[0] = 4
    r = ps.pair_search(W, c, [L], 8, WIDE_U)
    assert r.blk_rank[0, 0] == np.float32(Fr(80, 85))


def test_rank_score_conventions_and_sign():
    L = f32(A.nf(4))
    W = np.zeros((1, 48), dtype=np.float32)
    W[0, 16] = 1e-12                                  # second block: the scale underflows, reconstruction 0
    W[0, 32:48] = si.student_t_weights(1, 16, 5.0, 77)[0]
    r = ps.pair_search(W, np.ones(48, dtype=np.float32), [L], 16, UE4M4)
    assert r.blk_rank[0, 0] == 1.0 and r.blk_rank[0, 1] == 0.0        # no norm: 1; nothing reconstructed: 0
    assert 0.9 < r.blk_rank[0, 2] <= 1.0
    # a negative cosine keeps its sign: a one-entry-per-side codebook whose reconstruction points away
    # cannot be built with the absmax rule, so plant it through the channel norms instead: c = 0 on
    # the elements that match, so only the mismatching element counts
    L3 = f32([-1, 0.25, 1])
    Wb = f32([[1.0, -0.1]])                           # -0.1 -> nearest entry 0.25 (midpoint -0.375): w * w_hat < 0
    r = ps.pair_search(Wb, f32([0.0, 1.0]), [L3], 2, WIDE_U)
    assert r.blk_rank[0, 0] < 0 and r.blk_cos[0, 0] < 0
    assert abs(float(r.blk_rank[0, 0]) + float(r.blk_cos[0, 0]) ** 2) < 1e-6


@pytest.mark.parametrize("fmt,g", [(UE4M4, 16), (E4M3, 32), (WIDE, 8), (UE4M4, 64)])
def test_rank_score_is_the_signed_squared_cosine_and_ranks_like_it(fmt, g):
    W = si.bf16_round(si.student_t_weights(48, 1024, 4.0, 810 + g, row_sigma=0.5, outlier_frac=0.002))
    c = si.channel_norms(1024, 1.0, 811)
    tabs = [f32(A.nf(4)), f32(A.sh(4)), f32(A.negate(A.sh(4)))]
    r = ps.pair_search(W, c, tabs, g, fmt)
    # value: against exact rational arithmetic on the reconstruction the oracle reports (codes, scale code)
    cos = r.blk_cos.astype(np.float64)
    assert np.max(np.abs(r.blk_rank.astype(np.float64) - np.sign(cos) * cos * cos)) < 1e-6
    # ranking: wherever two blocks' cosines differ by more than the binary32 resolution, the score orders
    # them the same way
    for a in range(3):
        order = np.argsort(r.blk_rank[a], kind="stable")
        cs = cos[a][order]
        assert np.all(np.diff(cs) > -1e-6)
    # scaling the layer by a power of two (and the layer shift with it) changes no score: the two
    # quotients are formed of sums that scale together
    r2 = ps.pair_search(W * np.float32(2.0 ** -20), c, tabs, g, fmt, k=20)
    assert np.array_equal(r.blk_rank, r2.blk_rank)
    r3 = ps.pair_search(W, c * np.float32(2.0 ** 30), tabs, g, fmt)
    assert np.array_equal(r.blk_rank, r3.blk_rank)
