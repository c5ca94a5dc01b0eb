"""Pins for the argmax scale rule of the oracle (Section "Block Scaling", argmax scaling): hand-worked
blocks, the property the paper states (the dominant element reconstructs to the larger endpoint),
and its relation to the absmax rule with both signs tried."""
import numpy as np
import pytest

from oracle import atoms as A, pairsearch as ps
import sop_inputs as si

WIDE = ps.make_fmt(1, 8, 7, bias=119, max_code=244 * 128 + 127)
E4M3 = ps.make_fmt(1, 4, 3)
S1E5M5 = ps.make_fmt(1, 5, 5)


def f32(x):
    return np.asarray(x, dtype=np.float32)


def test_hand_worked_blocks():
    # endpoints t- = -1, t+ = 0.5: the larger endpoint is the negative one, t* = -1.
    L = f32([-1, 0, 0.5])
    c = f32([1, 1])
    # dominant element -0.9: s = -0.9 / -1 = +0.9 (positive sign); 0.3/0.9 = 0.33 -> 0.5
    r = ps.pair_search(f32([[0.3, -0.9]]), c, [L], 2, WIDE, scale_rule=ps.ARGMAX)
    q = int(r.scale_code[0, 0])
    assert q >> 15 == 0 and abs(ps.scale_value(WIDE, q & 0x7FFF) - 0.9) < 0.9 * 2 ** -8
    assert ps.unpack_codes(r.codes[0], 3, 1, 2).tolist() == [[2, 0]]
    assert abs(r.blk_err[0, 0] - 0.0225) < 2e-3
    # dominant element +0.9: s = 0.9 / -1 = -0.9 (negative sign): w/s = (-1, 0.33) -> (-1, 0.5): w_hat = (0.9, -0.45)
    r = ps.pair_search(f32([[0.9, -0.3]]), c, [L], 2, WIDE, scale_rule=ps.ARGMAX)
    q = int(r.scale_code[0, 0])
    assert q >> 15 == 1 and abs(ps.scale_value(WIDE, q & 0x7FFF) - 0.9) < 0.9 * 2 ** -8
    assert ps.unpack_codes(r.codes[0], 3, 1, 2).tolist() == [[0, 2]]
    assert abs(r.blk_err[0, 0] - 0.0225) < 2e-3
    # the sign-negated atom {-0.5, 0, 1}: t* = +1, so the signs come out the other way round
    Ln = f32(A.negate(L))
    r = ps.pair_search(f32([[0.3, -0.9]]), c, [Ln], 2, WIDE, scale_rule=ps.ARGMAX)
    assert int(r.scale_code[0, 0]) >> 15 == 1
    r = ps.pair_search(f32([[0.9, -0.3]]), c, [Ln], 2, WIDE, scale_rule=ps.ARGMAX)
    assert int(r.scale_code[0, 0]) >> 15 == 0
    # argmax can clip what absmax would not: block (0.8, -0.9) against {-0.5, 0, 1}: x* = -0.9 -> s = -0.9,
    # w/s = (-0.89, 1) -> (-0.5, 1): w_hat = (0.45, -0.9), error 0.35^2
    r = ps.pair_search(f32([[0.8, -0.9]]), c, [Ln], 2, WIDE, scale_rule=ps.ARGMAX)
    assert ps.unpack_codes(r.codes[0], 3, 1, 2).tolist() == [[0, 2]]
    assert abs(r.blk_err[0, 0] - 0.35 ** 2) < 3e-3
    # ties: equal magnitudes of opposite sign -> the positive element is x*
    r = ps.pair_search(f32([[0.5, -0.5]]), c, [Ln], 2, WIDE, scale_rule=ps.ARGMAX)
    assert int(r.scale_code[0, 0]) >> 15 == 0
    # unsigned scale words cannot carry the argmax scale
    with pytest.raises(ValueError):
        ps.pair_search(f32([[0.5, -0.5]]), c, [Ln], 2, ps.make_fmt(0, 4, 4), scale_rule=ps.ARGMAX)


@pytest.mark.parametrize("atom", ["nf4", "sh4", "neg_sh4", "lopsided"])
def test_dominant_element_reconstructs_to_the_larger_endpoint(atom):
    L = {"nf4": A.nf(4), "sh4": A.sh(4), "neg_sh4": A.negate(A.sh(4)),
         "lopsided": np.array([-0.4, -0.1, 0.0, 0.2, 0.5, 1.0])}[atom]
    L = A.to_f32(L)
    M, K, g = 16, 256, 16
    W = si.student_t_weights(M, K, 5.0, 41)
    c = si.channel_norms(K, 0.5, 42)
    r = ps.pair_search(W, c, [L], g, WIDE, scale_rule=ps.ARGMAX)
    codes = ps.unpack_codes(r.codes[0], L.size, M, K).reshape(-1, g)
    blk = W.reshape(-1, g)
    star = np.abs(blk).argmax(axis=1)
    t_pos = L[-1] >= -L[0]
    want = L.size - 1 if t_pos else 0
    assert np.all(codes[np.arange(blk.shape[0]), star] == want)
    # the scale is |x*| / |t*| to the precision of the wide scale word, its sign as the paper states
    sc = r.scale_code[0]
    mag = np.array([ps.scale_value(WIDE, int(q) & 0x7FFF) for q in sc])
    xs = blk[np.arange(blk.shape[0]), star]
    tstar = L[-1] if t_pos else L[0]
    assert np.allclose(mag, np.abs(xs) / abs(tstar), rtol=2 ** -8)
    assert np.array_equal((sc >> 15) == 1, (xs / tstar) < 0)
    # so x* reconstructs to itself within the scale word's rounding
    what = np.where((sc >> 15) == 1, -mag, mag) * tstar
    assert np.allclose(what, xs, rtol=2 ** -8)


def test_relation_to_absmax_with_both_signs():
    M, K, g = 32, 512, 16
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 51, row_sigma=0.4))
    c = si.channel_norms(K, 1.0, 52)
    nf4, sh4 = A.to_f32(A.nf(4)), A.to_f32(A.sh(4))
    e2m3 = A.to_f32(A.exmy_grid(2, 3))
    for fmt in (E4M3, S1E5M5):
        arg = ps.pair_search(W, c, [nf4, sh4, e2m3], g, fmt, scale_rule=ps.ARGMAX)
        both = ps.pair_search(W, c, [nf4, sh4, e2m3], g, fmt)
        # NF4 has endpoints of equal magnitude: the argmax scale magnitude is the absmax one, so the
        # argmax candidate is one of the two candidates absmax tries, and the better of the two is no worse
        assert np.array_equal(arg.scale_code[0] & 0x7FFF, both.scale_code[0] & 0x7FFF)
        assert np.all(both.blk_err[0] <= arg.blk_err[0])
        same_sign = (arg.scale_code[0] >> 15) == (both.scale_code[0] >> 15)
        assert np.array_equal(arg.blk_err[0][same_sign], both.blk_err[0][same_sign])
        assert 0.3 < same_sign.mean() < 1.0
        # a grid closed under negation: the sign changes nothing, argmax equals absmax (block errors
        # bit for bit; a scaled weight exactly halfway between two grid values goes to the other
        # neighbour under the other sign, with the same error but another cosine)
        assert np.array_equal(arg.blk_err[2], both.blk_err[2])
        assert abs(arg.acos_atom[2] - both.acos_atom[2]) < 1e-5
        # in general trying both signs under absmax is at least as good on average
        assert both.acos_atom[1] >= arg.acos_atom[1] - 1e-4
        # pairs still pick the smaller error per block
        sel = (arg.sel_words & 1).astype(bool)
        assert np.array_equal(sel, arg.blk_err[1] < arg.blk_err[0])


def test_negating_layer_and_atom_mirrors_the_result():
    M, K, g = 12, 256, 16
    W = si.bf16_round(si.student_t_weights(M, K, 4.0, 61))
    c = si.channel_norms(K, 1.0, 62)
    L = A.to_f32(A.sh(4))
    r1 = ps.pair_search(W, c, [L], g, S1E5M5, scale_rule=ps.ARGMAX)
    r2 = ps.pair_search(-W, c, [A.to_f32(A.negate(L))], g, S1E5M5, scale_rule=ps.ARGMAX)
    # blocks without an exact +/- tie for the dominant element mirror exactly
    blk = W.reshape(-1, g)
    tie = blk.max(axis=1) == -blk.min(axis=1)
    assert np.array_equal(r1.blk_err[0][~tie], r2.blk_err[0][~tie])
    assert np.array_equal(r1.scale_code[0][~tie], r2.scale_code[0][~tie])
