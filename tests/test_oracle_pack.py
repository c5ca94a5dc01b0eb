"""Pins for the oracle's materialisation: scale-word bit positions against the paper's layout table,
payload size against the bits-per-weight identity, and decode(pack(search)) against the search."""
import os

import numpy as np
import pytest

from oracle import atoms as A, pack as PK, pairsearch as ps
import sop_inputs as si

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_layouts():
    out = []
    for line in open(os.path.join(GOLD, "scale_word_layouts.txt")):
        line = line.split("#")[0].strip()
        if line:
            key, val = [t.strip() for t in line.split("=")]
            name, b, w, x, y = key.split("_")
            out.append((name, int(b), int(w), int(x), int(y), val))
    return out


@pytest.mark.parametrize("name,b,w,x,y,text", read_layouts())
def test_bit_positions_follow_the_printed_layouts(name, b, w, x, y, text):
    assert len(text) == b
    pos = {ch: sum(1 << (b - 1 - i) for i, t in enumerate(text) if t == ch) for ch in "semu"}
    m = b - w - x - y
    all_mag = (1 << (x + y)) - 1
    # magnitude field: exponent followed by mantissa in the contiguous middle
    word = int(PK.pack_words(np.array([all_mag], np.uint16), None, w, x, y, b)[0])
    assert word == pos["e"] | pos["m"]
    exp_only = ((1 << x) - 1) << y
    assert int(PK.pack_words(np.array([exp_only], np.uint16), None, w, x, y, b)[0]) == pos["e"]
    if w:
        assert int(PK.pack_words(np.array([0x8000], np.uint16), None, w, x, y, b)[0]) == pos["s"]
    else:
        assert pos["s"] == 0
    assert bin(pos["u"]).count("1") == m
    if m:
        sel_word = int(PK.pack_words(np.array([0], np.uint16), np.array([1]), w, x, y, b)[0])
        assert sel_word & pos["u"] == sel_word and bin(sel_word).count("1") == 1
        # the selector is the first metabit: the topmost metabit position
        assert sel_word == 1 << (pos["u"].bit_length() - 1)
    else:
        with pytest.raises(ValueError):
            PK.pack_words(np.array([0], np.uint16), np.array([1]), w, x, y, b)
    # nothing ever lands outside the container, and unpacking inverts packing
    rng = np.random.default_rng(b * 100 + x)
    mag = rng.integers(0, all_mag + 1, 200).astype(np.uint16)
    sgn = (rng.integers(0, 2, 200) * w).astype(np.uint16)
    sel = rng.integers(0, 2, 200) if m else None
    words = PK.pack_words(mag | (sgn << 15), sel, w, x, y, b)
    assert (words.astype(np.uint32) >> b == 0).all()
    s2, m2, l2 = PK.unpack_words(words, w, x, y, b)
    assert np.array_equal(s2, sgn) and np.array_equal(m2, mag)
    if m:
        assert np.array_equal(l2, sel)


def test_payload_is_n_bits_per_code_little_endian():
    # n = 4: two codes a byte, the first in the low half
    cd = np.arange(16, dtype=np.uint8).reshape(1, 16)
    assert np.array_equal(PK.pack_payload(cd, 4)[0], np.array([(2 * i) | ((2 * i + 1) << 4) for i in range(8)], np.uint8))
    # n = 6, g = 16: 12 bytes (2n bytes for n-bit codes); the bit string read as one integer
    rng = np.random.default_rng(3)
    for n in (3, 4, 5, 6, 8):
        for g in (8, 16, 32, 64):
            cd = rng.integers(0, 1 << n, (5, g))
            pl = PK.pack_payload(cd, n)
            assert pl.shape == (5, g * n // 8)
            for r in range(5):
                big = sum(int(c) << (i * n) for i, c in enumerate(cd[r]))
                assert bytes(pl[r]) == big.to_bytes(g * n // 8, "little")
            assert np.array_equal(PK.unpack_payload(pl, n, g), cd)
    assert PK.pack_payload(np.zeros((1, 16), np.uint8), 6).shape[1] == 12
    with pytest.raises(ValueError):
        PK.pack_payload(np.full((1, 16), 16), 4)


def test_bits_per_weight_of_the_packed_arrays():
    # stored bits per weight = (container bits + g * n) / g, the paper's s/g + b
    for (b, g, n) in ((12, 16, 6), (8, 16, 6), (8, 16, 4), (8, 16, 5), (12, 16, 4)):
        payload_bytes = g * n // 8
        assert (b + 8 * payload_bytes) / g == A.bits_per_weight(b, g, n)


@pytest.mark.parametrize("fmtname", ["UE4M3", "S1E5M5", "S0E5M5"])
def test_decoding_the_packed_layer_reproduces_the_search(fmtname):
    w, x, y, b = {"UE4M3": (0, 4, 3, 8), "S1E5M5": (1, 5, 5, 12), "S0E5M5": (0, 5, 5, 12)}[fmtname]
    fmt = ps.make_fmt(w, x, y)
    M, K, g = 24, 256, 16
    W = si.bf16_round(si.student_t_weights(M, K, 5.0, 77, row_sigma=0.3))
    c = si.channel_norms(K, 0.8, 78)
    tabs = [A.to_f32(A.nf(4)), A.to_f32(A.sh(4))]
    k = 3
    res = ps.pair_search(W, c, tabs, g, fmt, k=k)
    words, payload, n = PK.materialise(res, tabs, M, K, g, 0, 1, 0, w, x, y, b)
    assert n == 4 and payload.shape == (M * K // g, 8) and (words.astype(np.uint32) >> b == 0).all()
    What = PK.reconstruct(words, payload, n, g, M, K, tabs[0], tabs[1], fmt, k, w, x, y, b)
    # the weighted error of the decoded layer, block by block, is the search's error of the chosen atom
    d = (W.astype(np.float64) - What.astype(np.float64)).reshape(-1, g)
    err = (np.tile(c.astype(np.float64), M).reshape(-1, g) * d * d).sum(axis=1)
    sel = (res.sel_words & 1).astype(bool)
    chosen = np.where(sel, res.blk_err[1], res.blk_err[0]).astype(np.float64)
    assert np.allclose(err, chosen, rtol=2e-5, atol=1e-12)
    assert sel.any() and not sel.all()
    # single codebook into a format without a metabit
    w1, p1, n1 = PK.materialise(res, tabs, M, K, g, 1, None, None, w, x, y, b)
    What1 = PK.reconstruct(w1, p1, n1, g, M, K, tabs[1], None, fmt, k, w, x, y, b)
    d1 = (W.astype(np.float64) - What1.astype(np.float64)).reshape(-1, g)
    err1 = (np.tile(c.astype(np.float64), M).reshape(-1, g) * d1 * d1).sum(axis=1)
    assert np.allclose(err1, res.blk_err[1].astype(np.float64), rtol=2e-5, atol=1e-12)
