"""Materialisation in the oracle: the scale word of every block with its sign bit and its codebook
selector at the bit positions the paper fixes, and the block's codes as a dense n-bit payload.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

Followed passages: Section "Scale Format", paragraphs "The SwExMy notation" (a b-bit container holds
w sign bits, x exponent bits, y mantissa bits and m = b - w - x - y metabits), "Bit placement"
(sign and metabits at the two ends, exponent then mantissa in the middle; with a sign bit, bit b-1
is the sign and the metabits are bits m-1..0; without one, bit b-1 becomes the first metabit and
the others are bits m-2..0) and "Worked examples" (the layout table); Section "Per-Layer Pair
Search" (one metabit per block says which of the two codebooks reconstructs it); the bits-per-weight
identity s/g + b of the introduction (a block of g = 16 six-bit codes is 12 bytes, 2n bytes for n bits).

Readings (the paper is silent):
  - the selector is the FIRST metabit: bit b-1 without a sign bit, bit m-1 with one; the other
    metabits are written as zero;
  - a format without a metabit cannot carry a selector: packing one into it is an error;
  - the codes of a block form a little-endian bit string: code i occupies bits i*n .. i*n+n-1,
    byte j holds bits 8j .. 8j+7 (for n = 4 this is two codes per byte, the first in the low half).
"""
from __future__ import annotations

import numpy as np

from . import pairsearch as ops


def layout(w: int, x: int, y: int, b: int) -> dict:
    """Bit positions inside the b-bit container."""
    m = b - w - x - y
    if w not in (0, 1) or x < 1 or y < 0 or m < 0 or b > 16:
        raise ValueError("not a SwExMy word in a container of at most 16 bits")
    low_meta = m if w == 1 else max(m - 1, 0)          # metabits at the LSB end
    if m == 0:
        sel_pos = None
    elif w == 1:
        sel_pos = m - 1
    else:
        sel_pos = b - 1
    return dict(m=m, sign_pos=(b - 1) if w == 1 else None, mag_shift=low_meta, mag_bits=x + y, sel_pos=sel_pos)


def pack_words(scale_code: np.ndarray, sel: np.ndarray | None, w: int, x: int, y: int, b: int) -> np.ndarray:
    """scale_code: u16 per block as the search writes it (bit 15 = sign, low bits = magnitude code
    of x+y bits); sel: 0/1 per block or None.  Returns the container value of every block (u16)."""
    lay = layout(w, x, y, b)
    sc = np.asarray(scale_code, dtype=np.uint16).astype(np.uint32)
    mag = sc & 0x7FFF
    sgn = sc >> 15
    if (mag >> lay["mag_bits"]).any():
        raise ValueError("magnitude code wider than x + y bits")
    if w == 0 and sgn.any():
        raise ValueError("sign bit set for an unsigned format")
    word = mag << lay["mag_shift"]
    if w == 1:
        word |= sgn << lay["sign_pos"]
    if sel is not None:
        if lay["sel_pos"] is None:
            raise ValueError("the format has no metabit for the selector")
        word |= (np.asarray(sel).astype(np.uint32) & 1) << lay["sel_pos"]
    return word.astype(np.uint16)


def unpack_words(words: np.ndarray, w: int, x: int, y: int, b: int):
    """Inverse of pack_words: (sign, magnitude code, selector) per block (selector 0 without metabit)."""
    lay = layout(w, x, y, b)
    v = np.asarray(words, dtype=np.uint16).astype(np.uint32)
    mag = (v >> lay["mag_shift"]) & ((1 << lay["mag_bits"]) - 1)
    sgn = (v >> lay["sign_pos"]) & 1 if w == 1 else np.zeros_like(v)
    sel = (v >> lay["sel_pos"]) & 1 if lay["sel_pos"] is not None else np.zeros_like(v)
    return sgn, mag, sel


def pack_payload(codes: np.ndarray, n_bits: int) -> np.ndarray:
    """codes [N_b, g] -> [N_b, g*n/8] bytes, little-endian bit string per block."""
    cd = np.asarray(codes).astype(np.uint32)
    Nb, g = cd.shape
    if (cd >> n_bits).any():
        raise ValueError("code wider than n bits")
    bits = np.zeros((Nb, g * n_bits), dtype=np.uint8)
    for i in range(g):
        for t in range(n_bits):
            bits[:, i * n_bits + t] = (cd[:, i] >> t) & 1
    return np.packbits(bits, axis=1, bitorder="little")


def unpack_payload(payload: np.ndarray, n_bits: int, g: int) -> np.ndarray:
    bits = np.unpackbits(np.asarray(payload, dtype=np.uint8), axis=1, bitorder="little").astype(np.uint32)
    out = np.zeros((bits.shape[0], g), dtype=np.uint32)
    for i in range(g):
        for t in range(n_bits):
            out[:, i] |= bits[:, i * n_bits + t] << t
    return out


def code_bits(n_entries: int) -> int:
    n = 1
    while (1 << n) < n_entries:
        n += 1
    return n


def materialise(res: ops.Result, tabs: list, M: int, K: int, g: int, a: int, b: int | None, q: int | None,
                w: int, x: int, y: int, cb: int):
    """Pick, per block, atom a (selector 0) or atom b (selector 1, bit q of the block's selector
    word) out of an emitting search result and pack it.  b = None: single codebook, no selector.
    Returns (words u16 [N_b], payload u8 [N_b, g*n/8], n)."""
    Nb = M * K // g
    ca = ops.unpack_codes(res.codes[a], tabs[a].size, M, K).reshape(Nb, g)
    if b is None:
        n = code_bits(tabs[a].size)
        return pack_words(res.scale_code[a], None, w, x, y, cb), pack_payload(ca, n), n
    cbk = ops.unpack_codes(res.codes[b], tabs[b].size, M, K).reshape(Nb, g)
    sel = (res.sel_words >> q) & 1
    n = code_bits(max(tabs[a].size, tabs[b].size))
    sc = np.where(sel == 1, res.scale_code[b], res.scale_code[a])
    cd = np.where(sel[:, None] == 1, cbk, ca)
    return pack_words(sc, sel, w, x, y, cb), pack_payload(cd, n), n


def reconstruct(words: np.ndarray, payload: np.ndarray, n_bits: int, g: int, M: int, K: int, tab_a: np.ndarray,
                tab_b: np.ndarray | None, fmt, k: int, w: int, x: int, y: int, cb: int) -> np.ndarray:
    """Decoder: [M,K] binary32 weights s * L[code] from the packed arrays (s = +-value(magnitude code) * 2^-k)."""
    sgn, mag, sel = unpack_words(words, w, x, y, cb)
    val = np.array([ops.scale_value(fmt, int(qv)) for qv in range(int(mag.max()) + 1)], dtype=np.float64)
    s = (val[mag] * 2.0 ** (-k)).astype(np.float32)
    s = np.where(sgn == 1, -s, s).astype(np.float32)
    cd = unpack_payload(payload, n_bits, g)
    ta = np.asarray(tab_a, dtype=np.float32)
    yv = ta[np.minimum(cd, ta.size - 1)]
    if tab_b is not None:
        tb = np.asarray(tab_b, dtype=np.float32)
        yv = np.where(sel[:, None] == 1, tb[np.minimum(cd, tb.size - 1)], yv)
    return (s[:, None] * yv).astype(np.float32).reshape(M, K)
