"""ctypes front end of the C oracle (sop_oracle.c).  TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sop_oracle.c")
_LIB = os.path.join(_HERE, "libsop_oracle.so")

WSE, COS, MSE = 0, 1, 2
ABSMAX, ARGMAX = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with contraction off so every written operation rounds once."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
                               "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Fmt(C.Structure):
    _fields_ = [("sign_bits", C.c_int), ("exp_bits", C.c_int), ("man_bits", C.c_int),
                ("bias", C.c_int), ("max_code", C.c_int)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.sopo_scale_value.restype = C.c_double
        L.sopo_scale_value.argtypes = [C.POINTER(_Fmt), C.c_int]
        L.sopo_scale_encode.argtypes = [C.POINTER(_Fmt), C.c_float]
        L.sopo_scale_encode_exhaustive.argtypes = [C.POINTER(_Fmt), C.c_float]
        L.sopo_pair_search.restype = C.c_int
        _lib = L
    return _lib


def make_fmt(sign_bits, exp_bits, man_bits, container_bits=None, bias=-1, max_code=-1) -> _Fmt:
    """Scale format descriptor; defaults follow the paper's bias 2^(x-1)-1 with every code finite."""
    if bias < 0:
        bias = 2 ** (exp_bits - 1) - 1
    if max_code < 0:
        max_code = 2 ** (exp_bits + man_bits) - 1
    return _Fmt(sign_bits, exp_bits, man_bits, bias, max_code)


def scale_value(fmt: _Fmt, q: int) -> float:
    return lib().sopo_scale_value(C.byref(fmt), int(q))


def scale_encode(fmt: _Fmt, s: float, exhaustive: bool = False) -> int:
    f = lib().sopo_scale_encode_exhaustive if exhaustive else lib().sopo_scale_encode
    return f(C.byref(fmt), C.c_float(float(s)))


def all_pairs(n_atoms: int) -> np.ndarray:
    """Every pair a < b in lexicographic order."""
    return np.array([(a, b) for a in range(n_atoms) for b in range(a + 1, n_atoms)], dtype=np.int32).reshape(-1, 2)


@dataclass
class Result:
    acos_pair: np.ndarray
    acos_atom: np.ndarray
    sel_words: np.ndarray    # [M*K/g] u32, bit p = selector of pair p
    scale_code: np.ndarray   # [A][M*K/g] u16
    codes: list              # per atom: packed code plane (u8)
    blk_err: np.ndarray      # [A][M*K/g] f32
    blk_cos: np.ndarray      # [A][M*K/g] f32
    blk_rank: np.ndarray = None   # [A][M*K/g] f32: ranking score of step 2 (signed squared block cosine, binary32)


def pair_search(W: np.ndarray, c: np.ndarray, atoms: list, g: int, fmt: _Fmt, k: int = 0, metric: int = WSE,
                pairs: np.ndarray | None = None, want_codes: bool = True, n_threads: int = 0,
                scale_rule: int = ABSMAX) -> Result:
    """Run the oracle on a layer.  W is fp32 [M,K] (bf16 data already widened); atoms is a list of
    ascending fp32 tables."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    c = np.ascontiguousarray(c, dtype=np.float32)
    M, K = W.shape
    A = len(atoms)
    tabs = [np.ascontiguousarray(a, dtype=np.float32) for a in atoms]
    n_entries = np.array([t.size for t in tabs], dtype=np.int32)
    flat = np.concatenate(tabs).astype(np.float32)
    if pairs is None:
        pairs = all_pairs(A)
    pairs = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
    P = pairs.shape[0]
    Bk = K // g
    Nb = M * Bk
    plane = [M * K // 2 if t.size <= 16 else M * K for t in tabs]
    acos_pair = np.zeros(max(P, 1), dtype=np.float64)
    acos_atom = np.zeros(A, dtype=np.float64)
    sel = np.zeros(Nb, dtype=np.uint32)
    sc = np.zeros((A, Nb), dtype=np.uint16)
    # one code plane per atom, back to back: half a byte per element up to 16 entries, else a byte
    codes = np.zeros(sum(plane), dtype=np.uint8) if want_codes else None
    be = np.zeros((A, Nb), dtype=np.float32)
    bc = np.zeros((A, Nb), dtype=np.float32)
    br = np.zeros((A, Nb), dtype=np.float32)

    def p(a, t):
        return a.ctypes.data_as(C.POINTER(t)) if a is not None else None

    rc = lib().sopo_pair_search(
        p(W, C.c_float), C.c_int64(M), C.c_int64(K), C.c_int64(K), p(c, C.c_float), C.c_int(g),
        C.c_int(A), p(n_entries, C.c_int), p(flat, C.c_float), C.c_int(P), p(pairs, C.c_int),
        C.byref(fmt), C.c_int(k), C.c_int(metric), C.c_int(scale_rule),
        p(acos_pair, C.c_double), p(acos_atom, C.c_double), p(sel, C.c_uint32), p(sc, C.c_uint16),
        p(codes, C.c_uint8), p(be, C.c_float), p(bc, C.c_float), p(br, C.c_float), C.c_int(n_threads))
    if rc != 0:
        raise ValueError(f"oracle rejected the arguments (code {rc})")
    code_list = None
    if codes is not None:
        offs = np.concatenate([[0], np.cumsum(plane)])
        code_list = [codes[offs[a]:offs[a + 1]] for a in range(A)]
    return Result(acos_pair[:P], acos_atom, sel, sc, code_list, be, bc, br)


def unpack_codes(plane: np.ndarray, n_entries: int, M: int, K: int) -> np.ndarray:
    """Code plane -> [M,K] array of indices."""
    if n_entries <= 16:
        out = np.empty(M * K, dtype=np.uint8)
        out[0::2] = plane & 0xF
        out[1::2] = plane >> 4
        return out.reshape(M, K)
    return plane.reshape(M, K).copy()


def num_threads() -> int:
    return lib().sopo_num_threads()
