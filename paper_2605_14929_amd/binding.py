"""ctypes binding of include/sop.h.  Names follow the C entry points; no arithmetic lives here."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
F32, BF16 = 0, 1
SCALE_ABSMAX, SCALE_ARGMAX = 0, 1
SEL_WSE, SEL_COS, SEL_MSE = 0, 1, 2
MAX_ATOMS, MAX_ENTRIES = 8, 64
_STATUS = {1: "SOP_EINVAL", 2: "SOP_ESHAPE", 3: "SOP_EATOM", 4: "SOP_EFMT", 5: "SOP_ENOMEM", 6: "SOP_EHIP"}


class SopError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{_STATUS.get(status, status)}: {text}")
        self.status = status


class ScaleFmt(C.Structure):
    """sop_scale_fmt: SwExMy scale word in a b-bit container."""
    _fields_ = [("sign_bits", C.c_int), ("exp_bits", C.c_int), ("man_bits", C.c_int), ("container_bits", C.c_int),
                ("bias", C.c_int), ("max_code", C.c_int)]


class _Layer(C.Structure):
    """sop_layer: one linear layer of a model-wide search."""
    _fields_ = [("W", C.c_void_p), ("M", C.c_int64), ("K", C.c_int64), ("ldw", C.c_int64), ("c", C.c_void_p),
                ("k", C.c_int), ("sel_words", C.c_void_p)]


class WeightFmt(C.Structure):
    """sop_weight_fmt: ExMy weight grid."""
    _fields_ = [("exp_bits", C.c_int), ("man_bits", C.c_int), ("bias", C.c_int), ("max_code", C.c_int)]


class _Atom(C.Structure):
    _fields_ = [("n_entries", C.c_int), ("values", C.POINTER(C.c_float))]


LAYER_MAX_P = 7
LAYER_MAX_ATOMS = 16
LAYER_MAX_PAIRS = 120


class _LayerOpts(C.Structure):
    """sop_layer_opts"""
    _fields_ = [("n_p", C.c_int), ("p_percent", C.c_double * LAYER_MAX_P), ("fit_entries", C.c_int), ("fit_iters", C.c_int),
                ("fit_bins", C.c_int), ("fit_init", C.POINTER(C.c_float)), ("weighted_fit", C.c_int),
                ("fit_grid", C.POINTER(C.c_double)), ("n_fit_grid", C.c_int), ("pack", C.c_int)]


class _LayerResult(C.Structure):
    """sop_layer_result"""
    _fields_ = [("kind", C.c_int), ("a", C.c_int), ("b", C.c_int), ("j", C.c_int), ("p_percent", C.c_double), ("acos", C.c_double),
                ("n_entries_b", C.c_int), ("table_b", C.c_float * MAX_ENTRIES), ("acos_fixed", C.c_double * LAYER_MAX_PAIRS),
                ("acos_atom", C.c_double * LAYER_MAX_ATOMS), ("acos_fitted", (C.c_double * LAYER_MAX_P) * LAYER_MAX_ATOMS), ("n_bits", C.c_int)]


class _Outputs(C.Structure):
    _fields_ = [("acos_pair", C.c_void_p), ("acos_atom", C.c_void_p), ("sel_words", C.c_void_p),
                ("scale_code", C.c_void_p), ("codes", C.c_void_p), ("blk_cos", C.c_void_p), ("blk_err", C.c_void_p),
                ("blk_rank", C.c_void_p)]


def lib_path() -> str:
    return os.path.join(_HERE, "libsop_hip.so")


_lib = None


def lib():
    """Load libsop_hip.so; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise SopError(6, f"{path} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(the pair search has no CPU fallback)")
        # PyTorch ships its own HIP runtime; two HIP runtimes in one process cannot both own the GPU.
        # Importing torch first makes the loader resolve this library's libamdhip64.so.7 dependency
        # to the copy torch already mapped (same soname), so both sides share one runtime.
        import torch  # noqa: F401
        L = C.CDLL(path)
        L.sop_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
        L.sop_destroy.argtypes = [C.c_void_p]
        L.sop_set_alphabet.argtypes = [C.c_void_p, C.POINTER(_Atom), C.c_int]
        L.sop_check_alphabet.argtypes = [C.POINTER(_Atom), C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int64)]
        L.sop_set_pairs.argtypes = [C.c_void_p, C.POINTER(C.c_int), C.c_int]
        L.sop_set_scale_rule.argtypes = [C.c_void_p, C.c_int]
        L.sop_workspace_bytes.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.POINTER(C.c_size_t)]
        L.sop_pair_search.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_int,
                                      ScaleFmt, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.POINTER(_Outputs), C.c_void_p]
        L.sop_pair_search_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_int,
                                             ScaleFmt, C.c_int, C.c_int, C.POINTER(_Outputs), C.c_void_p]
        L.sop_search_layer_workspace.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.POINTER(_LayerOpts), C.POINTER(C.c_size_t)]
        L.sop_search_layer.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_int, ScaleFmt, C.c_int,
                                       C.c_int, C.POINTER(_Atom), C.c_int, C.POINTER(_LayerOpts), C.c_void_p, C.c_size_t,
                                       C.POINTER(_LayerResult), C.c_void_p, C.c_void_p, C.c_void_p]
        L.sop_prepare_scale.argtypes = [C.c_void_p, ScaleFmt, C.c_int, C.c_void_p]
        L.sop_last_error.argtypes = [C.c_void_p]
        L.sop_last_error.restype = C.c_char_p
        L.sop_atom_nf.argtypes = [C.c_int, C.POINTER(C.c_float)]
        L.sop_atom_sh.argtypes = [C.c_int, C.c_double, C.c_double, C.POINTER(C.c_float)]
        L.sop_atom_negate.argtypes = [C.POINTER(C.c_float), C.c_int, C.POINTER(C.c_float)]
        L.sop_lloyd_1d.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_int64, C.POINTER(C.c_double), C.c_int, C.c_int]
        L.sop_atom_bof.argtypes = [C.c_int, C.POINTER(C.c_double), C.c_int64, C.c_int, C.c_int, C.POINTER(C.c_float)]
        L.sop_dd_histogram.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_int, C.c_int,
                                       C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sop_dd_fit.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]     # (host arrays by address: the fit is called in loops)
        L.sop_dd_fit_grid.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.sop_weight_grid.argtypes = [WeightFmt, C.c_double, C.c_void_p, C.c_void_p]
        L.sop_scale_histogram.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_float, C.c_float,
                                          ScaleFmt, C.c_void_p, C.c_void_p]
        L.sop_layer_scope_error.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, WeightFmt, ScaleFmt,
                                            C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sop_sum_f32.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        L.sop_read_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        L.sop_issue_probe.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float, C.c_float, C.c_void_p, C.POINTER(C.c_int), C.c_void_p]
        L.sop_pair_search_layers.argtypes = [C.c_void_p, C.POINTER(_Layer), C.c_int, C.c_int, C.c_int, ScaleFmt, C.c_int,
                                             C.c_void_p, C.c_void_p, C.c_void_p]
        L.sop_partition.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sop_partition_levels.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(C.c_int64), C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_void_p]
        L.sop_dd_histogram_levels.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_int, C.c_int,
                                              C.c_int64, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.sop_pack_blocks.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, ScaleFmt, C.c_void_p, C.c_void_p, C.c_int,
                                      C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                      C.POINTER(C.c_int), C.c_void_p]
        L.sop_layer_shift.argtypes = [C.POINTER(C.c_int64), C.c_int64, ScaleFmt, C.POINTER(C.c_int), C.POINTER(C.c_double)]
        _lib = L
    return _lib


def _fp(a, t=C.c_float):
    return a.ctypes.data_as(C.POINTER(t))


def _check(status, ctx=None):
    if status != 0:
        raise SopError(status, (lib().sop_last_error(ctx) or b"").decode())


# ---- host atom builders (C implementations) ----
def sop_atom_nf(n_bits: int) -> np.ndarray:
    out = np.empty(2 ** n_bits, dtype=np.float32)
    _check(lib().sop_atom_nf(n_bits, _fp(out)))
    return out


def sop_atom_sh(n_bits: int, alpha: float = 1.5, c: float = -0.02) -> np.ndarray:
    out = np.empty(2 ** n_bits, dtype=np.float32)
    _check(lib().sop_atom_sh(n_bits, alpha, c, _fp(out)))
    return out


def sop_atom_negate(values: np.ndarray) -> np.ndarray:
    v = np.ascontiguousarray(values, dtype=np.float32)
    out = np.empty_like(v)
    _check(lib().sop_atom_negate(_fp(v), v.size, _fp(out)))
    return out


def sop_lloyd_1d(samples: np.ndarray, weights, init: np.ndarray, iters: int) -> np.ndarray:
    x = np.ascontiguousarray(samples, dtype=np.float64)
    w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float64)
    cent = np.array(init, dtype=np.float64).copy()
    _check(lib().sop_lloyd_1d(_fp(x, C.c_double), None if w is None else _fp(w, C.c_double), x.size, _fp(cent, C.c_double), cent.size, iters))
    return cent


def sop_atom_bof(n_bits: int, draws: np.ndarray, g: int = 16, iters: int = 50) -> np.ndarray:
    d = np.ascontiguousarray(draws, dtype=np.float64)
    out = np.empty(2 ** n_bits, dtype=np.float32)
    _check(lib().sop_atom_bof(n_bits, _fp(d, C.c_double), d.size, g, iters, _fp(out)))
    return out


def sop_dd_fit(hist: np.ndarray, n_entries: int, iters: int, init: np.ndarray) -> np.ndarray:
    """Weighted Lloyd fit on an [H] int64 histogram (host)."""
    h = np.ascontiguousarray(hist, dtype=np.int64).reshape(-1)
    ini = np.ascontiguousarray(init, dtype=np.float32)
    out = np.empty(n_entries, dtype=np.float32)
    _check(lib().sop_dd_fit(h.ctypes.data, h.size, n_entries, iters, ini.ctypes.data, out.ctypes.data))
    return out


def sop_dd_fit_grid(hist: np.ndarray, cand: np.ndarray, n_entries: int):
    """Best n_entries of the ascending candidate values for an [H] int64 histogram (host):
    (indices into cand, cost)."""
    h = np.ascontiguousarray(hist, dtype=np.int64).reshape(-1)
    g = np.ascontiguousarray(cand, dtype=np.float64).reshape(-1)
    chosen = np.empty(n_entries, dtype=np.int32)
    cost = C.c_double(0.0)
    _check(lib().sop_dd_fit_grid(h.ctypes.data, h.size, g.ctypes.data, g.size, n_entries, chosen.ctypes.data, C.byref(cost)))
    return chosen.astype(np.int64), cost.value


def sop_weight_grid(wfmt: "WeightFmt", top: float = 0.0) -> np.ndarray:
    """Distinct values of an ExMy weight grid, ascending (host)."""
    out = np.empty(2 * (1 << (wfmt.exp_bits + wfmt.man_bits)) + 1, dtype=np.float64)
    n = C.c_int(0)
    _check(lib().sop_weight_grid(wfmt, C.c_double(top), out.ctypes.data, C.byref(n)))
    return out[:n.value].copy()


def sop_layer_shift(hist: np.ndarray, n_blocks: int, fmt: "ScaleFmt"):
    """(k*, fraction of block scales in the normal range) from a [2, 320] int64 exponent histogram (host)."""
    h = np.ascontiguousarray(hist, dtype=np.int64).reshape(-1)
    if h.size != 640:
        raise SopError(1, "the exponent histogram has 2 x 320 entries")
    k, frac = C.c_int(), C.c_double()
    _check(lib().sop_layer_shift(_fp(h, C.c_int64), n_blocks, fmt, C.byref(k), C.byref(frac)))
    return k.value, frac.value


def sop_check_alphabet(tables):
    """Host-only check of the search table built for these atoms; returns (n_bins, n_checked)."""
    tabs = [np.ascontiguousarray(t, dtype=np.float32) for t in tables]
    arr = (_Atom * len(tabs))()
    for i, t in enumerate(tabs):
        arr[i].n_entries = t.size
        arr[i].values = _fp(t)
    nb, nc = C.c_int(), C.c_int64()
    _check(lib().sop_check_alphabet(arr, len(tabs), C.byref(nb), C.byref(nc)))
    return nb.value, nc.value


_FMTS = {
    "UE4M4": (0, 4, 4, 8, -1, -1), "E4M3": (1, 4, 3, 8, -1, -1), "UE4M3": (0, 4, 3, 8, -1, -1),
    "UE4M6": (0, 4, 6, 10, -1, -1), "E4M5": (1, 4, 5, 10, -1, -1), "UE5M7": (0, 5, 7, 12, -1, -1),
    "E5M6": (1, 5, 6, 12, -1, -1), "E4M7": (1, 4, 7, 12, -1, -1), "S1E5M5": (1, 5, 5, 12, -1, -1),
    "S0E6M5": (0, 6, 5, 12, -1, -1), "UE5M3": (0, 5, 3, 8, -1, -1),
    # bf16-like 16-bit scale kept inside binary32's normal range (values 2^-125 .. < 2^126)
    "E8M7": (1, 8, 7, 16, 119, 244 * 128 + 127),
}


def fmt_by_name(name: str) -> ScaleFmt:
    return ScaleFmt(*_FMTS[name])


def build_alphabet(names, bof_draws=None) -> list:
    """Tables for names such as "NF4", "SH5", "BOF4", "-NF4" using the library's own builders."""
    out = []
    for nm in names:
        neg = nm.startswith("-")
        base = nm[1:] if neg else nm
        kind, n = base[:-1], int(base[-1])
        if kind == "NF":
            t = sop_atom_nf(n)
        elif kind == "SH":
            t = sop_atom_sh(n)
        elif kind == "BOF":
            if bof_draws is None:
                raise ValueError("BOF atoms need N(0,1) draws")
            t = sop_atom_bof(n, bof_draws)
        else:
            raise ValueError(f"unknown atom {nm}")
        out.append(sop_atom_negate(t) if neg else t)
    return out


@dataclass
class Outputs:
    """Device tensors produced by Context.pair_search (None when not requested)."""
    acos_pair: object = None
    acos_atom: object = None
    sel_words: object = None
    scale_code: object = None
    codes: object = None
    code_planes: list = None
    blk_cos: object = None
    blk_err: object = None
    blk_rank: object = None


class Context:
    """sop_ctx with PyTorch tensors for device memory and the current stream."""

    def __init__(self, device: int = 0):
        self._h = C.c_void_p()
        _check(lib().sop_create(C.byref(self._h), device))
        self.device = device
        self.n_atoms = 0
        self.n_entries = []
        self.n_pairs = 0
        self._ws = None

    def close(self):
        if self._h:
            lib().sop_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_alphabet(self, tables):
        tabs = [np.ascontiguousarray(t, dtype=np.float32) for t in tables]
        arr = (_Atom * len(tabs))()
        for i, t in enumerate(tabs):
            arr[i].n_entries = t.size
            arr[i].values = _fp(t)
        _check(lib().sop_set_alphabet(self._h, arr, len(tabs)), self._h)
        self.n_atoms = len(tabs)
        self.n_entries = [t.size for t in tabs]
        self.n_pairs = self.n_atoms * (self.n_atoms - 1) // 2

    def set_pairs(self, pairs):
        if pairs is None or len(pairs) == 0:
            _check(lib().sop_set_pairs(self._h, None, 0), self._h)
            self.n_pairs = self.n_atoms * (self.n_atoms - 1) // 2
            return
        p = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
        _check(lib().sop_set_pairs(self._h, _fp(p, C.c_int), p.shape[0]), self._h)
        self.n_pairs = p.shape[0]

    def workspace_bytes(self, M, K, g) -> int:
        n = C.c_size_t()
        _check(lib().sop_workspace_bytes(self._h, M, K, g, C.byref(n)), self._h)
        return n.value

    def alloc_outputs(self, M, K, g, emit=False, sel=True) -> Outputs:
        """Allocate output tensors for a layer (device memory comes from PyTorch)."""
        import torch
        dev = torch.device("cuda", self.device)
        A, P, Bk = self.n_atoms, self.n_pairs, K // g
        Nb = M * Bk
        o = Outputs()
        o.acos_atom = torch.empty(A, dtype=torch.float64, device=dev)
        o.acos_pair = torch.empty(max(P, 1), dtype=torch.float64, device=dev)
        if sel and P:
            # one selector word per block: 16-bit words up to 16 pairs, 32-bit words beyond
            o.sel_words = torch.empty(Nb, dtype=torch.int16 if P <= 16 else torch.int32, device=dev)
        if emit:
            o.scale_code = torch.empty((A, Nb), dtype=torch.int16, device=dev)
            planes = [M * K // 2 if n <= 16 else M * K for n in self.n_entries]
            o.codes = torch.empty(sum(planes), dtype=torch.uint8, device=dev)
            offs = np.concatenate([[0], np.cumsum(planes)])
            o.code_planes = [o.codes[int(offs[a]):int(offs[a + 1])] for a in range(A)]
            o.blk_cos = torch.empty((A, Nb), dtype=torch.float32, device=dev)
            o.blk_err = torch.empty((A, Nb), dtype=torch.float32, device=dev)
            o.blk_rank = torch.empty((A, Nb), dtype=torch.float32, device=dev)
        return o

    def layer_scope_error(self, W, c, wfmt: WeightFmt, sfmt: ScaleFmt, k: int = 0, want_codes: bool = False, stream=None):
        """sop_layer_scope_error on torch CUDA tensors; returns (out [4] float64 device tensor, codes or None)."""
        import torch
        if not W.is_cuda or (c is not None and not c.is_cuda):
            raise SopError(1, "W and c must be CUDA tensors (no CPU fallback)")
        if W.dim() != 2 or W.stride(1) != 1:
            raise SopError(2, "W must be a 2-D tensor with contiguous rows")
        dt = BF16 if W.dtype == torch.bfloat16 else (F32 if W.dtype == torch.float32 else None)
        if dt is None:
            raise SopError(1, "W must be float32 or bfloat16")
        M, K = W.shape
        out = torch.empty(4, dtype=torch.float64, device=W.device)
        codes = torch.empty((M, K), dtype=torch.int16, device=W.device) if want_codes else None
        st = torch.cuda.current_stream(W.device).cuda_stream if stream is None else stream
        _check(lib().sop_layer_scope_error(self._h, C.c_void_p(W.data_ptr()), dt, M, K, W.stride(0),
                                           None if c is None else C.c_void_p(c.data_ptr()), wfmt, sfmt, k, C.c_void_p(out.data_ptr()),
                                           None if codes is None else C.c_void_p(codes.data_ptr()), C.c_void_p(st)), self._h)
        return out, codes

    def sum_f32(self, x, stream=None):
        """sop_sum_f32 on a contiguous float32 CUDA tensor; returns a [1] float64 device tensor."""
        import torch
        if not x.is_cuda or x.dtype != torch.float32 or not x.is_contiguous():
            raise SopError(1, "x must be a contiguous float32 CUDA tensor")
        out = torch.empty(1, dtype=torch.float64, device=x.device)
        st = torch.cuda.current_stream(x.device).cuda_stream if stream is None else stream
        _check(lib().sop_sum_f32(self._h, C.c_void_p(x.data_ptr()), x.numel(), C.c_void_p(out.data_ptr()), C.c_void_p(st)), self._h)
        return out

    def read_probe(self, x, out=None, stream=None):
        """sop_read_probe on a contiguous CUDA tensor whose size is a multiple of 16 bytes; returns the
        [2048] int32 device tensor of per-workgroup checksums."""
        import torch
        if not x.is_cuda or not x.is_contiguous():
            raise SopError(1, "x must be a contiguous CUDA tensor")
        if out is None:
            out = torch.empty(2048, dtype=torch.int32, device=x.device)
        st = torch.cuda.current_stream(x.device).cuda_stream if stream is None else stream
        _check(lib().sop_read_probe(self._h, C.c_void_p(x.data_ptr()), x.numel() * x.element_size(), C.c_void_p(out.data_ptr()), C.c_void_p(st)), self._h)
        return out

    def issue_probe(self, kind: int, waves_per_simd: int, iters: int, a: float = 0.5, b: float = 0.25, out=None, stream=None):
        """sop_issue_probe: returns the [compute units * waves_per_simd * 256] float32 device tensor of per-lane chain sums."""
        import torch
        dev = torch.device("cuda", self.device)
        n = torch.cuda.get_device_properties(dev).multi_processor_count * int(waves_per_simd) * 256
        if out is None:
            out = torch.empty(n, dtype=torch.float32, device=dev)
        elif out.numel() < n or out.dtype != torch.float32 or not out.is_cuda:
            raise SopError(1, "out must be a CUDA float32 tensor of compute units * waves_per_simd * 256 elements")
        st = torch.cuda.current_stream(dev).cuda_stream if stream is None else stream
        nwg = C.c_int(0)
        _check(lib().sop_issue_probe(self._h, int(kind), int(waves_per_simd), int(iters), float(a), float(b),
                                     C.c_void_p(out.data_ptr()), C.byref(nwg), C.c_void_p(st)), self._h)
        if nwg.value != n:
            raise SopError(6, "the library counts another number of compute units than PyTorch")
        return out

    def pair_search_layers(self, layers, g, fmt: ScaleFmt, metric: int = SEL_WSE, shifts=None, want_sel: bool = False, stream=None):
        """sop_pair_search_layers: layers is a list of (W [M,K], c [K]) CUDA tensors of one dtype.  Returns
        (acos_pair [L,P] float64, acos_atom [L,A] float64, list of selector-word tensors or None);
        asynchronous on the current (or given) stream."""
        import torch
        if not layers:
            raise SopError(1, "no layers")
        dev = layers[0][0].device
        dtypes = {W.dtype for W, _ in layers}
        if dtypes not in ({torch.bfloat16}, {torch.float32}):
            raise SopError(1, "all layers must be bfloat16, or all float32")
        dt = BF16 if torch.bfloat16 in dtypes else F32
        n = len(layers)
        arr = (_Layer * n)()
        sels = [] if want_sel else None
        for i, (W, c) in enumerate(layers):
            if not (W.is_cuda and c.is_cuda) or W.dim() != 2 or W.stride(1) != 1 or c.dtype != torch.float32 or not c.is_contiguous():
                raise SopError(1, f"layer {i}: W must be a 2-D CUDA tensor with contiguous rows, c a contiguous float32 CUDA tensor")
            M, K = W.shape
            arr[i].W, arr[i].M, arr[i].K, arr[i].ldw, arr[i].c = W.data_ptr(), M, K, W.stride(0), c.data_ptr()
            arr[i].k = 0 if shifts is None else int(shifts[i])
            if want_sel:
                sw = torch.empty(M * K // g, dtype=torch.int16 if self.n_pairs <= 16 else torch.int32, device=dev)
                sels.append(sw)
                arr[i].sel_words = sw.data_ptr()
        tp = torch.empty((n, max(self.n_pairs, 1)), dtype=torch.float64, device=dev)
        ta = torch.empty((n, self.n_atoms), dtype=torch.float64, device=dev)
        st = torch.cuda.current_stream(dev).cuda_stream if stream is None else stream
        _check(lib().sop_pair_search_layers(self._h, arr, n, dt, g, fmt, metric,
                                            C.c_void_p(tp.data_ptr()) if self.n_pairs else None, C.c_void_p(ta.data_ptr()),
                                            C.c_void_p(st)), self._h)
        return tp[:, :self.n_pairs], ta, sels

    def search_layer(self, W, c, g, fmt: ScaleFmt, atoms, p_grid=(), k: int = 0, metric: int = SEL_WSE, fit_entries: int = 16,
                     fit_iters: int = 20, fit_bins: int = 1024, fit_init=None, weighted_fit: bool = True, fit_grid=None,
                     pack: bool = False, stream=None):
        """sop_search_layer on torch CUDA tensors.  Returns (result structure, words or None, payload or None); the
        workspace is a torch tensor kept by the context and grown on demand."""
        import torch
        dt = BF16 if W.dtype == torch.bfloat16 else (F32 if W.dtype == torch.float32 else None)
        if dt is None or not (W.is_cuda and c.is_cuda) or W.dim() != 2 or W.stride(1) != 1:
            raise SopError(1, "W must be a 2-D float32 or bfloat16 CUDA tensor with contiguous rows, c a CUDA tensor")
        M, K = W.shape
        tabs = [np.ascontiguousarray(t, dtype=np.float32) for t in atoms]
        arr = (_Atom * len(tabs))()
        for i, t in enumerate(tabs):
            arr[i].n_entries = t.size
            arr[i].values = _fp(t)
        o = _LayerOpts()
        o.n_p = len(p_grid)
        for i, p in enumerate(list(p_grid)[:LAYER_MAX_P]):
            o.p_percent[i] = float(p)
        o.fit_entries, o.fit_iters, o.fit_bins, o.weighted_fit, o.pack = fit_entries, fit_iters, fit_bins, int(bool(weighted_fit)), int(bool(pack))
        keep = []
        if fit_init is not None:
            ini = np.ascontiguousarray(fit_init, dtype=np.float32); keep.append(ini)
            o.fit_init = _fp(ini)
        if fit_grid is not None:
            gr = np.ascontiguousarray(fit_grid, dtype=np.float64); keep.append(gr)
            o.fit_grid = _fp(gr, C.c_double); o.n_fit_grid = gr.size
        need = C.c_size_t()
        _check(lib().sop_search_layer_workspace(self._h, M, K, g, len(tabs), C.byref(o), C.byref(need)), self._h)
        if self._ws is None or self._ws.numel() < need.value:
            self._ws = torch.empty(need.value, dtype=torch.uint8, device=W.device)
        words = payload = None
        if pack:
            n = 1
            while (1 << n) < max(max(t.size for t in tabs), fit_entries if len(p_grid) else 0):
                n += 1                                          # room for the widest codebook that can win
            words = torch.empty(M * K // g, dtype=torch.int16, device=W.device)
            payload = torch.empty((M * K // g, g * n // 8), dtype=torch.uint8, device=W.device)
        res = _LayerResult()
        st = torch.cuda.current_stream(W.device).cuda_stream if stream is None else stream
        _check(lib().sop_search_layer(self._h, C.c_void_p(W.data_ptr()), dt, M, K, W.stride(0), C.c_void_p(c.data_ptr()), g, fmt, k, metric,
                                      arr, len(tabs), C.byref(o), C.c_void_p(self._ws.data_ptr()), self._ws.numel(), C.byref(res),
                                      None if words is None else C.c_void_p(words.data_ptr()),
                                      None if payload is None else C.c_void_p(payload.data_ptr()), C.c_void_p(st)), self._h)
        self.n_atoms = 0
        if pack and payload.shape[1] != g * res.n_bits // 8:
            payload = payload.reshape(-1)[:M * K // g * (g * res.n_bits // 8)].reshape(M * K // g, g * res.n_bits // 8)
        return res, words, payload

    def prepare_scale(self, fmt: ScaleFmt, k: int = 0, stream=None):
        """sop_prepare_scale: write the scale table of (fmt, k) ahead of the searches that use it."""
        import torch
        st = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _check(lib().sop_prepare_scale(self._h, fmt, k, C.c_void_p(st)), self._h)

    def set_scale_rule(self, rule: int):
        """SCALE_ABSMAX (default) or SCALE_ARGMAX for later pair_search calls."""
        _check(lib().sop_set_scale_rule(self._h, rule), self._h)

    def partition(self, score, n_top: int, higher_is_better: bool = True, stream=None):
        """sop_partition on a contiguous float32 CUDA tensor of per-block scores; returns device
        tensors (pool_b [N_b] uint8, tau [1] float32, n_a [1] int64)."""
        import torch
        if not score.is_cuda or score.dtype != torch.float32 or not score.is_contiguous():
            raise SopError(1, "score must be a contiguous float32 CUDA tensor")
        n = score.numel()
        pool_b = torch.empty(n, dtype=torch.uint8, device=score.device)
        tau = torch.empty(1, dtype=torch.float32, device=score.device)
        n_a = torch.empty(1, dtype=torch.int64, device=score.device)
        st = torch.cuda.current_stream(score.device).cuda_stream if stream is None else stream
        _check(lib().sop_partition(self._h, C.c_void_p(score.data_ptr()), n, n_top, 1 if higher_is_better else 0,
                                   C.c_void_p(pool_b.data_ptr()), C.c_void_p(tau.data_ptr()), C.c_void_p(n_a.data_ptr()),
                                   C.c_void_p(st)), self._h)
        return pool_b, tau, n_a

    def partition_levels(self, score, n_tops, higher_is_better: bool = True, stream=None):
        """sop_partition_levels on a contiguous float32 CUDA tensor of per-block scores; returns device tensors
        (level [N_b] uint8, tau [L] float32, n_a [L] int64)."""
        import torch
        if not score.is_cuda or score.dtype != torch.float32 or not score.is_contiguous():
            raise SopError(1, "score must be a contiguous float32 CUDA tensor")
        n, L = score.numel(), len(n_tops)
        level = torch.empty(n, dtype=torch.uint8, device=score.device)
        tau = torch.empty(L, dtype=torch.float32, device=score.device)
        n_a = torch.empty(L, dtype=torch.int64, device=score.device)
        tops = (C.c_int64 * L)(*[int(t) for t in n_tops])
        st = torch.cuda.current_stream(score.device).cuda_stream if stream is None else stream
        _check(lib().sop_partition_levels(self._h, C.c_void_p(score.data_ptr()), n, tops, L, 1 if higher_is_better else 0,
                                          C.c_void_p(level.data_ptr()), C.c_void_p(tau.data_ptr()), C.c_void_p(n_a.data_ptr()),
                                          C.c_void_p(st)), self._h)
        return level, tau, n_a

    def dd_histogram_levels(self, W, c, g, level, n_levels: int, n_bins: int = 1024, row_step: int = 1, stream=None):
        """sop_dd_histogram_levels on torch CUDA tensors; returns an [n_levels, n_bins] int64 device tensor."""
        import torch
        dt = BF16 if W.dtype == torch.bfloat16 else (F32 if W.dtype == torch.float32 else None)
        if dt is None or not W.is_cuda or W.dim() != 2 or W.stride(1) != 1:
            raise SopError(1, "W must be a 2-D float32 or bfloat16 CUDA tensor with contiguous rows")
        M, K = W.shape
        hist = torch.empty((n_levels, n_bins), dtype=torch.int64, device=W.device)
        st = torch.cuda.current_stream(W.device).cuda_stream if stream is None else stream
        _check(lib().sop_dd_histogram_levels(self._h, C.c_void_p(W.data_ptr()), dt, M, K, W.stride(0),
                                             None if c is None else C.c_void_p(c.data_ptr()), g, n_bins, row_step,
                                             C.c_void_p(level.data_ptr()), n_levels, C.c_void_p(hist.data_ptr()), C.c_void_p(st)), self._h)
        return hist

    def pack_blocks(self, out, M, K, g, fmt: ScaleFmt, a: int, b=None, pair_q: int = 0, stream=None):
        """sop_pack_blocks on the outputs of an emitting pair_search: atom a alone (b None) or the
        pair (a, b) with selector bit pair_q.  Returns (words [N_b] int16, payload [N_b, g*n/8] uint8, n)."""
        import torch
        if out.scale_code is None or out.code_planes is None:
            raise SopError(1, "pack_blocks needs the scale codes and code planes of an emitting search")
        two = b is not None
        if two and out.sel_words is None:
            raise SopError(1, "pack_blocks of a pair needs the selector words")
        ents = self.n_entries
        n = 1
        while (1 << n) < (max(ents[a], ents[b]) if two else ents[a]):
            n += 1
        Nb = M * K // g
        dev = out.scale_code.device
        words = torch.empty(Nb, dtype=torch.int16, device=dev)
        payload = torch.empty((Nb, g * n // 8), dtype=torch.uint8, device=dev)
        nb = C.c_int(0)
        st = torch.cuda.current_stream(dev).cuda_stream if stream is None else stream
        ptr = lambda t: C.c_void_p(t.data_ptr())
        _check(lib().sop_pack_blocks(self._h, M, K, g, fmt, ptr(out.scale_code[a]), ptr(out.code_planes[a]), ents[a],
                                     ptr(out.scale_code[b]) if two else None, ptr(out.code_planes[b]) if two else None, ents[b] if two else 0,
                                     ptr(out.sel_words) if two else None, out.sel_words.element_size() if two else 0, pair_q,
                                     ptr(words), ptr(payload), C.byref(nb), C.c_void_p(st)), self._h)
        assert nb.value == n
        return words, payload, n

    def scale_histogram(self, W, g, t_pos: float, t_neg: float, fmt: ScaleFmt, stream=None):
        """sop_scale_histogram on a torch CUDA tensor; returns a [2, 320] int64 device tensor."""
        import torch
        if not W.is_cuda:
            raise SopError(1, "W must be a CUDA tensor (no CPU fallback)")
        if W.dim() != 2 or W.stride(1) != 1:
            raise SopError(2, "W must be a 2-D tensor with contiguous rows")
        dt = BF16 if W.dtype == torch.bfloat16 else (F32 if W.dtype == torch.float32 else None)
        if dt is None:
            raise SopError(1, "W must be float32 or bfloat16")
        M, K = W.shape
        hist = torch.empty((2, 320), dtype=torch.int64, device=W.device)
        st = torch.cuda.current_stream(W.device).cuda_stream if stream is None else stream
        _check(lib().sop_scale_histogram(self._h, C.c_void_p(W.data_ptr()), dt, M, K, W.stride(0), g, t_pos, t_neg, fmt,
                                         C.c_void_p(hist.data_ptr()), C.c_void_p(st)), self._h)
        return hist

    def dd_histogram(self, W, c, g, n_bins: int = 1024, row_step: int = 1, block_mask=None, stream=None):
        """sop_dd_histogram on torch CUDA tensors; returns an [n_bins] int64 device tensor."""
        import torch
        if not W.is_cuda or (c is not None and not c.is_cuda):
            raise SopError(1, "W and c must be CUDA tensors (no CPU fallback)")
        if W.dim() != 2 or W.stride(1) != 1:
            raise SopError(2, "W must be a 2-D tensor with contiguous rows")
        dt = BF16 if W.dtype == torch.bfloat16 else (F32 if W.dtype == torch.float32 else None)
        if dt is None:
            raise SopError(1, "W must be float32 or bfloat16")
        M, K = W.shape
        hist = torch.empty(n_bins, dtype=torch.int64, device=W.device)
        st = torch.cuda.current_stream(W.device).cuda_stream if stream is None else stream
        _check(lib().sop_dd_histogram(self._h, C.c_void_p(W.data_ptr()), dt, M, K, W.stride(0),
                                      None if c is None else C.c_void_p(c.data_ptr()), g, n_bins, row_step, None if block_mask is None else C.c_void_p(block_mask.data_ptr()),
                                      C.c_void_p(hist.data_ptr()), C.c_void_p(st)), self._h)
        return hist

    def pair_search(self, W, c, g, fmt: ScaleFmt, k: int = 0, metric: int = SEL_WSE, out: Outputs = None,
                    emit: bool = False, stream=None, static: bool = False) -> Outputs:
        """sop_pair_search on torch CUDA tensors: W [M,K] float32 or bfloat16 (row stride = W.stride(0)),
        c [K] float32.  Asynchronous on the current (or given) stream.  static=True calls
        sop_pair_search_static (the caller then passes `out`, so that nothing is allocated)."""
        import torch
        if not (W.is_cuda and c.is_cuda):
            raise SopError(1, "W and c must be CUDA tensors (no CPU fallback)")
        if W.dim() != 2 or W.stride(1) != 1:
            raise SopError(2, "W must be a 2-D tensor with contiguous rows")
        if W.dtype == torch.bfloat16:
            dt = BF16
        elif W.dtype == torch.float32:
            dt = F32
        else:
            raise SopError(1, "W must be float32 or bfloat16")
        if c.dtype != torch.float32 or not c.is_contiguous():
            raise SopError(1, "c must be a contiguous float32 tensor")
        M, K = W.shape
        if out is None:
            out = self.alloc_outputs(M, K, g, emit=emit)
        st = torch.cuda.current_stream(W.device).cuda_stream if stream is None else stream

        def ptr(t):
            return None if t is None else C.c_void_p(t.data_ptr())

        o = _Outputs(ptr(out.acos_pair), ptr(out.acos_atom), ptr(out.sel_words), ptr(out.scale_code), ptr(out.codes),
                     ptr(out.blk_cos), ptr(out.blk_err), ptr(out.blk_rank))
        if static:
            _check(lib().sop_pair_search_static(self._h, C.c_void_p(W.data_ptr()), dt, M, K, W.stride(0), C.c_void_p(c.data_ptr()), g,
                                                fmt, k, metric, C.byref(o), C.c_void_p(st)), self._h)
            return out
        _check(lib().sop_pair_search(self._h, C.c_void_p(W.data_ptr()), dt, M, K, W.stride(0), C.c_void_p(c.data_ptr()), g,
                                     fmt, k, metric, None, 0, C.byref(o),
                                     C.c_void_p(st)), self._h)
        return out
