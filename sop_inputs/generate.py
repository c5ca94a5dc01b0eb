"""Seeded generators.  All draws use numpy's PCG64 so a (seed, shape) pair fixes the tensor."""
from __future__ import annotations

import numpy as np


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 container (uint16), round-to-nearest-even on the dropped 16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 container (uint16) -> fp32, exact widening."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the bf16 grid, returned as fp32."""
    return bf16_bits_to_f32(bf16_bits(x))


def student_t_weights(M: int, K: int, nu: float, seed: int, *, row_sigma: float | None = None,
                      row_seed: int | None = None, outlier_frac: float = 0.0,
                      outlier_mult: float = 20.0, outlier_seed: int | None = None,
                      scale: float = 1.0, chunk_rows: int = 1024) -> np.ndarray:
    """W[M,K] fp32: Student-t(nu) entries, optional per-row log-normal factor exp(row_sigma*z),
    optional Bernoulli(outlier_frac) mask of entries multiplied by outlier_mult."""
    g = _rng(seed)
    W = np.empty((M, K), dtype=np.float32)
    for r0 in range(0, M, chunk_rows):                      # chunked to bound the fp64 temporaries
        r1 = min(M, r0 + chunk_rows)
        W[r0:r1] = g.standard_t(nu, size=(r1 - r0, K)).astype(np.float32)
    if outlier_frac > 0.0:
        go = _rng(outlier_seed if outlier_seed is not None else seed + 7)
        for r0 in range(0, M, chunk_rows):
            r1 = min(M, r0 + chunk_rows)
            mask = go.random(size=(r1 - r0, K)) < outlier_frac
            W[r0:r1][mask] *= np.float32(outlier_mult)
    if row_sigma is not None:
        gr = _rng(row_seed if row_seed is not None else seed + 1)
        W *= np.exp(row_sigma * gr.standard_normal(M)).astype(np.float32)[:, None]
    if scale != 1.0:
        W *= np.float32(scale)
    return W


def channel_norms(K: int, sigma: float, seed: int) -> np.ndarray:
    """c[K] fp32, log-normal: exp(sigma * z)."""
    return np.exp(sigma * _rng(seed).standard_normal(K)).astype(np.float32)


def normal_draws(n: int, seed: int) -> np.ndarray:
    """n raw N(0,1) draws (fp64).  Fitted-codebook builders on both sides consume these."""
    return _rng(seed).standard_normal(n)


# Scale formats as (sign_bits, exp_bits, man_bits, container_bits, bias, max_code); -1 = default.
UE4M4 = (0, 4, 4, 8, -1, -1)
E4M3 = (1, 4, 3, 8, -1, -1)
UE4M6 = (0, 4, 6, 10, -1, -1)
E4M5 = (1, 4, 5, 10, -1, -1)
UE5M7 = (0, 5, 7, 12, -1, -1)
E5M6 = (1, 5, 6, 12, -1, -1)
E4M7 = (1, 4, 7, 12, -1, -1)
S1E5M5 = (1, 5, 5, 12, -1, -1)
# bf16-like 16-bit signed scale.  Bias and top code are chosen so that every scale value and its
# reciprocal stay inside fp32's normal range (values 2^-125 .. just under 2^126).
E8M7 = (1, 8, 7, 16, 119, 244 * 128 + 127)

SCALE_FORMATS = {
    "UE4M4": UE4M4, "E4M3": E4M3, "UE4M6": UE4M6, "E4M5": E4M5, "UE5M7": UE5M7,
    "E5M6": E5M6, "E4M7": E4M7, "S1E5M5": S1E5M5, "E8M7": E8M7,
}

# The five benchmark configurations: tensor recipes only (method parameters are listed beside
# them so tests and the bench agree on what each configuration means).
CONFIGS = {
    "C1": dict(M=256, K=1024, dtype="f32", nu=5.0, row_sigma=0.5, c_sigma=1.0, outlier_frac=0.0,
               seeds=(1001, 1002, 1003, 1004), g=16, fmt="UE4M4",
               atoms=("NF4", "SH4", "-NF4", "-SH4")),
    "C2": dict(M=4096, K=4096, dtype="bf16", nu=4.0, row_sigma=0.5, c_sigma=1.0, outlier_frac=1e-3,
               seeds=(2001, 2002, 2003, 2004), g=16, fmt="E4M3",
               atoms=("NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4")),
    "C3_up": dict(M=11008, K=4096, dtype="bf16", nu=4.0, row_sigma=None, c_sigma=1.0, outlier_frac=0.0,
                  seeds=(3001, 3002, 3003, 3004), g=16, fmt="UE4M4",
                  atoms=("NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4")),
    "C3_down": dict(M=4096, K=11008, dtype="bf16", nu=4.0, row_sigma=None, c_sigma=1.0, outlier_frac=0.0,
                    seeds=(3011, 3012, 3013, 3014), g=16, fmt="UE4M4",
                    atoms=("NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4")),
    "C5": dict(M=28672, K=8192, dtype="bf16", nu=4.0, row_sigma=None, c_sigma=1.0, outlier_frac=0.0,
               seeds=(5001, 5002, 5003, 5004), g=16, fmt="UE4M4",
               atoms=("NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4")),
}


def make_config(name: str, rows: int | None = None):
    """Return (W fp32 [M,K] already on the bf16 grid when dtype is bf16, c fp32 [K], cfg dict).
    `rows` truncates M (the first rows of the same stream, so a slice equals the full tensor's head
    only when chunk boundaries agree; callers that need a head slice generate once and slice)."""
    cfg = dict(CONFIGS[name])
    M = cfg["M"] if rows is None else int(rows)
    sw, sr, sc, so = cfg["seeds"]
    W = student_t_weights(M, cfg["K"], cfg["nu"], sw, row_sigma=cfg["row_sigma"], row_seed=sr,
                          outlier_frac=cfg["outlier_frac"], outlier_seed=so)
    if cfg["dtype"] == "bf16":
        W = bf16_round(W)
    c = channel_norms(cfg["K"], cfg["c_sigma"], sc)
    cfg["M"] = M
    return W, c, cfg


def layer_shapes_7b():
    """The 7 linear layers of one 7B-shaped transformer block: (name, M, K)."""
    return [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
            ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]


def model_7b_layers(n_blocks: int, seed: int = 4001, rows: int | None = None):
    """Configuration 4: the linear layers of a 7B-shaped model, block by block.  Yields
    (name, W fp32 on the bf16 grid [M,K], c fp32 [K], nu): Student-t weights whose tail index nu is
    drawn per layer from U(3, 8), one log-normal (sigma 1) channel-norm vector per layer.  `rows`
    truncates every layer to its first rows (tests)."""
    r = _rng(seed)
    for b in range(n_blocks):
        for i, (name, M, K) in enumerate(layer_shapes_7b()):
            nu = float(r.uniform(3.0, 8.0))
            s = seed + 1000 * (b + 1) + 10 * i
            Mr = M if rows is None else min(M, int(rows))
            W = bf16_round(student_t_weights(Mr, K, nu, s))
            c = channel_norms(K, 1.0, s + 1)
            yield f"block{b}.{name}", W, c, nu


def model_7b_layer(block: int, index: int, seed: int = 4001, rows: int | None = None):
    """Layer `index` (0..6 in the order of layer_shapes_7b) of block `block` of configuration 4, as
    model_7b_layers() yields it, without drawing the layers before it."""
    r = _rng(seed)
    nu = 0.0
    for _ in range(7 * block + index + 1):                 # the tail indices are drawn in layer order
        nu = float(r.uniform(3.0, 8.0))
    name, M, K = layer_shapes_7b()[index]
    s = seed + 1000 * (block + 1) + 10 * index
    Mr = M if rows is None else min(M, int(rows))
    return f"block{block}.{name}", bf16_round(student_t_weights(Mr, K, nu, s)), channel_norms(K, 1.0, s + 1), nu
