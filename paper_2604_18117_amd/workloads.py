"""Seeded synthetic inputs and layer shapes.

This module holds no arithmetic of the method itself: it only names the layer shapes and
draws the random source tensors (X, W, L, R) that both the GPU library and the CPU oracle
are fed with.  The shapes imitate the linear layers of the two diffusion transformers the
paper evaluates (a 1152-wide and a 2240-wide DiT, Section 4.1); the value distributions are
Gaussian weights, Gaussian activations with a few strong outlier channels (the situation
activation smoothing addresses, Section 3.4) and a heavy-tailed Laplace input for the second
MLP projection.  Nothing here comes from the paper's models or datasets.

Draw order for one layer, from ``numpy.random.default_rng(seed)``:
X, outlier column set, W, L, R.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Layer:
    name: str
    M: int
    K: int
    N: int
    r: int
    family: str            # "int" (INT4 main, integer branch) | "mx" (MXFP4 main, FP8 branch) | "mxb" (MXFP8e4 branch)
                           # | "mxi" (MXINT4 main, MXINT8 branch activations, MXINT8 / MXINT4 branch weights)
    g: int                 # main weight group along K (INT: 64|128; MX: 32)
    br_w_bits: int         # branch weight width (INT: 8|6|4; MX: 8)
    br_a_bits: int         # branch activation width (INT: 8|6; MX: 8)
    x_dtype: str           # "f32" | "bf16"
    x_dist: str = "normal"  # "normal" | "laplace"
    outlier_scale: float = 1.0
    n_outliers: int = 0
    w_std: float = 0.02
    lr_std: float = 1e-3
    seed: int = 0
    a_group: int = 0       # INT family: 0 = one main activation scale per token; 64 = SINT4 blocks for both main operands


def _n_out(K: int) -> int:
    return int(round(0.01 * K))


def _int_layer(name, M, K, N, r, g, bw, ba, **kw) -> Layer:
    return Layer(name, M, K, N, r, "int", g, bw, ba, kw.pop("x_dtype", "bf16"), **kw)


# Configuration 1: the small single layer the oracle finishes in well under a second.
CFG1 = [_int_layer("c1_single", 256, 1152, 1152, 16, 64, 8, 8, x_dtype="f32",
                   outlier_scale=20.0, n_outliers=12)]
# Configuration 2: 1152-wide DiT, fused QKV projection on 2 x 4096 tokens.
CFG2 = [_int_layer("c2_qkv", 8192, 1152, 3456, 32, 64, 8, 8, outlier_scale=15.0,
                   n_outliers=_n_out(1152))]
# Configuration 3: the MLP pair of the same model; W4A8 branch, main group 128.
CFG3 = [_int_layer("c3_fc1", 8192, 1152, 4608, 32, 128, 4, 8, outlier_scale=15.0,
                   n_outliers=_n_out(1152)),
        _int_layer("c3_fc2", 8192, 4608, 1152, 32, 128, 4, 8, x_dist="laplace")]
# Configuration 4: 2240-wide DiT; QKV and the pointwise expansion; W6A6 branch.
CFG4 = [_int_layer("c4_qkv", 8192, 2240, 6720, 64, 64, 6, 6, outlier_scale=25.0,
                   n_outliers=_n_out(2240), w_std=0.015),
        _int_layer("c4_expand", 8192, 2240, 11200, 64, 64, 6, 6, outlier_scale=25.0,
                   n_outliers=_n_out(2240), w_std=0.015)]


def _mx_layer(name, K, N) -> Layer:
    return Layer(name, 16384, K, N, 32, "mx", 32, 8, 8, "bf16")


# Configuration 5: the seven linears of one 1152-wide DiT block, MX formats.
CFG5 = [_mx_layer("c5_qkv", 1152, 3456), _mx_layer("c5_attn_out", 1152, 1152),
        _mx_layer("c5_cross_q", 1152, 1152), _mx_layer("c5_cross_kv", 1152, 2304),
        _mx_layer("c5_cross_out", 1152, 1152), _mx_layer("c5_fc1", 1152, 4608),
        _mx_layer("c5_fc2", 4608, 1152)]

# The same seven layers with an MXFP8e4 (block-scaled E4M3) branch: the all-MX mixed-precision setting.
CFG5B = [replace(l, name="c5b" + l.name[2:], family="mxb") for l in CFG5]
# ... and with an MXFP6e2 (block-scaled E2M3) branch of rank 64: W6A6 in the branch.
CFG5B6 = [replace(l, name="c5b6" + l.name[2:], family="mxb", r=64, br_w_bits=6, br_a_bits=6) for l in CFG5]

# The same seven layers in the integer MX formats: MXINT4 main, MXINT8 branch of rank 64 (the pairing of
# the paper's mixed-precision table for integer formats), and MXINT4 branch weights of rank 128.
CFG5I = [replace(l, name="c5i" + l.name[2:], family="mxi", r=64) for l in CFG5]
CFG5I4 = [replace(l, name="c5i4" + l.name[2:], family="mxi", r=128, br_w_bits=4) for l in CFG5]

# Configuration 2 and the 2240-wide QKV layer with the literal SINT4 blocks (FP16 scale per 64 values along K) for the
# activations as well as the weights.
CFG2S = [replace(CFG2[0], name="c2s_qkv", a_group=64)]
CFG4S = [replace(CFG4[0], name="c4s_qkv", a_group=64)]

# The 2240-wide QKV projection in the all-MX setting (2240 = 35 x 64: one padding chunk inside the blobs).
CFG4M = [Layer("c4m_qkv", 8192, 2240, 6720, 64, "mxb", 32, 8, 8, "bf16", outlier_scale=25.0, n_outliers=_n_out(2240),
               w_std=0.015)]

CONFIGS: Dict[str, List[Layer]] = {"c1": CFG1, "c2": CFG2, "c3": CFG3, "c4": CFG4, "c5": CFG5, "c5b": CFG5B, "c5b6": CFG5B6,
                                   "c5i": CFG5I, "c5i4": CFG5I4, "c2s": CFG2S, "c4s": CFG4S, "c4m": CFG4M}
LAYERS: Dict[str, Layer] = {l.name: l for ls in CONFIGS.values() for l in ls}


def shrink(layer: Layer, M: Optional[int] = None, K: Optional[int] = None,
           N: Optional[int] = None, r: Optional[int] = None) -> Layer:
    """Same recipe at a smaller shape (for parity tests the oracle finishes in seconds)."""
    kw = {}
    if M is not None:
        kw["M"] = M
    if K is not None:
        kw["K"] = K
        if layer.n_outliers:
            kw["n_outliers"] = max(1, _n_out(K))
    if N is not None:
        kw["N"] = N
    if r is not None:
        kw["r"] = r
    return replace(layer, **kw)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already bf16-representable."""
    return (np.ascontiguousarray(a, np.float32).view(np.uint32) >> 16).astype(np.uint16)


def make_inputs(layer: Layer) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """(X, W, L, R) as fp32 arrays; X holds bf16-representable values when x_dtype is bf16."""
    rng = np.random.default_rng(layer.seed)
    M, K, N, r = layer.M, layer.K, layer.N, layer.r
    if layer.x_dist == "normal":
        X = rng.standard_normal((M, K), dtype=np.float32)
    elif layer.x_dist == "laplace":
        X = rng.laplace(0.0, 0.5, size=(M, K)).astype(np.float32)
    else:
        raise ValueError(layer.x_dist)
    cols = rng.choice(K, size=layer.n_outliers, replace=False) if layer.n_outliers else np.empty(0, np.int64)
    if cols.size:
        X[:, cols] *= np.float32(layer.outlier_scale)
    W = (rng.standard_normal((N, K), dtype=np.float32) * np.float32(layer.w_std))
    L = (rng.standard_normal((N, r), dtype=np.float32) * np.float32(layer.lr_std))
    R = (rng.standard_normal((r, K), dtype=np.float32) * np.float32(layer.lr_std))
    if layer.x_dtype == "bf16":
        X = round_to_bf16(X)
    return X, W, L, R


def to_dev_x(X: np.ndarray, x_dtype: str):
    """X as a device tensor of the layer's input type (marshalling only; torch is imported on use)."""
    import torch
    if x_dtype == "bf16":
        bits = f32_to_bf16_bits(X).view(np.int16)
        return torch.from_numpy(bits.copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(X, np.float32)).cuda()


def bf16_to_bits(t) -> np.ndarray:
    """uint16 bit patterns of a bf16 device tensor, on the host."""
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
