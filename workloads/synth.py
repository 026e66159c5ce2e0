"""Seeded synthetic inputs for the EfQAT backward hot path.

This module holds NO arithmetic of the method (no quantizer, no importance, no
gradient): only a counter-based random generator, dtype casts and the table of
layer shapes.  Both the CPU oracle's tests and the HIP path's tests/bench feed
from it, so the two sides see identical bits.

The shapes stand in for the paper's workloads (Section 4: ResNet-50 / ImageNet,
BERT-base / SQuAD v1.1): only layer shapes are used; values are i.i.d. normal
with the initialisation scales a trained network of that family has.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(z: np.ndarray) -> np.ndarray:
    """One round of the SplitMix64 output function on a uint64 array."""
    with np.errstate(over="ignore"):
        z = (z + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        return z ^ (z >> np.uint64(31))


def uniform01(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n doubles in (0,1): value i depends only on (seed, stream, offset+i)."""
    ctr = np.arange(offset, offset + n, dtype=np.uint64)
    with np.errstate(over="ignore"):
        key = _splitmix64(np.array([seed], dtype=np.uint64) * np.uint64(0x632BE59BD9B4E019)
                          + np.uint64(stream) * np.uint64(0xD1342543DE82EF95))
        bits = _splitmix64(ctr ^ key)
    # 53 random bits, shifted by half an ulp so 0 and 1 are excluded
    return ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _normal_chunk(seed: int, stream: int, lo: int, m: int) -> np.ndarray:
    u1 = uniform01(seed, 2 * stream, m, lo)
    u2 = uniform01(seed, 2 * stream + 1, m, lo)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def normal(seed: int, stream: int, shape, std: float = 1.0, mean: float = 0.0) -> np.ndarray:
    """fp64 N(mean, std^2) samples by Box-Muller on the counter-based uniforms.  Sample i depends only on
    (seed, stream, i), so large arrays are filled chunk by chunk on a few host threads with identical results."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float64)
    chunk = 1 << 22
    los = list(range(0, n, chunk))

    def fill(lo):
        m = min(chunk, n - lo)
        out[lo:lo + m] = _normal_chunk(seed, stream, lo, m)

    workers = min(len(los), 16, len(os.sched_getaffinity(0)))
    if workers > 1:
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(fill, los))
    else:
        for lo in los:
            fill(lo)
    return (out * std + mean).reshape(shape)


# ---------------------------------------------------------------- dtype casts
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp64/fp32 values to bfloat16 (nearest even); returns uint16 bit patterns."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    rnd = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns exactly to fp32."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_bf16_values(x: np.ndarray) -> np.ndarray:
    """fp32 array holding x rounded to bfloat16 precision."""
    return bf16_bits_to_f32(to_bf16_bits(x)).reshape(np.shape(x))


# ------------------------------------------------------------- layer factories
def linear_layer(seed: int, T: int, c_in: int, c_out: int, act_dtype: str = "bf16",
                 w_std: float = 0.02, x_abs: bool = False, row_scale_sigma: float = 0.0):
    """One synthetic linear layer: X [T,c_in], W [c_out,c_in], dY [T,c_out].

    act_dtype "bf16": X and dY are fp32 arrays whose values are bf16-representable;
    "f32": plain fp32.  W is always fp32 (master weights).  row_scale_sigma > 0
    multiplies each weight row by a log-normal factor (outlier channels, as the
    paper's channel-importance figure describes for trained networks).
    """
    X = normal(seed, 0, (T, c_in))
    if x_abs:
        X = np.abs(X)
    W = normal(seed, 1, (c_out, c_in), std=w_std)
    if row_scale_sigma > 0.0:
        W = W * np.exp(row_scale_sigma * normal(seed, 3, (c_out, 1)))
    dY = normal(seed, 2, (T, c_out))
    if act_dtype == "bf16":
        X, dY = as_bf16_values(X), as_bf16_values(dY)
    else:
        X, dY = X.astype(np.float32), dY.astype(np.float32)
    return X, W.astype(np.float32), dY


def conv_layer(seed: int, N: int, H: int, W_: int, c_in: int, c_out: int, kh: int, kw: int,
               stride: int = 1, pad: int = 0, act_dtype: str = "bf16", w_std: float = 0.02,
               x_abs: bool = True):
    """One synthetic conv layer: X NHWC, W OHWI (fp32), dY N,Ho,Wo,c_out."""
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W_ + 2 * pad - kw) // stride + 1
    X = normal(seed, 0, (N, H, W_, c_in))
    if x_abs:
        X = np.abs(X)
    Wt = normal(seed, 1, (c_out, kh, kw, c_in), std=w_std)
    dY = normal(seed, 2, (N, Ho, Wo, c_out))
    if act_dtype == "bf16":
        X, dY = as_bf16_values(X), as_bf16_values(dY)
    else:
        X, dY = X.astype(np.float32), dY.astype(np.float32)
    return X, Wt.astype(np.float32), dY


# ------------------------------------------------------------------ workloads
# (name, T, c_in, c_out) per layer; fractions as (num, den)
CFG1 = dict(name="cfg1_linear256", seed=0, layers=[("lin", 256, 256, 256)], act_dtype="f32",
            w_bits=8, a_bits=8, fractions=[(1, 4)])
CFG2 = dict(name="cfg2_bert_ffn", seed=2000,
            layers=[("ffn1", 12288, 768, 3072), ("ffn2", 12288, 3072, 768)], act_dtype="bf16",
            w_bits=8, a_bits=8, fractions=[(0, 1), (1, 20), (1, 4), (1, 1)])
CFG3 = dict(name="cfg3_bert_stack", seed=3000,
            layers=[("qkv", 12288, 768, 2304), ("out", 12288, 768, 768),
                    ("ffn1", 12288, 768, 3072), ("ffn2", 12288, 3072, 768)], n_repeat=12,
            act_dtype="bf16", w_bits=(4, 8), a_bits=8, fractions=[(1, 20), (1, 4), (1, 1)])
CFG4 = dict(name="cfg4_resnet_conv", seed=4000,
            conv=dict(N=64, H=14, W=14, c_in=256, c_out=256, kh=3, kw=3, stride=1, pad=1),
            conv1x1=dict(N=64, H=14, W=14, c_in=256, c_out=1024, kh=1, kw=1, stride=1, pad=0),
            act_dtype="bf16", w_bits=4, a_bits=8, fractions=[(1, 20), (1, 4), (1, 1)])
CFG5 = dict(name="cfg5_llm_mlp", seed=5000,
            layers=[("up", 8192, 4096, 11008), ("down", 8192, 11008, 4096)], act_dtype="bf16",
            w_bits=4, a_bits=8,
            fractions=[(1, 100), (1, 50), (1, 20), (1, 10), (1, 4), (1, 2), (1, 1)])
