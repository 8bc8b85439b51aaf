"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds no arithmetic of the method itself: it only draws random
tensors with the shapes and value distributions of LLaMA-shaped fine-tuning
layers, converts fp32 to bf16 bit patterns, and builds the 16-entry 4-bit
codebook that is handed to both implementations as data.  It depends on
numpy/scipy only, so both the CPU checker and the GPU binding can use it
without importing each other.

Value recipe (stand-in for real LLaMA weights / activations, which are not
available offline): W ~ N(0, 0.02^2) in fp32 with 0.1 % of the entries
(chosen uniformly) multiplied by 20; X, dY ~ N(0, 1) rounded to bf16;
A ~ U(-b, b) with b = 1/sqrt(D_in/lambda) rounded to bf16; B ~ N(0, 0.01^2)
rounded to bf16.  Every tensor is a pure function of (seed, stream index).
"""
from __future__ import annotations

import dataclasses
import numpy as np


# ----------------------------------------------------------------------------
# bf16 <-> fp32 bit conversions (format plumbing, round-to-nearest-even)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array of bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> exact fp32 values."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# counter-based random streams
# ----------------------------------------------------------------------------
def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed) & (2**64 - 1), int(stream)]))


def normal_f32(seed: int, stream: int, shape, std: float = 1.0) -> np.ndarray:
    return (_rng(seed, stream).standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def uniform_f32(seed: int, stream: int, shape, bound: float) -> np.ndarray:
    u = _rng(seed, stream).random(shape, dtype=np.float32)
    return ((u * np.float32(2.0) - np.float32(1.0)) * np.float32(bound)).astype(np.float32)


def base_weight(seed: int, stream: int, d_out: int, d_in: int,
                std: float = 0.02, outlier_frac: float = 1e-3, outlier_gain: float = 20.0) -> np.ndarray:
    """fp32 [d_out, d_in] weight with a sparse set of amplified entries."""
    g = _rng(seed, stream)
    w = g.standard_normal((d_out, d_in), dtype=np.float32) * np.float32(std)
    mask = g.random((d_out, d_in), dtype=np.float32) < np.float32(outlier_frac)
    w[mask] *= np.float32(outlier_gain)
    return w


def codebook_nf4_style() -> np.ndarray:
    """A 16-entry ascending codebook on [-1, 1] built from normal quantiles.

    Own construction (the values of the published NF4 table are deliberately
    not reproduced): eight positive levels are the N(0,1) quantiles at nine
    evenly spaced probabilities from 0.5 to 1-d (dropping the first, which is
    zero), seven negative levels are the mirrored quantiles at eight evenly
    spaced probabilities (again dropping zero), d = 1/32; both sides are
    divided by the quantile at 1-d so the extreme entries are exactly -1 and
    +1, and one entry is exactly 0.  Computed in fp64, rounded to fp32.
    """
    from scipy.stats import norm
    d = 1.0 / 32.0
    top = norm.ppf(1.0 - d)
    pos = norm.ppf(np.linspace(0.5, 1.0 - d, 9))[1:] / top
    neg = -norm.ppf(np.linspace(0.5, 1.0 - d, 8))[1:][::-1] / top
    cb = np.concatenate([neg, [0.0], pos]).astype(np.float32)
    cb[0], cb[-1] = np.float32(-1.0), np.float32(1.0)
    assert cb.shape == (16,) and np.all(np.diff(cb) > 0)
    return cb


def codebook_int4() -> np.ndarray:
    """The uniform INT4 code values 0..15 (min-max quantizer)."""
    return np.arange(16, dtype=np.float32)


# ----------------------------------------------------------------------------
# workload descriptions (BASELINE configs)
# ----------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Projection:
    name: str
    d_out: int
    d_in: int


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    tokens: int
    rank: int                 # D_rank of the paper; inner rank R = lam * rank
    projections: tuple
    seed: int
    lam: int = 2
    block: int = 64
    scale_mode: int = 0       # 1: double-quantized block scales, groups of 256
    s: float = 1.0


def _llama_layer(h: int, f: int):
    return (Projection("q_proj", h, h), Projection("k_proj", h, h), Projection("v_proj", h, h),
            Projection("o_proj", h, h), Projection("gate_proj", f, h), Projection("up_proj", f, h),
            Projection("down_proj", h, f))


WORKLOADS = {
    "tiny": Workload("tiny", 256, 16, (Projection("proj", 512, 512),), seed=0),
    "llama7b_attn": Workload("llama7b_attn", 8192, 64, (Projection("q_proj", 4096, 4096),), seed=1000),
    "llama7b_mlp": Workload("llama7b_mlp", 8192, 64,
                            (Projection("gate_proj", 11008, 4096), Projection("up_proj", 11008, 4096),
                             Projection("down_proj", 4096, 11008)), seed=2000),
    "llama13b_layer": Workload("llama13b_layer", 16384, 64, _llama_layer(5120, 13824), seed=3000),
    "llama65b_layer": Workload("llama65b_layer", 8192, 128, _llama_layer(8192, 22016), seed=4000, scale_mode=1),
}


@dataclasses.dataclass
class LayerTensors:
    W: np.ndarray        # fp32 [d_out, d_in]
    X: np.ndarray        # uint16 bf16 bits [T, d_in]
    dY: np.ndarray       # uint16 bf16 bits [T, d_out]
    A: np.ndarray        # uint16 bf16 bits [d_in/lam1, R]
    B: np.ndarray        # uint16 bf16 bits [R, d_out/lam2]


def make_layer(seed: int, tokens: int, d_out: int, d_in: int, R: int, lam1: int, lam2: int,
               b_std: float = 0.01, channel_outliers: bool = False) -> LayerTensors:
    """Draw one adapted layer's tensors.  Streams: 0 W, 1 X, 2 dY, 3 A, 4 B, 5 channel mask."""
    W = base_weight(seed, 0, d_out, d_in)
    X = normal_f32(seed, 1, (tokens, d_in))
    if channel_outliers:
        # 0.5 % of input channels carry 20x larger activations
        ch = _rng(seed, 5).random(d_in) < 0.005
        X[:, ch] *= np.float32(20.0)
    dY = normal_f32(seed, 2, (tokens, d_out))
    A = uniform_f32(seed, 3, (d_in // lam1, R), 1.0 / np.sqrt(d_in / lam1))
    B = normal_f32(seed, 4, (R, d_out // lam2), b_std)
    return LayerTensors(W, f32_to_bf16_bits(X), f32_to_bf16_bits(dY), f32_to_bf16_bits(A), f32_to_bf16_bits(B))


def sample_rows(total: int, count: int, seed: int) -> np.ndarray:
    """A sorted, deterministic sample of `count` distinct row indices in [0, total)."""
    count = min(count, total)
    return np.sort(_rng(seed, 99).choice(total, size=count, replace=False)).astype(np.int64)
