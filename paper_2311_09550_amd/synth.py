"""Seeded synthetic inputs for the W4A8 linear path.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic (no quantisation, no packing, no scaling by absmax).  It
serves the CPU oracle's tests and the GPU library's tests alike, so both see
bit-identical inputs.

The tensors stand in for LLaMA linear layers: weights ~ N(0, sigma=0.02) as at
initialisation, activations ~ N(0,1) with a fixed 0.1 % of the channels scaled
by 50 (channel-wise outliers, the structure Sec. 1 of the paper describes for
large models).  No trained weights or dataset are used or needed.
"""
from __future__ import annotations

import math

import numpy as np

BASE_SEED = 0

# (N, K) of the fused linears of one decoder layer, by model size.
LLAMA_SHAPES = {
    "7b": {"qkv": (12288, 4096), "o": (4096, 4096), "gate_up": (22016, 4096), "down": (4096, 11008)},
    "13b": {"qkv": (15360, 5120), "o": (5120, 5120), "gate_up": (27648, 5120), "down": (5120, 13824)},
    "70b": {"qkv": (10240, 8192), "o": (8192, 8192), "gate_up": (57344, 8192), "down": (8192, 28672)},
}

# GEMM shapes the paper itself timed (Table 5); N = 11088 is printed there.
PAPER_TABLE5_SHAPES = [(4096, 4096), (1024, 8192), (11088, 4096), (5120, 5120)]


def rng(*tag: int) -> np.random.Generator:
    """PCG64 stream keyed by the base seed and an integer tag (config id, N, K, M, ...)."""
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([BASE_SEED, *tag])))


def uniform_codes(M: int, N: int, K: int, config_id: int = 1):
    """Config-1 style raw codes: int8 activations uniform on [-127,127], int4 weight
    values uniform on [-8,7] (unpacked, one per int8), fp32 scales uniform [1e-3,1e-2]."""
    g = rng(config_id, N, K, M)
    xq = g.integers(-127, 128, size=(M, K), dtype=np.int8)
    wq = g.integers(-8, 8, size=(N, K), dtype=np.int8)
    s_a = g.uniform(1e-3, 1e-2, size=M).astype(np.float32)
    s_w = g.uniform(1e-3, 1e-2, size=N).astype(np.float32)
    return xq, wq, s_a, s_w


def outlier_channels(K: int, config_id: int = 2) -> np.ndarray:
    """ceil(0.001*K) channel indices, fixed per (config, K): outliers are channel-wise."""
    g = rng(config_id, 0, K, 0)
    n_out = int(math.ceil(0.001 * K))
    return np.sort(g.choice(K, size=n_out, replace=False))


def activations_fp16(M: int, K: int, config_id: int = 2, tag: int = 0) -> np.ndarray:
    """fp16 [M][K]: N(0,1) with the outlier channels multiplied by 50."""
    g = rng(config_id, tag, K, M)
    x = g.standard_normal(size=(M, K), dtype=np.float32)
    x[:, outlier_channels(K, config_id)] *= 50.0
    return x.astype(np.float16)


def weights_fp16(N: int, K: int, config_id: int = 2, sigma: float = 0.02) -> np.ndarray:
    """fp16 [N][K]: N(0, sigma), sigma being the standard deviation."""
    g = rng(config_id, N, K, -1 & 0xFFFF)
    w = g.standard_normal(size=(N, K), dtype=np.float32)
    w *= np.float32(sigma)
    return w.astype(np.float16)


def group_scales(N: int, K: int, group: int = 128, config_id: int = 1) -> np.ndarray:
    """fp32 [K/group][N]: one positive scale per group of `group` consecutive k of every output channel, drawn
    log-uniformly over [1e-3, 1e-2] (a decade of spread inside a channel, as group-wise weight quantisation gives
    when a channel's magnitude varies along k)."""
    g = rng(config_id, N, K, group, 7)
    return np.exp(g.uniform(math.log(1e-3), math.log(1e-2), size=(K // group, N))).astype(np.float32)
