"""Seeded synthetic inputs for the W4A8 linear-layer path.

This module holds NO arithmetic of the method: it only draws random tensors
with the shapes and value distributions of the benchmark configurations and
rounds them to their storage types.  It is the one module that both the HIP
tests/benchmark and the CPU-oracle tests use, so that both sides see the same
bits.  Everything is returned as numpy arrays of raw bit patterns
(uint16 for bfloat16 / binary16).

The distributions stand in for LLaMA / OPT checkpoints and text activations:
activations are standard normal with a small set of outlier channels scaled
up (the shape described for post-LayerNorm inputs in the paper's Figure 1
discussion), weights are N(0, 0.02), LoRC factors are N(0, 0.01).
"""
from dataclasses import dataclass, field

import numpy as np


def f32_to_bf16_bits(a):
    """Round binary32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32)


def f32_to_f16_bits(a):
    return np.ascontiguousarray(a, np.float32).astype(np.float16).view(np.uint16)


@dataclass(frozen=True)
class Config:
    name: str
    K: int
    N: int
    Ms: tuple
    G: int
    mode: int            # 1 = M1 (pow2 group scales), 2 = M2 (column scale x 2^-k)
    outlier_frac: float  # fraction of input channels that are outliers (0 -> use outlier_count)
    outlier_count: int
    outlier_gain: float
    rank: int = 0        # LoRC rank (0 = none)
    seed: int = 0


CONFIGS = {
    "tiny": Config("tiny", 256, 256, (16,), 128, 1, 0.0, 4, 20.0),
    "opt1p3b_fc1": Config("opt1p3b_fc1", 2048, 8192, (2048,), 256, 2, 0.01, 0, 20.0),
    "llama7b_qkv": Config("llama7b_qkv", 4096, 12288, (1, 16, 256, 4096), 128, 1, 0.01, 0, 20.0),
    "llama7b_ffn_up": Config("llama7b_ffn_up", 4096, 11008, (1, 16, 256, 4096), 128, 1, 0.01, 0, 20.0),
    "llama13b_ffn_lorc": Config("llama13b_ffn_lorc", 5120, 13824, (16, 2048), 128, 1, 0.01, 0, 20.0, rank=8),
    "llama70b_ffn_decode": Config("llama70b_ffn_decode", 8192, 28672, (1, 4, 16, 64), 128, 1, 0.01, 0, 50.0, rank=8),
    # long K into few output channels: the down projections and the attention output of the same models
    "llama7b_ffn_down": Config("llama7b_ffn_down", 11008, 4096, (16, 4096), 128, 1, 0.01, 0, 20.0),
    "llama13b_ffn_down": Config("llama13b_ffn_down", 13824, 5120, (16, 2048), 128, 1, 0.01, 0, 20.0, rank=8),
    "llama70b_ffn_down": Config("llama70b_ffn_down", 28672, 8192, (1, 16, 64), 128, 1, 0.01, 0, 50.0, rank=8),
    "llama7b_attn_out": Config("llama7b_attn_out", 4096, 4096, (16, 4096), 128, 1, 0.01, 0, 20.0),
}


def _rng(seed, tensor_id):
    return np.random.Generator(np.random.Philox(key=[int(seed), int(tensor_id)]))


def outlier_channels(cfg):
    n_out = cfg.outlier_count if cfg.outlier_count else int(cfg.K * cfg.outlier_frac)
    return np.sort(_rng(cfg.seed, 3).choice(cfg.K, size=n_out, replace=False))


def make_x(cfg, M):
    """Activations: bf16 bits [M, K]."""
    x = _rng(cfg.seed, 1).standard_normal((M, cfg.K), dtype=np.float32)
    x[:, outlier_channels(cfg)] *= np.float32(cfg.outlier_gain)
    return f32_to_bf16_bits(x)


def make_w(cfg, K=None, N=None):
    """Weights: bf16 bits [K, N] (input feature k, output channel n)."""
    K = cfg.K if K is None else K
    N = cfg.N if N is None else N
    rng = _rng(cfg.seed, 2)
    out = np.empty((K, N), np.uint16)
    step = max(1, (1 << 24) // N)
    for k0 in range(0, K, step):
        k1 = min(K, k0 + step)
        out[k0:k1] = f32_to_bf16_bits(rng.standard_normal((k1 - k0, N), dtype=np.float32) * np.float32(0.02))
    return out


def make_uv(cfg, rank=None):
    """LoRC factors: U [K, r], V [r, N] as binary16 bits."""
    r = cfg.rank if rank is None else rank
    u = _rng(cfg.seed, 4).standard_normal((cfg.K, r), dtype=np.float32) * np.float32(0.01)
    v = _rng(cfg.seed, 5).standard_normal((r, cfg.N), dtype=np.float32) * np.float32(0.01)
    return f32_to_f16_bits(u), f32_to_f16_bits(v)
