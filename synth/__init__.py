"""Seeded synthetic inputs shared by the CPU oracle tests and the HIP path.

This module only *makes data*: random bf16 tensors with the shapes, value
distributions and outlier structure of the workloads (Llama-3 shaped linear
layers, KV caches with outlier key channels, activation vectors, calibration
norms, token ids).  It contains none of the method's arithmetic (no selection,
truncation, packing, GEMV, attention or acceptance) and imports neither the
oracle nor the HIP binding.

All tensors that stand for bf16 data are returned as ``numpy.uint16`` bit
patterns, which is what both sides consume.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
    "normal_bf16",
    "weight_matrix",
    "act_norm",
    "activations",
    "kv_tensor",
    "token_ids",
    "LlamaShape",
    "LLAMA3_8B",
    "LLAMA3_70B",
    "TINY",
    "layer_weights",
    "model_weights",
    "rope_table",
]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit pattern (data generation only)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (b + 0x7FFF + ((b >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(u: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))


def normal_bf16(shape, sigma: float, seed: int, stream: int = 0) -> np.ndarray:
    g = _rng(seed, stream)
    x = g.standard_normal(size=shape, dtype=np.float32) * np.float32(sigma)
    return f32_to_bf16_bits(x)


def weight_matrix(rows: int, cols: int, seed: int, sigma: float = 0.02,
                  outlier_frac: float = 0.005, outlier_scale: float = 20.0) -> np.ndarray:
    """W ~ N(0, sigma^2) with a seeded set of input columns scaled up (outlier channels)."""
    g = _rng(seed, 1)
    x = g.standard_normal(size=(rows, cols), dtype=np.float32) * np.float32(sigma)
    n_out = int(round(outlier_frac * cols))
    if n_out > 0:
        idx = _rng(seed, 2).choice(cols, size=n_out, replace=False)
        x[:, idx] *= np.float32(outlier_scale)
    return f32_to_bf16_bits(x)


def act_norm(cols: int, seed: int) -> np.ndarray:
    """Stand-in for per-input-channel activation L2 norms from a calibration set:
    positive, log-normally spread, a few channels much larger."""
    g = _rng(seed, 3)
    a = np.exp(g.standard_normal(size=cols, dtype=np.float32) * np.float32(0.5))
    idx = _rng(seed, 4).choice(cols, size=max(1, cols // 200), replace=False)
    a[idx] *= np.float32(8.0)
    return a.astype(np.float32)


def activations(n: int, ncols: int, seed: int, sigma: float = 1.0) -> np.ndarray:
    """Activation block as bf16 bits, shape [ncols, n] (one row per token column)."""
    return normal_bf16((ncols, n), sigma, seed, stream=5)


def kv_tensor(tokens: int, heads: int, dim: int, seed: int, outlier_channels: int = 4,
              outlier_scale: float = 10.0, sigma: float = 1.0) -> np.ndarray:
    """[tokens, heads, dim] bf16 bits; `outlier_channels` fixed channels per head scaled up
    (keys show channel-wise outliers; pass 0 for value-like tensors)."""
    g = _rng(seed, 6)
    x = g.standard_normal(size=(tokens, heads, dim), dtype=np.float32) * np.float32(sigma)
    if outlier_channels > 0:
        for h in range(heads):
            idx = _rng(seed, 100 + h).choice(dim, size=outlier_channels, replace=False)
            x[:, h, idx] *= np.float32(outlier_scale)
    return f32_to_bf16_bits(x)


def token_ids(n: int, vocab: int, seed: int) -> np.ndarray:
    return _rng(seed, 7).integers(0, vocab, size=n, dtype=np.int32)


class LlamaShape:
    """Shape of a Llama-3 style decoder (names follow the usual architecture terms)."""

    def __init__(self, name, hidden, n_layers, n_q_heads, n_kv_heads, head_dim, ffn, vocab,
                 rope_theta=500000.0, rms_eps=1e-5):
        self.name = name
        self.hidden = hidden
        self.n_layers = n_layers
        self.n_q_heads = n_q_heads
        self.n_kv_heads = n_kv_heads
        self.head_dim = head_dim
        self.ffn = ffn
        self.vocab = vocab
        self.rope_theta = rope_theta
        self.rms_eps = rms_eps

    @property
    def q_dim(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim


LLAMA3_8B = LlamaShape("llama3-8b", 4096, 32, 32, 8, 128, 14336, 128256)
LLAMA3_70B = LlamaShape("llama3-70b", 8192, 80, 64, 8, 128, 28672, 128256)
# small shape the oracle finishes in seconds; head_dim stays 128 (the KV group size)
TINY = LlamaShape("tiny", 256, 2, 4, 2, 128, 512, 1000)


def layer_weights(shape: LlamaShape, seed: int, layer: int = 0, sigma: float = 0.02) -> dict:
    """bf16 bit patterns of one decoder layer: wqkv [(q+2kv) x hidden], wo [hidden x q],
    wgu [2*ffn x hidden] with gate row i at 2i and up row i at 2i+1, wd [hidden x ffn],
    and the two RMSNorm gains."""
    s = seed * 1000 + layer * 10
    h = shape.hidden
    g1 = f32_to_bf16_bits(1.0 + 0.1 * _rng(s, 8).standard_normal(size=h, dtype=np.float32))
    g2 = f32_to_bf16_bits(1.0 + 0.1 * _rng(s, 9).standard_normal(size=h, dtype=np.float32))
    return {
        "wqkv": weight_matrix(shape.q_dim + 2 * shape.kv_dim, h, s + 1, sigma),
        "wo": weight_matrix(h, shape.q_dim, s + 2, sigma),
        "wgu": weight_matrix(2 * shape.ffn, h, s + 3, sigma),
        "wd": weight_matrix(h, shape.ffn, s + 4, sigma),
        "g_attn": g1,
        "g_ffn": g2,
    }


def model_weights(shape: LlamaShape, seed: int, sigma: float = 0.02) -> dict:
    """Whole random-init model (only for shapes small enough to hold on the host)."""
    s = seed * 1000 + 999
    return {
        "embed": normal_bf16((shape.vocab, shape.hidden), 1.0, s, stream=10),
        "layers": [layer_weights(shape, seed, l, sigma) for l in range(shape.n_layers)],
        "g_final": f32_to_bf16_bits(
            1.0 + 0.1 * _rng(s, 11).standard_normal(size=shape.hidden, dtype=np.float32)),
        "lm_head": weight_matrix(shape.vocab, shape.hidden, s + 5, sigma),
    }


def rope_table(max_pos: int, head_dim: int, theta: float) -> np.ndarray:
    """cos/sin table [max_pos, head_dim/2, 2] float32, computed in float64 on the host.
    It is an *input* to both sides (data, not arithmetic of the method)."""
    half = head_dim // 2
    inv = theta ** (-np.arange(half, dtype=np.float64) * 2.0 / head_dim)
    ang = np.arange(max_pos, dtype=np.float64)[:, None] * inv[None, :]
    return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)
