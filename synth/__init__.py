"""Seeded synthetic inputs shared by the CPU oracle tests and the HIP path.

This module only *makes data*: random bf16 tensors with the shapes, value
distributions and outlier structure of the workloads (Llama-3 shaped linear
layers, KV caches with outlier key channels, activation vectors, calibration
norms, token ids).  It contains none of the method's arithmetic (no selection,
truncation, packing, GEMV, attention or acceptance) and imports neither the
oracle nor the HIP binding.

All tensors that stand for bf16 data are returned as ``numpy.uint16`` bit
patterns, which is what both sides consume (the ``hash_*`` generators at the end, for tensors
too large to draw on the host during a GPU test, return torch int16 tensors on the requested
device with identical bits on CPU and GPU).
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
    "hash_normal_bf16",
    "hash_weight_matrix",
    "hash_kv_tensor",
    "hash_gain",
    "hash_act_norm",
    "llama70b_layer_case",
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


# ---------------------------------------------------------------------------------------------
# Counter-based generator for tensors too large to draw on the host in a GPU test: the same
# integer arithmetic gives the same bits with torch on the CPU (oracle side, golden scripts) and
# on the GPU (HIP side).  value = (sum of twelve uniform 16-bit integers - 6 * 65535) * sigma /
# 65536 (Irwin-Hall, unit variance, +-6 sigma), one float32 multiply, round-to-nearest-even to
# bf16; no library math functions.
# ---------------------------------------------------------------------------------------------
_M64 = (1 << 64) - 1


def _wrap64(v: int) -> int:
    """Python int -> the int64 with the same low 64 bits."""
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


def _mix64(torch, z):
    """splitmix64 finaliser on int64 tensors (wrapping multiply, logical shifts emulated)."""
    z = (z ^ ((z >> 30) & ((1 << 34) - 1))) * _wrap64(0xBF58476D1CE4E5B9)
    z = (z ^ ((z >> 27) & ((1 << 37) - 1))) * _wrap64(0x94D049BB133111EB)
    return z ^ ((z >> 31) & ((1 << 33) - 1))


def hash_normal_bf16(shape, sigma: float, seed: int, tensor_id: int, device="cpu", col_scale=None):
    """bf16 bit patterns (torch int16 tensor of `shape`) of N(0, sigma^2)-like values that depend
    only on (seed, tensor_id, flat index).  col_scale: optional float32 tensor over the last axis,
    multiplied in (a second float32 multiply), e.g. outlier channels."""
    import torch
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, dtype=torch.int16, device=device)
    base = _wrap64(seed * 0x9E3779B97F4A7C15 + tensor_id * 0xD1B54A32D192ED03)
    scale = torch.tensor(sigma / 65536.0, dtype=torch.float32, device=device)
    cols = int(shape[-1])
    step = 1 << 24
    for i0 in range(0, n, step):
        idx = torch.arange(i0, min(n, i0 + step), dtype=torch.int64, device=device)
        acc = torch.zeros_like(idx)
        for j in range(3):
            h = _mix64(torch, (idx * 3 + j) * _wrap64(0x9E3779B97F4A7C15) + base)
            for q in range(4):
                acc += (h >> (16 * q)) & 0xFFFF
        v = (acc - 6 * 65535).to(torch.float32) * scale
        if col_scale is not None:
            v = v * col_scale[idx % cols]
        b = v.view(torch.int32)
        r = (b + 0x7FFF + ((b >> 16) & 1)) >> 16          # finite values only: no NaN handling needed
        out[i0:i0 + idx.numel()] = r.to(torch.int16)
    return out.reshape(tuple(int(s) for s in shape))


def hash_weight_matrix(rows: int, cols: int, seed: int, tensor_id: int, device="cpu", sigma: float = 0.02,
                       outlier_every: int = 200, outlier_scale: float = 20.0):
    """Weight matrix with outlier input columns (every `outlier_every`-th column starting at a
    seed-dependent offset is scaled up), as bf16 bits on `device`."""
    import torch
    cs = torch.ones(cols, dtype=torch.float32, device=device)
    if outlier_every > 0:
        cs[(seed * 7 + tensor_id * 13) % outlier_every::outlier_every] = outlier_scale
    return hash_normal_bf16((rows, cols), sigma, seed, tensor_id, device, cs)


def hash_kv_tensor(tokens: int, heads: int, dim: int, seed: int, tensor_id: int, device="cpu",
                   outlier_channels: int = 4, outlier_scale: float = 10.0):
    """[tokens, heads, dim] bf16 bits; `outlier_channels` channels (the same in every head, spread
    over the head dimension) scaled up, as keys show."""
    import torch
    cs = torch.ones(dim, dtype=torch.float32, device=device)
    for c in range(outlier_channels):
        cs[(seed * 5 + tensor_id * 3 + c * (dim // max(1, outlier_channels)) + 1) % dim] = outlier_scale
    return hash_normal_bf16((tokens, heads, dim), 1.0, seed, tensor_id, device, cs)


def hash_gain(n: int, seed: int, tensor_id: int, device="cpu"):
    """RMSNorm gain 1 + 0.1 * normal as bf16 bits (float32 add, round-to-nearest-even)."""
    import torch
    v = hash_normal_bf16((n,), 0.1, seed, tensor_id, device).view(torch.bfloat16).to(torch.float32) + 1.0
    b = v.view(torch.int32)
    return ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).to(torch.int16)


def hash_act_norm(cols: int, seed: int, tensor_id: int, device="cpu"):
    """Stand-in for calibration activation norms: float32 powers of two between 1/2 and 8, a
    few channels at 8 (integer-driven, so identical on CPU and GPU)."""
    import torch
    idx = torch.arange(cols, dtype=torch.int64, device=device)
    h = _mix64(torch, idx * _wrap64(0x9E3779B97F4A7C15) + _wrap64(seed * 0x2545F4914F6CDD1D + tensor_id))
    table = torch.tensor([0.5, 0.75, 1.0, 1.0, 1.25, 1.5, 2.0, 1.0], dtype=torch.float32, device=device)
    a = table[(h & 7)]
    a[((h >> 8) & 0xFF) == 0] = 8.0
    return a


def llama70b_layer_case(device="cpu"):
    """Inputs of the Llama-3-70B-shaped one-layer case (hidden 8192, 64 q / 8 kv heads, FFN 28672;
    a 512-row output head and vocabulary keep the oracle affordable), 8192 cached positions whose
    keys have outlier channels, draft length 8: identical bits on CPU and GPU."""
    shape = LlamaShape("llama3-70b-1l", 8192, 1, 64, 8, 128, 28672, 512)
    seed, ctx_len, k = 5, 8192, 8
    qkv_rows = shape.q_dim + 2 * shape.kv_dim
    dims = {"wqkv": (qkv_rows, shape.hidden, 1), "wo": (shape.hidden, shape.q_dim, 2),
            "wgu": (2 * shape.ffn, shape.hidden, 3), "wd": (shape.hidden, shape.ffn, 4),
            "lm_head": (shape.vocab, shape.hidden, 5)}
    case = {"shape": shape, "ctx_len": ctx_len, "k": k, "keep": 600, "t": 4, "dims": dims, "seed": seed,
            "tokens": [(7 + 37 * i) % shape.vocab for i in range(k + 1)]}
    case["weight"] = lambda name: hash_weight_matrix(dims[name][0], dims[name][1], seed, dims[name][2], device)
    case["act_norm"] = lambda name: hash_act_norm(dims[name][1], seed, 20 + dims[name][2], device)
    case["embed"] = lambda: hash_normal_bf16((shape.vocab, shape.hidden), 1.0, seed, 6, device)
    case["gain"] = lambda which: hash_gain(shape.hidden, seed, 7 + which, device)     # 0 attn, 1 ffn, 2 final
    case["K"] = lambda: hash_kv_tensor(ctx_len, shape.n_kv_heads, 128, seed, 10, device, outlier_channels=4)
    case["V"] = lambda: hash_kv_tensor(ctx_len, shape.n_kv_heads, 128, seed, 11, device, outlier_channels=0)
    return case
