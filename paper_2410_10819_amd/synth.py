"""Seeded synthetic inputs shared by the tests, the benchmark and the oracle's callers.

Holds none of the method's arithmetic: only (a) a counter-based generator of
bf16 values that are approximately N(0,1) and addressable by
(seed, layer, tensor, batch index, position, head, channel), so any slice of a
multi-gigabyte tensor can be regenerated on the CPU, (b) a plain numpy-RNG
generator, (c) bf16 bit-pattern helpers and (d) the seeded retrieval-head
choice.  The benchmark configurations use N(0,1) Q/K/V of the Llama-2-7B /
Llama-3-8B attention shapes in place of real activations.

The device twin of the counter-based generator (csrc/synth_fill.hip) uses the
same integer recipe and the same table, so both produce identical bits.
"""
from __future__ import annotations

import numpy as np

TENSOR_Q, TENSOR_K, TENSOR_V = 0, 1, 2
_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)


def f32_to_bf16_bits(x) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(bits) -> np.ndarray:
    return bf16_bits_to_f32(bits).astype(np.float64)


_TABLE = None


def normal_table_bf16() -> np.ndarray:
    """65536 bf16 bit patterns: the standard-normal quantile at (k + 0.5) / 65536."""
    global _TABLE
    if _TABLE is None:
        from scipy.special import ndtri
        p = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
        _TABLE = f32_to_bf16_bits(ndtri(p).astype(np.float32))
    return _TABLE


def _mix(x: np.ndarray) -> np.ndarray:
    """64-bit finaliser (xor-shift / multiply rounds) on uint64 arrays."""
    x = x ^ (x >> np.uint64(30))
    x = x * _C1
    x = x ^ (x >> np.uint64(27))
    x = x * _C2
    x = x ^ (x >> np.uint64(31))
    return x


def stream_key(seed: int, layer: int, tensor: int, batch_idx: int) -> int:
    """One 64-bit key per (seed, layer, tensor, sequence)."""
    with np.errstate(over="ignore"):
        a = _mix(np.array([seed], dtype=np.uint64) * _GOLDEN + np.uint64(1))
        b = _mix(a + np.array([(layer << 40) | (tensor << 32) | batch_idx], dtype=np.uint64))
    return int(b[0])


def counter_bf16(seed, layer, tensor, batch_idx, pos_start, n_pos, n_heads, head_dim, heads=None) -> np.ndarray:
    """bf16 bits [n_pos, n_heads, head_dim] of positions pos_start .. pos_start+n_pos-1.

    With `heads` (a list of head indices) only those heads are produced:
    [n_pos, len(heads), head_dim], the same bits the full tensor holds there.
    """
    key = np.uint64(stream_key(seed, layer, tensor, batch_idx))
    tab = normal_table_bf16()
    head_list = np.arange(n_heads, dtype=np.uint64) if heads is None else np.asarray(heads, dtype=np.uint64)
    # counter of (pos, head, d) = (pos * n_heads + head) * head_dim + d
    inner = (head_list[:, None] * np.uint64(head_dim) + np.arange(head_dim, dtype=np.uint64)[None, :]).reshape(-1)
    out = np.empty((n_pos, inner.size), dtype=np.uint16)
    per_pos = np.uint64(n_heads * head_dim)
    block = max(1, (1 << 17) // max(inner.size, 1))        # keep the temporaries cache-sized
    for p0 in range(0, n_pos, block):
        p1 = min(n_pos, p0 + block)
        pos = np.arange(pos_start + p0, pos_start + p1, dtype=np.uint64)
        with np.errstate(over="ignore"):
            idx = pos[:, None] * per_pos + inner[None, :]
            h = _mix(key ^ (idx * _GOLDEN))
        out[p0:p1] = tab[(h >> np.uint64(48)).astype(np.int64)]
    return out.reshape(n_pos, head_list.size, head_dim)


def counter_bf16_batch(seed, layer, tensor, batch, pos_start, n_pos, n_heads, head_dim) -> np.ndarray:
    """[batch, n_pos, n_heads, head_dim] bf16 bits."""
    return np.stack([counter_bf16(seed, layer, tensor, b, pos_start, n_pos, n_heads, head_dim)
                     for b in range(batch)])


def randn_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    """N(0,1) from a numpy Generator, rounded to bf16 bits."""
    return f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


def retrieval_mask(seed: int, n_layers: int, n_kv_heads: int, ratio: float) -> np.ndarray:
    """uint8 [n_layers, n_kv_heads], 1 = retrieval head; round(ratio * n_kv_heads)
    heads per layer chosen by a seeded permutation."""
    n_ret = int(round(ratio * n_kv_heads))
    out = np.zeros((n_layers, n_kv_heads), dtype=np.uint8)
    for layer in range(n_layers):
        perm = np.random.default_rng(seed + layer).permutation(n_kv_heads)
        out[layer, perm[:n_ret]] = 1
    return out
