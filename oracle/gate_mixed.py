"""Gate-mixed attention forward of the identification phase (test infrastructure).

Section 2.2 (Optimization-based Identification) attaches a gate value alpha in [0, 1] to every KV
head and, in the forward pass, mixes the outputs of full (causal) attention and of streaming
attention (sink + recent tokens only) of that head's query heads:

    attn = alpha * full_attn + (1 - alpha) * streaming_attn

with both terms as defined by the pair of attention equations of the same section.  This is a whole-
sequence forward (no KV cache).  The oracle is that definition written out in float64, one query at
a time.

The appendix (Experimental Details) says that training computes the streaming term with a
block-sparse approximation of the Lambda mask, shown only in a figure that this build does not
have; the paper gives neither the block size nor the rounding rule.  Reading taken here ("parity
unpinned" with respect to the paper): with block size B, query i sees key j <= i iff key block
j // B is one of the first ceil(sink / B) blocks, or lies fewer than ceil((recent - 1) / B) + 1
blocks before the query's block i // B.  It is the smallest block-aligned mask of that shape that
contains the Lambda mask for every i, and B = 1 gives the Lambda mask itself.

Pins (tests/test_oracle_gate.py): alpha = 1 against torch's causal SDPA; alpha = 0 and general
alpha against closed forms for uniform attention (zero queries); per-KV-head gates under GQA;
linearity in alpha; block mask: B = 1 equals the Lambda mask, containment, a hand-listed case.
"""
from __future__ import annotations

import numpy as np

from .duo_oracle import visible_mask


def visible_mask_block(i: int, sink: int, recent: int, block: int) -> np.ndarray:
    """Keys 0..i that query i sees under the block-sparse approximation of the Lambda mask."""
    assert block >= 1
    j = np.arange(i + 1)
    n_sink_blocks = -(-sink // block)
    n_local_blocks = -(-(recent - 1) // block) + 1
    return (j // block < n_sink_blocks) | (i // block - j // block < n_local_blocks)


def _attend(qv, keys, vals, scale):
    s = scale * (keys @ qv)
    e = np.exp(s - s.max())
    return (e / e.sum()) @ vals


def gate_mixed_rows(q_rows, k, v, alpha, positions, sink, recent, scale=None, block=0):
    """Rows `positions` of the gate-mixed forward: q_rows [n, Hq, D] are the queries at those positions,
    k/v [T, Hkv, D] the whole sequence, alpha [Hkv] -> out [n, Hq, D] (float64).

    Query head h uses KV head g = h // (Hq / Hkv) and that head's gate.  block = 0: the streaming term
    uses the Lambda mask; block >= 1: its block-sparse approximation.
    """
    q_rows = np.asarray(q_rows, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    alpha = np.asarray(alpha, dtype=np.float64)
    n, hq, d = q_rows.shape
    hkv = k.shape[1]
    assert hq % hkv == 0 and alpha.shape == (hkv,) and len(positions) == n
    group = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((n, hq, d))
    for r, i in enumerate(positions):
        i = int(i)
        vis = visible_mask(i, sink, recent, False) if block == 0 else visible_mask_block(i, sink, recent, block)
        for h in range(hq):
            g = h // group
            full = _attend(q_rows[r, h], k[: i + 1, g], v[: i + 1, g], scale)
            stream = _attend(q_rows[r, h], k[: i + 1, g][vis], v[: i + 1, g][vis], scale)
            out[r, h] = alpha[g] * full + (1.0 - alpha[g]) * stream
    return out


def gate_mixed_attention(q, k, v, alpha, sink, recent, scale=None, block=0):
    """The whole forward: q [T, Hq, D], k/v [T, Hkv, D], alpha [Hkv] -> out [T, Hq, D] (float64)."""
    q = np.asarray(q, dtype=np.float64)
    return gate_mixed_rows(q, k, v, alpha, np.arange(q.shape[0]), sink, recent, scale, block)
