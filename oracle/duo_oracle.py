"""Float64 oracle of mixed retrieval/streaming-head attention (test infrastructure).

Source of every definition: the paper's Section 2.2 (the unnumbered pair of
equations defining full_attn and streaming_attn and the sentence describing the
two masks), Section 2.3 "Decoding" and "Chunked Pre-filling", and the caption
of the decoding/pre-filling figure (one sink, two recent tokens, chunks of 4).

The method (an evicting cache, tile skipping, split-K) reaches the plain
definition's result up to rounding, so the oracle IS the definition: it keeps
the whole K/V history of every head and applies the mask.  No ring buffer, no
online softmax, no blocking.

Readings taken where the paper is silent (each is listed in the design notes):
  * masked pairs are excluded from the softmax (score = -inf), not multiplied by 0;
  * scores are scaled by 1/sqrt(head_dim) unless a scale is given;
  * the recent window of a query at position i counts the query itself:
    positions i-R+1 .. i (flip R_INCLUDES_SELF for the other reading);
  * sink set and window are united; nothing is visible beyond position i;
  * in chunked pre-filling a streaming query sees exactly the Lambda mask,
    independent of the chunk size; the deployment text's variant (causal attention
    over [pruned cache || chunk]) is a second mode, visible_mask_deployed;
  * query head h uses KV head h // (Hq / Hkv).

Parity pins (tests/test_oracle_*.py): pure-Python brute force on tiny inputs
including the figure's 16-token case; one-hot-V probes with closed-form
1/|Vis(i)|; torch SDPA (causal) for retrieval heads; R >= N equals causal;
S = 0 equals sliding-window; softmax rows sum to one; GQA == MHA with repeated
KV heads; chunk-size independence; prefill tail == decode steps; closed-form
cache contents.  The 2e-2 / 2e-3 output tolerance is not fixed by the paper:
"parity unpinned" for the tolerance value only.
"""
from __future__ import annotations

import numpy as np

# Reading of "recent tokens": True -> the query's own position is one of the R
# recent positions (window i-R+1..i); False -> R previous positions plus self.
R_INCLUDES_SELF = True


def _window_start(i: int, recent: int) -> int:
    """First position of the recent window of a query at position i."""
    return i - recent + 1 if R_INCLUDES_SELF else i - recent


def visible_mask(i: int, sink: int, recent: int, retrieval: bool) -> np.ndarray:
    """Boolean vector over key positions 0..i: which keys query i may attend to.

    Retrieval head: the causal (lower-triangular) mask row.  Streaming head: the
    Lambda-like mask row - the first `sink` positions plus the recent window
    (Section 2.2, sentence after the two attention equations).
    """
    j = np.arange(i + 1)
    if retrieval:
        return np.ones(i + 1, dtype=bool)
    return (j < sink) | (j >= _window_start(i, recent))


def visible_count(i: int, sink: int, recent: int, retrieval: bool) -> int:
    return int(visible_mask(i, sink, recent, retrieval).sum())


def visible_mask_deployed(i: int, pos0: int, sink: int, recent: int, retrieval: bool) -> np.ndarray:
    """Which keys 0..i the query at position i sees when its chunk starts at position pos0 and the
    streaming heads run plain causal attention over [pruned cache || chunk], as the deployment
    text of Section 2.3 (Chunked Pre-filling) describes it: the cache pruned after the previous
    chunk holds the sink tokens and the last `recent` tokens before pos0, and every earlier token
    of the query's own chunk is visible.  Unlike the Lambda mask this depends on where the chunk
    starts.  Retrieval heads: causal, as always.
    """
    assert 0 <= pos0 <= i
    j = np.arange(i + 1)
    if retrieval:
        return np.ones(i + 1, dtype=bool)
    return (j < sink) | (j >= pos0 - recent)


def attention_rows(q, k_hist, v_hist, positions, retrieval_mask, sink, recent, scale=None, chunk_starts=None):
    """Attention of some queries of one sequence against the full K/V history.
    With chunk_starts (one chunk start per query) the streaming heads use the deployed
    chunk-causal visibility (visible_mask_deployed) instead of the Lambda mask.

    q            [n, Hq, D]   float64, query vectors
    k_hist/v_hist[T, Hkv, D]  float64, keys/values of positions 0..T-1
    positions    [n]          absolute position of each query (each < T)
    retrieval_mask [Hkv]      1 = retrieval (full attention), 0 = streaming
    returns (o [n, Hq, D], lse [Hq, n]) in float64.

    For each query and head: softmax over the visible keys of the scaled dot
    products, then the weighted sum of the visible values (Section 2.2).
    """
    q = np.asarray(q, dtype=np.float64)
    k_hist = np.asarray(k_hist, dtype=np.float64)
    v_hist = np.asarray(v_hist, dtype=np.float64)
    n, hq, d = q.shape
    hkv = k_hist.shape[1]
    assert hq % hkv == 0
    group = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    o = np.zeros((n, hq, d))
    lse = np.zeros((hq, n))
    for r, i in enumerate(positions):
        i = int(i)
        assert 0 <= i < k_hist.shape[0]
        for h in range(hq):
            g = h // group
            if chunk_starts is None:
                vis = visible_mask(i, sink, recent, bool(retrieval_mask[g]))
            else:
                vis = visible_mask_deployed(i, int(chunk_starts[r]), sink, recent, bool(retrieval_mask[g]))
            keys = k_hist[: i + 1, g, :][vis]
            vals = v_hist[: i + 1, g, :][vis]
            s = scale * (keys @ q[r, h])
            m = s.max()
            e = np.exp(s - m)
            z = e.sum()
            o[r, h] = (e / z) @ vals
            lse[h, r] = m + np.log(z)
    return o, lse


def prefill_chunk(q_chunk, k_hist, v_hist, pos0, retrieval_mask, sink, recent, scale=None):
    """One pre-filling chunk of one sequence (Section 2.3, Chunked Pre-filling).

    q_chunk holds the queries of positions pos0 .. pos0+n-1; k_hist/v_hist hold
    positions 0 .. pos0+n-1 (prefix and the chunk itself).
    """
    n = q_chunk.shape[0]
    return attention_rows(q_chunk, k_hist, v_hist, np.arange(pos0, pos0 + n),
                          retrieval_mask, sink, recent, scale)


def prefill_chunk_deployed(q_chunk, k_hist, v_hist, pos0, retrieval_mask, sink, recent, scale=None):
    """One pre-filling chunk with the deployed (chunk-causal) streaming attention of Section 2.3."""
    n = q_chunk.shape[0]
    return attention_rows(q_chunk, k_hist, v_hist, np.arange(pos0, pos0 + n), retrieval_mask, sink, recent, scale,
                          chunk_starts=np.full(n, pos0))


def decode_step(q_tok, k_hist, v_hist, retrieval_mask, sink, recent, scale=None):
    """One decoding step (Section 2.3, Decoding): the query of the newest token,
    position T-1, whose own key/value are the last rows of the history.
    q_tok [Hq, D] -> (o [Hq, D], lse [Hq])."""
    t = k_hist.shape[0]
    o, lse = attention_rows(q_tok[None], k_hist, v_hist, [t - 1],
                            retrieval_mask, sink, recent, scale)
    return o[0], lse[:, 0]


def merge_partials(m, l, o):
    """Merge softmax partials of disjoint key subsets of one query.

    m [P] subset maxima, l [P] subset sums of exp(s - m_p), o [P, D] subset
    sums of exp(s - m_p) * v.  Returns (normalised output [D], lse).  This is
    the associativity identity of the softmax-weighted sum; the paper only
    cites the technique (related work, FlashDecoding).
    """
    m = np.asarray(m, dtype=np.float64)
    l = np.asarray(l, dtype=np.float64)
    o = np.asarray(o, dtype=np.float64)
    big = m.max()
    w = np.exp(m - big)
    z = (w * l).sum()
    return (w[:, None] * o).sum(axis=0) / z, big + np.log(z)


def retained_positions(n_appended: int, sink: int, recent: int, retrieval: bool):
    """Closed form of the cache contents after n_appended tokens: every position
    for a retrieval head; the sinks plus the last `recent` positions for a
    streaming head (Section 2.3, Decoding; figure caption: constant memory)."""
    if retrieval:
        return list(range(n_appended))
    first = max(sink, n_appended - recent)
    return list(range(min(sink, n_appended))) + list(range(first, n_appended))


class CacheModel:
    """The two caches of one (layer, sequence, KV head) as Python lists.

    Written as the mechanism the paper describes - keep the sinks, keep at most
    `recent` later tokens, evict the oldest non-sink one - so it can be checked
    against retained_positions(), the closed form.
    """

    def __init__(self, sink: int, recent: int, retrieval: bool):
        self.sink, self.recent, self.retrieval = sink, recent, retrieval
        self.sinks = []    # (position, k_row, v_row)
        self.window = []   # (position, k_row, v_row), oldest first
        self.count = 0

    def append(self, k_row, v_row):
        p = self.count
        self.count += 1
        item = (p, np.array(k_row, copy=True), np.array(v_row, copy=True))
        if self.retrieval or p < self.sink:
            self.sinks.append(item)
            return
        self.window.append(item)
        if len(self.window) > self.recent:
            self.window.pop(0)

    def positions(self):
        return [it[0] for it in self.sinks] + [it[0] for it in self.window]

    def contents(self):
        items = self.sinks + self.window
        if not items:
            return [], None, None
        return ([it[0] for it in items], np.stack([it[1] for it in items]),
                np.stack([it[2] for it in items]))
