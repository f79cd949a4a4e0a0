"""Pins of the gate-mixed attention oracle (CPU only)."""
import numpy as np
import pytest

import oracle


def _rand(seed, t, hq, hkv, d):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((t, hq, d)), rng.standard_normal((t, hkv, d)), rng.standard_normal((t, hkv, d))


def test_alpha_one_is_causal_attention_torch_sdpa():
    import torch
    q, k, v = _rand(0, 37, 4, 2, 16)
    got = oracle.gate_mixed_attention(q, k, v, np.ones(2), sink=2, recent=5)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, 2, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, 2, axis=1)).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.abs(got - want).max() < 1e-12


@pytest.mark.parametrize("alpha", [0.0, 0.3, 1.0])
def test_uniform_attention_closed_form(alpha):
    # zero queries -> uniform weights: full = mean of v[0..i], streaming = mean over the Lambda set
    t, sink, recent = 23, 2, 4
    _, k, v = _rand(1, t, 1, 1, 8)
    q = np.zeros((t, 1, 8))
    got = oracle.gate_mixed_attention(q, k, v, np.array([alpha]), sink, recent)
    for i in range(t):
        vis = [j for j in range(i + 1) if j < sink or j > i - recent]
        want = alpha * v[: i + 1, 0].mean(axis=0) + (1 - alpha) * v[vis, 0].mean(axis=0)
        assert np.abs(got[i, 0] - want).max() < 1e-12


def test_gate_belongs_to_the_kv_head_of_the_query_group():
    # one-hot values at position 0 of KV head 0 and position 1 of KV head 1; zero queries
    t, hq, hkv, d = 12, 4, 2, 4
    q = np.zeros((t, hq, d))
    k = np.zeros((t, hkv, d))
    v = np.zeros((t, hkv, d))
    v[0, 0, 0] = 1.0
    v[1, 1, 1] = 1.0
    alpha = np.array([0.25, 0.75])
    sink, recent = 1, 3          # position 0 is a sink, position 1 is not
    got = oracle.gate_mixed_attention(q, k, v, alpha, sink, recent)
    i = 9
    n_vis = sink + recent
    for h in (0, 1):             # KV head 0: the one-hot sits in the sink, both terms see it
        assert got[i, h, 0] == pytest.approx(0.25 / (i + 1) + 0.75 / n_vis)
        assert got[i, h, 1] == 0.0
    for h in (2, 3):             # KV head 1: position 1 is outside the Lambda set at i = 9
        assert got[i, h, 1] == pytest.approx(0.75 / (i + 1))
        assert got[i, h, 0] == 0.0


def test_linear_in_alpha():
    q, k, v = _rand(2, 19, 2, 2, 8)
    a = np.array([0.2, 0.9])
    full = oracle.gate_mixed_attention(q, k, v, np.ones(2), 1, 3)
    stream = oracle.gate_mixed_attention(q, k, v, np.zeros(2), 1, 3)
    mix = oracle.gate_mixed_attention(q, k, v, a, 1, 3)
    want = np.repeat(a, 1)[None, :, None] * full + (1 - a)[None, :, None] * stream
    assert np.abs(mix - want).max() < 1e-12
    # and the streaming term is the Lambda-masked attention the deployment path uses
    want_stream, _ = oracle.attention_rows(q, k, v, np.arange(19), np.zeros(2), 1, 3)
    assert np.abs(stream - want_stream).max() < 1e-12


def test_block_mask_of_size_one_is_the_lambda_mask_and_larger_blocks_contain_it():
    for sink, recent in ((0, 1), (1, 2), (3, 5), (4, 4), (16, 64)):
        for i in range(0, 150, 7):
            lam = oracle.visible_mask(i, sink, recent, False)
            assert np.array_equal(oracle.visible_mask_block(i, sink, recent, 1), lam)
            for block in (2, 3, 4, 16, 64):
                blk = oracle.visible_mask_block(i, sink, recent, block)
                assert blk.shape == lam.shape and (blk | ~lam).all()


def test_block_mask_hand_listed_case():
    # sink 1, recent 3, block 2: sink block = keys {0, 1}; local blocks = ceil(2 / 2) + 1 = 2:
    # the query's own block and the one before it
    rows = {
        0: [0],
        1: [0, 1],
        2: [0, 1, 2],
        3: [0, 1, 2, 3],
        4: [0, 1, 2, 3, 4],
        5: [0, 1, 2, 3, 4, 5],
        6: [0, 1, 4, 5, 6],
        7: [0, 1, 4, 5, 6, 7],
        8: [0, 1, 6, 7, 8],
    }
    for i, want in rows.items():
        assert np.flatnonzero(oracle.visible_mask_block(i, 1, 3, 2)).tolist() == want


def test_block_sparse_streaming_term():
    t, sink, recent, block = 21, 1, 3, 2
    _, k, v = _rand(3, t, 1, 1, 4)
    q = np.zeros((t, 1, 4))
    got = oracle.gate_mixed_attention(q, k, v, np.array([0.0]), sink, recent, block=block)
    for i in range(t):
        vis = np.flatnonzero(oracle.visible_mask_block(i, sink, recent, block))
        assert np.abs(got[i, 0] - v[vis, 0].mean(axis=0)).max() < 1e-12
