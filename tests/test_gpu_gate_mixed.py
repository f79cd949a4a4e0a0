"""duo_attn_gate_mixed against the gate-mixed attention oracle (Section 2.2, identification forward)."""
import numpy as np
import pytest

import oracle
from paper_2410_10819_amd import binding as duo
from paper_2410_10819_amd import synth
from helpers import make_qkv, to_dev, from_dev_f64, assert_close

pytestmark = pytest.mark.gpu


def _run(hq, hkv, d, sink, recent, batch, t, alpha, block, seed=3, check_batches=None, rows=None):
    import torch
    q, k, v = make_qkv(seed, batch, t, hq, hkv, d)
    # the layer's own head classes must play no part: give it an arbitrary mix
    mask = np.array([(h * 7 + 1) % 2 for h in range(hkv)], dtype=np.uint8)
    handle = duo.duo_cache_create(1, batch, hq, hkv, d, sink, recent, 64, mask[None])
    try:
        out = torch.empty((batch, t, hq, d), dtype=torch.bfloat16, device="cuda")
        duo.duo_attn_gate_mixed(handle, 0, to_dev(q), to_dev(k), to_dev(v), t, alpha, out, block=block)
        torch.cuda.synchronize()
        assert duo.duo_cache_len(handle, 0) == 0
        got = from_dev_f64(out)
    finally:
        duo.duo_cache_destroy(handle)
    for b in (range(batch) if check_batches is None else check_batches):
        want = oracle.gate_mixed_attention(synth.bf16_bits_to_f64(q[b]), synth.bf16_bits_to_f64(k[b]),
                                           synth.bf16_bits_to_f64(v[b]), alpha, sink, recent, block=block)
        sel = slice(None) if rows is None else rows
        assert_close(got[b][sel], want[sel], "batch %d" % b)


@pytest.mark.parametrize("hq,hkv,d,sink,recent,t,block", [
    (8, 8, 64, 16, 64, 700, 0),        # MHA, several tiles and a ragged tail
    (8, 2, 128, 4, 32, 523, 0),        # GQA 4, window shorter than a tile
    (4, 4, 128, 64, 256, 1100, 0),     # the deployment constants
    (4, 2, 64, 0, 5, 130, 0),          # no sinks
    (2, 2, 128, 1, 2, 16, 0),          # the figure's parameters
    (8, 2, 128, 128, 256, 1500, 128),  # training constants, block-aligned mask
    (4, 4, 64, 16, 64, 700, 32),
    (4, 2, 128, 5, 40, 333, 7),        # a block size that divides nothing
    (4, 4, 64, 16, 64, 300, 1),        # block of one = the Lambda mask
])
def test_gate_mixed_forward(hq, hkv, d, sink, recent, t, block):
    rng = np.random.default_rng(hq * 100 + t)
    alpha = rng.uniform(0, 1, hkv).astype(np.float32)
    alpha[0] = 1.0                      # a pure retrieval head
    if hkv > 1:
        alpha[-1] = 0.0                 # and a pure streaming head
    _run(hq, hkv, d, sink, recent, 2 if t < 600 else 1, t, alpha, block)


def test_gate_values_are_validated():
    import torch
    mask = np.array([[1, 0]], dtype=np.uint8)
    h = duo.duo_cache_create(1, 1, 4, 2, 64, 4, 8, 16, mask)
    try:
        x = torch.zeros((1, 8, 4, 64), dtype=torch.bfloat16, device="cuda")
        kv = torch.zeros((1, 8, 2, 64), dtype=torch.bfloat16, device="cuda")
        for bad in ([0.5, 1.5], [-0.1, 0.2], [float("nan"), 0.0]):
            with pytest.raises(duo.DuoError) as e:
                duo.duo_attn_gate_mixed(h, 0, x, kv, kv, 8, bad, x.clone(), x.clone())
            assert e.value.status == duo.DUO_EINVAL
        with pytest.raises(duo.DuoError) as e:
            duo.duo_attn_gate_mixed(h, 0, x, kv, kv, 8, [0.5, 0.5], x.clone(), x.clone(), block=-2)
        assert e.value.status == duo.DUO_EINVAL
        with pytest.raises(duo.DuoError) as e:
            duo.duo_attn_gate_mixed(h, 0, x, kv, kv, 0, [0.5, 0.5], x.clone(), x.clone())
        assert e.value.status == duo.DUO_EINVAL
    finally:
        duo.duo_cache_destroy(h)
