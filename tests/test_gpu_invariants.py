"""Cost invariants of the method on the device (Section 2.3: streaming heads take time linear in the
chunk and constant in the context for pre-filling, and constant time and memory for decoding, while
retrieval heads grow with the context).  Checked as ratios of event-timed launches with wide margins:
a streaming-only layer must cost about the same at 8K and at 256K context, an all-retrieval layer
about as many times more as it has keys to visit."""
import numpy as np
import pytest

from paper_2410_10819_amd import binding as duo
from paper_2410_10819_amd import synth
from helpers import device_fill, device_table, fill_cache_by_append

pytestmark = pytest.mark.gpu

HQ, HKV, D, SINK, RECENT, CHUNK = 8, 8, 128, 64, 256, 4096


def _timed(fn, reps=5):
    import torch
    fn(); fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def _costs(all_retrieval, n_ctx):
    """(prefill ms of one 4096-token chunk, decode ms of one token) of a layer whose cache holds n_ctx tokens."""
    import torch
    mask = np.full((1, HKV), 1 if all_retrieval else 0, dtype=np.uint8)
    table = device_table()
    handle = duo.duo_cache_create(1, 1, HQ, HKV, D, SINK, RECENT, n_ctx + CHUNK, mask)
    try:
        fill_cache_by_append(duo, handle, table, 21, 0, 1, HKV, D, n_ctx)
        q = device_fill(table, 21, 0, synth.TENSOR_Q, 1, n_ctx, CHUNK, HQ, D)
        k = device_fill(table, 21, 0, synth.TENSOR_K, 1, n_ctx, CHUNK, HKV, D)
        v = device_fill(table, 21, 0, synth.TENSOR_V, 1, n_ctx, CHUNK, HKV, D)
        out = torch.empty_like(q)
        t_prefill = _timed(lambda: duo.duo_attn_prefill(handle, 0, q, k, v, CHUNK, out))
        q1, o1 = q[:, :1].contiguous(), torch.empty_like(q[:, :1])
        t_decode = _timed(lambda: duo.duo_attn_decode(handle, 0, q1, o1), reps=20)
        assert np.isfinite(out.float().cpu().numpy()).all()
    finally:
        duo.duo_cache_destroy(handle)
    return t_prefill, t_decode


def test_streaming_heads_cost_the_same_at_any_context_and_retrieval_heads_grow_with_it():
    short, long_ = 8192, 262144
    sp_s, sd_s = _costs(False, short)
    sp_l, sd_l = _costs(False, long_)
    rp_s, rd_s = _costs(True, short)
    rp_l, rd_l = _costs(True, long_)
    # streaming: constant in the context (32x more context, well under 1.5x the time)
    assert sp_l < 1.5 * sp_s, (sp_s, sp_l)
    assert sd_l < 1.5 * sd_s + 0.005, (sd_s, sd_l)
    # retrieval: the chunk visits (context + chunk / 2) keys per row: 25.8x more at 256K than at 8K
    assert rp_l > 10 * rp_s, (rp_s, rp_l)
    assert rd_l > 4 * rd_s, (rd_s, rd_l)
    # and a streaming layer is far cheaper than a retrieval layer at long context
    assert sp_l * 10 < rp_l and sd_l * 4 < rd_l


@pytest.mark.parametrize("kv_dtype", [0, 1, 2, 3])
def test_repeated_calls_give_identical_bits(kv_dtype):
    # the split-K partials are merged in a fixed order by whichever workgroup finishes last, and the
    # pre-filling kernel has no cross-workgroup accumulation: the same call twice gives the same bits
    import torch
    hq, hkv, d, n_ctx = 32, 8, 128, 20000
    mask = synth.retrieval_mask(5, 1, hkv, 0.5)
    table = device_table()
    handle = duo.duo_cache_create(1, 2, hq, hkv, d, SINK, RECENT, n_ctx + 600, mask, kv_dtype)
    try:
        fill_cache_by_append(duo, handle, table, 22, 0, 2, hkv, d, n_ctx)
        q = device_fill(table, 22, 0, synth.TENSOR_Q, 2, n_ctx, 512, hq, d)
        k = device_fill(table, 22, 0, synth.TENSOR_K, 2, n_ctx, 512, hkv, d)
        v = device_fill(table, 22, 0, synth.TENSOR_V, 2, n_ctx, 512, hkv, d)
        outs = []
        for _ in range(3):
            o_pre = torch.empty_like(q)
            lse = torch.empty((2, hq, 512), dtype=torch.float32, device="cuda")
            duo.duo_attn_prefill(handle, 0, q, k, v, 512, o_pre, lse=lse)
            o_dec = torch.empty_like(q[:, :1])
            duo.duo_attn_decode(handle, 0, q[:, :1].contiguous(), o_dec, k=k[:, :1].contiguous(), v=v[:, :1].contiguous())
            outs.append((o_pre, lse, o_dec))
        torch.cuda.synchronize()
        for o_pre, lse, o_dec in outs[1:]:
            assert torch.equal(o_pre, outs[0][0]) and torch.equal(lse, outs[0][1]) and torch.equal(o_dec, outs[0][2])
    finally:
        duo.duo_cache_destroy(handle)
