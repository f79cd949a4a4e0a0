"""duo_attn_decode_static (the allocation-free decode entry point, split-K scratch in a fixed array inside
the library) against duo_attn_decode (scratch owned by the handle): the two run the same kernels over the
same cache, so outputs and log-sum-exps must agree bit for bit - on two calls in a row, the second with a
smaller input, so that whatever the first call left in the shared array is there when the second starts.
Also against the float64 oracle, to the attention tolerance."""
import numpy as np
import pytest

import oracle
from paper_2410_10819_amd import binding as duo
from paper_2410_10819_amd import synth
from helpers import (ATOL_LSE, assert_close, cpu_history_bits, device_fill, device_table, fill_cache_by_append,
                     from_dev_bits)

pytestmark = pytest.mark.gpu

SINK, RECENT = 16, 64


def _one_call(batch, hq, hkv, d, n_ctx, kv_dtype, fused, seed):
    """Returns (static out bits, static lse, reference out bits, reference lse, mask)."""
    import torch
    mask = synth.retrieval_mask(seed, 1, hkv, 0.5)
    table = device_table()
    handle = duo.duo_cache_create(1, batch, hq, hkv, d, SINK, RECENT, n_ctx + 1, mask, kv_dtype)
    try:
        fill_cache_by_append(duo, handle, table, seed, 0, batch, hkv, d, n_ctx, chunk=4096)
        q = device_fill(table, seed, 0, synth.TENSOR_Q, batch, n_ctx, 1, hq, d)
        k = device_fill(table, seed, 0, synth.TENSOR_K, batch, n_ctx, 1, hkv, d) if fused else None
        v = device_fill(table, seed, 0, synth.TENSOR_V, batch, n_ctx, 1, hkv, d) if fused else None
        o_ref, o_st = torch.zeros_like(q), torch.zeros_like(q)
        l_ref = torch.zeros((batch, hq), dtype=torch.float32, device="cuda")
        l_st = torch.zeros_like(l_ref)
        duo.duo_attn_decode_static(handle, 0, q, o_st, k=k, v=v, lse=l_st)
        torch.cuda.synchronize()
        # once the runtime has loaded the kernels (first launch), a call leaves the free device memory as it was
        free0 = torch.cuda.mem_get_info()[0]
        o_st.zero_(); l_st.zero_()
        duo.duo_attn_decode_static(handle, 0, q, o_st, k=k, v=v, lse=l_st)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free0, "the static entry point changed the free device memory"
        duo.duo_attn_decode(handle, 0, q, o_ref, k=k, v=v, lse=l_ref)
        torch.cuda.synchronize()
        return from_dev_bits(o_st), l_st.cpu().numpy(), from_dev_bits(o_ref), l_ref.cpu().numpy(), mask[0]
    finally:
        duo.duo_cache_destroy(handle)


@pytest.mark.parametrize("hq,hkv,kv_dtype,fused", [
    (8, 8, 0, True),     # one query head per KV head, bf16: the vector-unit kernel, new token passed in
    (8, 2, 0, False),    # query groups of 4: the matrix-core kernel, token already appended
    (8, 2, 1, True),     # the same over fp8 codes
])
def test_static_scratch_decode_matches_the_handle_scratch_decode_twice_in_a_row(hq, hkv, kv_dtype, fused):
    d, seed = 128, 41
    # the first call splits every retrieval head over many workgroups (many partial rows and tickets in
    # use); the second, smaller one runs with whatever that left behind in the shared array
    for batch, n_ctx in ((3, 20000), (1, 3000)):
        o_st, l_st, o_ref, l_ref, mask = _one_call(batch, hq, hkv, d, n_ctx, kv_dtype, fused, seed)
        assert np.array_equal(o_st, o_ref), "outputs differ at batch %d, context %d" % (batch, n_ctx)
        assert np.array_equal(l_st.view(np.uint32), l_ref.view(np.uint32))
        if kv_dtype == 0:
            # and the definition: float64 attention of the query at position len (fused) or len - 1
            b = batch - 1
            total = n_ctx + (1 if fused else 0)
            kh = synth.bf16_bits_to_f64(cpu_history_bits(seed, 0, synth.TENSOR_K, b, total, hkv, d))
            vh = synth.bf16_bits_to_f64(cpu_history_bits(seed, 0, synth.TENSOR_V, b, total, hkv, d))
            qf = synth.bf16_bits_to_f64(synth.counter_bf16(seed, 0, synth.TENSOR_Q, b, n_ctx, 1, hq, d))
            want_o, want_lse = oracle.attention_rows(qf, kh, vh, [total - 1], mask, SINK, RECENT)
            assert_close(synth.bf16_bits_to_f64(o_st[b]), want_o, "static decode vs oracle")
            assert np.abs(l_st[b][:, None] - want_lse).max() <= ATOL_LSE


def test_static_scratch_decode_rejects_steps_beyond_its_array():
    # 4096 tickets at most: batch * n_kv_heads = 520 * 8 = 4160
    hq, hkv, d = 8, 8, 64
    mask = np.ones((1, hkv), dtype=np.uint8)
    import torch
    handle = duo.duo_cache_create(1, 520, hq, hkv, d, 4, 8, 16, mask)
    try:
        q = torch.zeros((520, 1, hq, d), dtype=torch.bfloat16, device="cuda")
        o = torch.zeros_like(q)
        duo.duo_kv_append(handle, 0, q, q, 1)
        with pytest.raises(duo.DuoError) as err:
            duo.duo_attn_decode_static(handle, 0, q, o)
        assert err.value.status == duo.DUO_ERANGE and "static scratch" in err.value.message
        duo.duo_attn_decode(handle, 0, q, o)     # the ordinary entry point takes it
        torch.cuda.synchronize()
    finally:
        duo.duo_cache_destroy(handle)


@pytest.mark.parametrize("hq,hkv,kv_dtype", [(8, 8, 0), (8, 2, 1)])
def test_static_scratch_decode_replays_from_a_graph(hq, hkv, kv_dtype):
    # the call allocates nothing and clears its tickets with a kernel, so it can be recorded into a HIP graph:
    # every replay, with eager work and synchronisations of the program between the replays, gives the eager bits
    import torch
    d, n_ctx, seed = 128, 9000, 51
    mask = synth.retrieval_mask(seed, 1, hkv, 0.5)
    table = device_table()
    handle = duo.duo_cache_create(1, 2, hq, hkv, d, 16, 64, n_ctx + 1, mask, kv_dtype)
    try:
        fill_cache_by_append(duo, handle, table, seed, 0, 2, hkv, d, n_ctx, chunk=4096)
        q = device_fill(table, seed, 0, synth.TENSOR_Q, 2, n_ctx, 1, hq, d)
        k = device_fill(table, seed, 0, synth.TENSOR_K, 2, n_ctx, 1, hkv, d)
        v = device_fill(table, seed, 0, synth.TENSOR_V, 2, n_ctx, 1, hkv, d)
        want = torch.zeros_like(q)
        duo.duo_attn_decode_static(handle, 0, q, want, k=k, v=v)      # eager: also the entry point's set-up on this device
        torch.cuda.synchronize()
        got = torch.zeros_like(q)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            duo.duo_attn_decode_static(handle, 0, q, got, k=k, v=v)
        for i in range(4):
            got.zero_()
            other = torch.zeros_like(q)
            duo.duo_attn_decode(handle, 0, q, other, k=k, v=v)         # the program's own eager work in between
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(got.view(torch.int16), want.view(torch.int16)), "replay %d differs from the eager call" % i
            assert torch.equal(other.view(torch.int16), want.view(torch.int16))
    finally:
        duo.duo_cache_destroy(handle)
