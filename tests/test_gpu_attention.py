"""duo_attn_prefill / duo_attn_decode against the float64 oracle, element by element."""
import numpy as np
import pytest

import oracle
from paper_2410_10819_amd import binding as duo
from paper_2410_10819_amd import synth
from helpers import (ATOL_LSE, assert_close, make_qkv, oracle_rows, run_scenario, to_dev, from_dev_f64)

pytestmark = pytest.mark.gpu


def _check_all(cfg, q, k, v, out_bits, lse, positions=None):
    total = q.shape[1]
    positions = np.arange(total) if positions is None else np.asarray(positions)
    worst = (0.0, 0.0)
    for b in range(cfg["batch"]):
        want_o, want_lse = oracle_rows(cfg, q, k, v, positions, b)
        got = synth.bf16_bits_to_f64(out_bits[b][positions])
        worst = max(worst, assert_close(got, want_o, "batch %d" % b))
        if lse is not None:
            assert np.abs(lse[b][:, positions] - want_lse).max() <= ATOL_LSE
    return worst


# configuration 1 of the benchmark list: 8 MHA heads, head_dim 64, 2048 prefill + 64 decode,
# sink 16, recent 256, 4 of 8 heads retrieval.
def _config1():
    mask = synth.retrieval_mask(0, 1, 8, 0.5)[0]
    return dict(batch=1, hq=8, hkv=8, d=64, sink=16, recent=256, mask=mask, max_seq=2048 + 64)


@pytest.mark.parametrize("chunks", [[2048], [256] * 8])
def test_config1_full_tensor_parity(chunks):
    cfg = _config1()
    q, k, v = make_qkv(1, 1, 2048 + 64, 8, 8, 64)
    out, lse, handle = run_scenario(duo, cfg, q, k, v, chunks, 64)
    try:
        _check_all(cfg, q, k, v, out, lse)
    finally:
        duo.duo_cache_destroy(handle)


def test_config1_numpy_rng_inputs_and_fused_decode():
    cfg = _config1()
    q, k, v = make_qkv(5, 1, 1024 + 48, 8, 8, 64, generator="numpy")
    cfg["max_seq"] = 1024 + 48
    out, lse, handle = run_scenario(duo, cfg, q, k, v, [1024], 48, fused_decode=True, pass_params=True)
    try:
        _check_all(cfg, q, k, v, out, lse)
    finally:
        duo.duo_cache_destroy(handle)


@pytest.mark.parametrize("hq,hkv,d,sink,recent,chunks,n_decode,batch", [
    (8, 2, 128, 4, 32, [300, 1, 77, 130], 20, 2),       # GQA 4, ragged chunks, batch 2
    (4, 4, 128, 64, 256, [129, 513], 9, 1),             # deployment constants, tile tails
    (16, 2, 64, 0, 5, [70, 70], 12, 1),                 # GQA 8, no sinks, tiny window
    (4, 2, 64, 3, 1, [65], 6, 3),                       # window of one token
    (2, 2, 128, 8, 1000, [100, 50], 5, 1),              # window longer than the sequence
])
def test_mixed_heads_ragged_shapes(hq, hkv, d, sink, recent, chunks, n_decode, batch):
    total = sum(chunks) + n_decode
    mask = np.array([(h % 2) for h in range(hkv)], dtype=np.uint8)
    cfg = dict(batch=batch, hq=hq, hkv=hkv, d=d, sink=sink, recent=recent, mask=mask, max_seq=total)
    q, k, v = make_qkv(hq * 100 + d, batch, total, hq, hkv, d)
    out, lse, handle = run_scenario(duo, cfg, q, k, v, chunks, n_decode)
    try:
        _check_all(cfg, q, k, v, out, lse)
    finally:
        duo.duo_cache_destroy(handle)


@pytest.mark.parametrize("kv_dtype", [0, 1])
@pytest.mark.parametrize("mode", [False, True, "step"])
def test_three_decode_forms_agree_with_the_oracle(mode, kv_dtype):
    # separate append + decode, un-committed k/v, and the one-launch step; the ring wraps
    # several times and the retrieval cache crosses split boundaries
    hq, hkv, d, sink, recent = 8, 4, 128, 4, 24
    n_fill, n_decode = 600, 70
    total = n_fill + n_decode
    mask = np.array([1, 0, 0, 1], dtype=np.uint8)
    cfg = dict(batch=2, hq=hq, hkv=hkv, d=d, sink=sink, recent=recent, mask=mask, max_seq=total, kv_dtype=kv_dtype)
    q, k, v = make_qkv(77, 2, total, hq, hkv, d)
    import torch
    handle = duo.duo_cache_create(1, 2, hq, hkv, d, sink, recent, total, mask[None], kv_dtype)
    try:
        duo.duo_kv_append(handle, 0, to_dev(k[:, :n_fill]), to_dev(v[:, :n_fill]), n_fill)
        got = np.zeros((2, n_decode, hq, d))
        for t in range(n_decode):
            p = n_fill + t
            qd, kd, vd = (to_dev(x[:, p:p + 1]) for x in (q, k, v))
            od = torch.empty((2, 1, hq, d), dtype=torch.bfloat16, device="cuda")
            if mode == "step":
                duo.duo_decode_step(handle, 0, qd, kd, vd, od)
            elif mode:
                duo.duo_attn_decode(handle, 0, qd, od, k=kd, v=vd)
                duo.duo_kv_append(handle, 0, kd, vd, 1)
            else:
                duo.duo_kv_append(handle, 0, kd, vd, 1)
                duo.duo_attn_decode(handle, 0, qd, od)
            got[:, t] = from_dev_f64(od)[:, 0]
            assert duo.duo_cache_len(handle, 0) == p + 1
        for b in range(2):
            want_o, _ = oracle_rows(cfg, q, k, v, np.arange(n_fill, total), b)
            assert_close(got[b], want_o, "mode %s batch %d" % (mode, b))
        # the caches end up identical to what plain appends produce (bit-exact, via export)
        pos_out = torch.empty(total, dtype=torch.int64, device="cuda")
        for h in range(hkv):
            dt = torch.uint8 if kv_dtype else torch.bfloat16
            ko = torch.zeros((total, d), dtype=dt, device="cuda")
            vo = torch.zeros((total, d), dtype=dt, device="cuda")
            ks = torch.zeros(total, dtype=torch.float32, device="cuda") if kv_dtype else None
            vs = torch.zeros(total, dtype=torch.float32, device="cuda") if kv_dtype else None
            n = duo.duo_cache_export(handle, 0, 1, h, ko, vo, pos_out, total, kscale_out=ks, vscale_out=vs)
            keep = oracle.retained_positions(total, sink, recent, bool(mask[h]))
            assert pos_out[:n].cpu().tolist() == keep
            want_k = k[1, keep, h]
            if kv_dtype:
                codes, scales = oracle.quantize_rows(synth.bf16_bits_to_f32(want_k))
                assert np.array_equal(ko[:n].cpu().numpy(), codes)
                assert np.array_equal(ks[:n].cpu().numpy().view(np.uint32), scales.view(np.uint32))
            else:
                assert np.array_equal(ko[:n].cpu().view(torch.int16).numpy().view(np.uint16), want_k)
    finally:
        duo.duo_cache_destroy(handle)


@pytest.mark.parametrize("mask_kind", ["all_retrieval", "all_streaming"])
def test_single_class_layers(mask_kind):
    hq, hkv, d, total = 4, 4, 64, 400
    mask = np.full(hkv, 1 if mask_kind == "all_retrieval" else 0, dtype=np.uint8)
    cfg = dict(batch=1, hq=hq, hkv=hkv, d=d, sink=4, recent=16, mask=mask, max_seq=total)
    q, k, v = make_qkv(9, 1, total, hq, hkv, d)
    out, lse, handle = run_scenario(duo, cfg, q, k, v, [150, 200], 50)
    try:
        _check_all(cfg, q, k, v, out, lse)
    finally:
        duo.duo_cache_destroy(handle)


def test_decode_only_from_empty_cache_and_split_independence():
    import torch
    hq, hkv, d, total = 8, 2, 128, 1500
    mask = np.array([1, 0], dtype=np.uint8)
    cfg = dict(batch=1, hq=hq, hkv=hkv, d=d, sink=4, recent=64, mask=mask, max_seq=total)
    q, k, v = make_qkv(21, 1, total, hq, hkv, d)
    handle = duo.duo_cache_create(1, 1, hq, hkv, d, 4, 64, total, mask[None])
    try:
        # first tokens one by one (fused form on the empty cache), then a bulk append
        outs = {}
        for t in range(3):
            qd, kd, vd = (to_dev(x[:, t:t + 1]) for x in (q, k, v))
            od = torch.empty((1, 1, hq, d), dtype=torch.bfloat16, device="cuda")
            duo.duo_attn_decode(handle, 0, qd, od, k=kd, v=vd)
            duo.duo_kv_append(handle, 0, kd, vd, 1)
            outs[t] = from_dev_f64(od)[0, 0]
        duo.duo_kv_append(handle, 0, to_dev(k[:, 3:total]), to_dev(v[:, 3:total]), total - 3)
        qd = to_dev(q[:, total - 1:total])
        results = []
        for splits in (0, 1, 2, 7, 64):
            duo.duo_set_decode_splits(handle, splits)
            od = torch.empty((1, 1, hq, d), dtype=torch.bfloat16, device="cuda")
            ld = torch.empty((1, hq), dtype=torch.float32, device="cuda")
            duo.duo_attn_decode(handle, 0, qd, od, lse=ld)
            results.append((from_dev_f64(od)[0, 0], ld.cpu().numpy()[0]))
        want_o, want_lse = oracle_rows(cfg, q, k, v, [0, 1, 2, total - 1])
        for t in range(3):
            assert_close(outs[t], want_o[t], "token %d" % t)
        for got, got_lse in results:
            assert_close(got, want_o[3], "last token")
            assert np.abs(got_lse - want_lse[:, 3]).max() <= ATOL_LSE
        # determinism: same call twice -> identical bits
        od2 = torch.empty((1, 1, hq, d), dtype=torch.bfloat16, device="cuda")
        duo.duo_attn_decode(handle, 0, qd, od2)
        od3 = torch.empty((1, 1, hq, d), dtype=torch.bfloat16, device="cuda")
        duo.duo_attn_decode(handle, 0, qd, od3)
        assert torch.equal(od2, od3)
    finally:
        duo.duo_cache_destroy(handle)


def test_one_hot_value_probe_on_device():
    # Q = 0 -> uniform softmax; V one-hot at j* -> output 1/|Vis| or exactly 0 (mask edges)
    import torch
    hq = hkv = 2
    d, sink, recent, total = 64, 16, 48, 200      # S + R = 64: power-of-two counts are exact in bf16
    mask = np.array([1, 0], dtype=np.uint8)
    cfg = dict(batch=1, hq=hq, hkv=hkv, d=d, sink=sink, recent=recent, mask=mask, max_seq=total)
    q = np.zeros((1, total, hq, d), dtype=np.uint16)
    k = make_qkv(2, 1, total, hq, hkv, d)[1]
    for jstar in (0, 15, 16, 100, 151, 152):
        v = np.zeros((1, total, hkv, d), dtype=np.uint16)
        v[0, jstar, :, 0] = 0x3F80                # bf16 1.0
        out, _, handle = run_scenario(duo, cfg, q, k, v, [128, 64], 8, want_lse=False)
        duo.duo_cache_destroy(handle)
        got = synth.bf16_bits_to_f64(out)[0, :, :, 0]
        for i in range(total):
            in_vis = jstar <= i and (jstar < sink or i - jstar < recent)
            if not in_vis:
                assert got[i, 1] == 0.0, (jstar, i)
            else:
                assert abs(got[i, 1] - 1.0 / min(i + 1, sink + recent)) <= 2.0 ** -8 / min(i + 1, 64)
            if jstar > i:
                assert got[i, 0] == 0.0
            else:
                assert abs(got[i, 0] - 1.0 / (i + 1)) <= 2.0 ** -8 / (i + 1)


@pytest.mark.parametrize("hq,hkv,d", [(8, 2, 128), (4, 4, 64)])
def test_fp8_cache_decode(hq, hkv, d):
    import torch
    total, n_decode = 700, 12
    mask = np.array([(h + 1) % 2 for h in range(hkv)], dtype=np.uint8)
    cfg = dict(batch=2, hq=hq, hkv=hkv, d=d, sink=8, recent=40, mask=mask, max_seq=total, kv_dtype=1)
    q, k, v = make_qkv(31, 2, total, hq, hkv, d)
    handle = duo.duo_cache_create(1, 2, hq, hkv, d, 8, 40, total, mask[None], duo.DUO_KV_FP8_E4M3)
    try:
        pos = total - n_decode
        duo.duo_kv_append(handle, 0, to_dev(k[:, :pos]), to_dev(v[:, :pos]), pos)
        got = np.zeros((2, n_decode, hq, d))
        got_lse = np.zeros((2, hq, n_decode))
        for t in range(n_decode):
            duo.duo_kv_append(handle, 0, to_dev(k[:, pos + t:pos + t + 1]), to_dev(v[:, pos + t:pos + t + 1]), 1)
            od = torch.empty((2, 1, hq, d), dtype=torch.bfloat16, device="cuda")
            ld = torch.empty((2, hq), dtype=torch.float32, device="cuda")
            duo.duo_attn_decode(handle, 0, to_dev(q[:, pos + t:pos + t + 1]), od, lse=ld)
            got[:, t] = from_dev_f64(od)[:, 0]
            got_lse[:, :, t] = ld.cpu().numpy()
        for b in range(2):
            want_o, want_lse = oracle_rows(cfg, q, k, v, np.arange(pos, total), b)
            assert_close(got[b], want_o, "fp8 batch %d" % b)
            assert np.abs(got_lse[b] - want_lse).max() <= ATOL_LSE
    finally:
        duo.duo_cache_destroy(handle)


@pytest.mark.parametrize("kv_dtype", [2, 3])
@pytest.mark.parametrize("hq,hkv,d,batch,n_fill", [(8, 2, 128, 2, 700), (32, 8, 128, 1, 4200), (8, 4, 64, 3, 1111)])
def test_int4_and_int8_cache_decode(hq, hkv, d, batch, n_fill, kv_dtype):
    # integer-code caches: fill by append, decode with the fused step (which quantises the new token
    # itself) and with append-then-attend; the oracle attends over its own codec's round trip
    mask = np.array([(h + 1) % 2 for h in range(hkv)], dtype=np.uint8)
    _decode_vs_oracle(hq, hkv, d, 8, 40, batch, n_fill, 5, kv_dtype, mask)
    cfg = dict(batch=batch, hq=hq, hkv=hkv, d=d, sink=8, recent=40, mask=mask, max_seq=n_fill + 3,
               kv_dtype=kv_dtype)
    q, k, v = make_qkv(77, batch, n_fill + 3, hq, hkv, d)
    out, lse, handle = run_scenario_decode_only(cfg, q, k, v, n_fill, 3)
    for b in range(batch):
        want_o, want_lse = oracle_rows(cfg, q, k, v, np.arange(n_fill, n_fill + 3), b)
        assert_close(out[b], want_o, "kv_dtype %d batch %d" % (kv_dtype, b))
        assert np.abs(lse[b] - want_lse).max() <= ATOL_LSE


def run_scenario_decode_only(cfg, q, k, v, n_fill, n_decode):
    """Append n_fill tokens, then n_decode times append one token and attend (two calls per step)."""
    import torch
    b, hq, hkv, d = cfg["batch"], cfg["hq"], cfg["hkv"], cfg["d"]
    handle = duo.duo_cache_create(1, b, hq, hkv, d, cfg["sink"], cfg["recent"], cfg["max_seq"],
                                  np.asarray(cfg["mask"], dtype=np.uint8)[None], cfg["kv_dtype"])
    try:
        duo.duo_kv_append(handle, 0, to_dev(k[:, :n_fill]), to_dev(v[:, :n_fill]), n_fill)
        out = np.zeros((b, n_decode, hq, d))
        lse = np.zeros((b, hq, n_decode))
        for t in range(n_decode):
            p = n_fill + t
            duo.duo_kv_append(handle, 0, to_dev(k[:, p:p + 1]), to_dev(v[:, p:p + 1]), 1)
            od = torch.empty((b, 1, hq, d), dtype=torch.bfloat16, device="cuda")
            ld = torch.empty((b, hq), dtype=torch.float32, device="cuda")
            duo.duo_attn_decode(handle, 0, to_dev(q[:, p:p + 1]), od, lse=ld)
            out[:, t] = from_dev_f64(od)[:, 0]
            lse[:, :, t] = ld.cpu().numpy()
    finally:
        duo.duo_cache_destroy(handle)
    return out, lse, handle


def _decode_vs_oracle(hq, hkv, d, sink, recent, batch, n_fill, n_decode, kv_dtype, mask, kernel=0, splits=0,
                      check_batches=None, seed=91):
    """Fill by append, then n_decode one-launch steps; every output row against the oracle."""
    import torch
    total = n_fill + n_decode
    cfg = dict(batch=batch, hq=hq, hkv=hkv, d=d, sink=sink, recent=recent, mask=mask, max_seq=total,
               kv_dtype=kv_dtype)
    q, k, v = make_qkv(seed, batch, total, hq, hkv, d)
    handle = duo.duo_cache_create(1, batch, hq, hkv, d, sink, recent, total, mask[None], kv_dtype)
    try:
        duo.duo_set_decode_kernel(handle, kernel)
        duo.duo_set_decode_splits(handle, splits)
        if n_fill:
            duo.duo_kv_append(handle, 0, to_dev(k[:, :n_fill]), to_dev(v[:, :n_fill]), n_fill)
        got = np.zeros((batch, n_decode, hq, d))
        got_lse = np.zeros((batch, hq, n_decode))
        for t in range(n_decode):
            p = n_fill + t
            qd, kd, vd = (to_dev(x[:, p:p + 1]) for x in (q, k, v))
            od = torch.empty((batch, 1, hq, d), dtype=torch.bfloat16, device="cuda")
            ld = torch.empty((batch, hq), dtype=torch.float32, device="cuda")
            duo.duo_decode_step(handle, 0, qd, kd, vd, od, lse=ld)
            got[:, t] = from_dev_f64(od)[:, 0]
            got_lse[:, :, t] = ld.cpu().numpy()
        assert duo.duo_cache_len(handle, 0) == total
    finally:
        duo.duo_cache_destroy(handle)
    for b in (range(batch) if check_batches is None else check_batches):
        want_o, want_lse = oracle_rows(cfg, q, k, v, np.arange(n_fill, total), b)
        assert_close(got[b], want_o, "batch %d" % b)
        assert np.abs(got_lse[b] - want_lse).max() <= ATOL_LSE


@pytest.mark.parametrize("d,kv_dtype", [(64, 0), (128, 0), (128, 1), (64, 2), (128, 2), (64, 3), (128, 3)])
def test_matrix_core_decode_kernel_with_one_query_head_per_kv_head(d, kv_dtype):
    # the matrix-core kernel forced onto an MHA layer (it pads the single head to 16 columns);
    # the context starts empty-ish, crosses the 32-row unit size and wraps the ring
    mask = np.array([1, 0, 1, 0], dtype=np.uint8)
    _decode_vs_oracle(4, 4, d, 5, 40, 2, 27, 45, kv_dtype, mask, kernel=1)
    _decode_vs_oracle(4, 4, d, 5, 40, 1, 0, 3, kv_dtype, mask, kernel=1)          # from an empty cache
    _decode_vs_oracle(4, 4, d, 5, 40, 1, 1500, 4, kv_dtype, mask, kernel=1, splits=7)


@pytest.mark.parametrize("kv_dtype", [0, 1, 2, 3])
def test_query_group_of_eight(kv_dtype):
    mask = np.array([0, 1], dtype=np.uint8)
    _decode_vs_oracle(16, 2, 128, 4, 28, 2, 333, 6, kv_dtype, mask)
    _decode_vs_oracle(16, 2, 64, 4, 28, 1, 95, 3, kv_dtype, mask, splits=3)


def test_decode_workgroups_that_cross_segment_borders():
    # more retrieval (sequence, head) segments than workgroups: every workgroup handles the end of
    # one segment and the start of the next, and whole segments in between
    mask = np.array([1, 0, 1, 1], dtype=np.uint8)
    _decode_vs_oracle(8, 4, 64, 3, 20, 120, 210, 2, 0, mask, check_batches=(0, 57, 119))


def test_all_streaming_and_all_retrieval_layers_on_the_matrix_core_kernel():
    for mask in (np.zeros(2, dtype=np.uint8), np.ones(2, dtype=np.uint8)):
        _decode_vs_oracle(8, 2, 128, 4, 16, 2, 150, 3, 0, mask)


@pytest.mark.parametrize("hq,hkv,d,sink,recent,chunks,batch", [
    (8, 8, 64, 16, 256, [700, 300, 1, 47, 1000], 1),      # configuration-1 constants, ragged chunks
    (8, 2, 128, 4, 32, [300, 1, 77, 130, 64], 2),         # GQA 4, window shorter than a tile
    (4, 4, 128, 64, 256, [129, 513, 200], 1),             # deployment constants
    (4, 2, 64, 0, 5, [70, 70, 3], 1),                     # no sinks
    (2, 2, 128, 1, 2, [4, 4, 4, 4], 1),                   # the figure's parameters
])
def test_deployed_chunk_causal_prefill(hq, hkv, d, sink, recent, chunks, batch):
    # duo_attn_prefill_deployed: streaming heads see [retained cache || chunk] causally; the result
    # depends on the chunk starts, which the oracle is given per position
    total = sum(chunks)
    mask = np.array([(h % 2) for h in range(hkv)], dtype=np.uint8)
    cfg = dict(batch=batch, hq=hq, hkv=hkv, d=d, sink=sink, recent=recent, mask=mask, max_seq=total + 4)
    q, k, v = make_qkv(hq * 10 + d + recent, batch, total + 4, hq, hkv, d)
    out, lse, handle = run_scenario(duo, cfg, q, k, v, chunks, 4, deployed=True)
    duo.duo_cache_destroy(handle)
    starts = np.concatenate([np.full(n, p) for p, n in zip(np.cumsum([0] + chunks[:-1]), chunks)])
    for b in range(batch):
        want_o, want_lse = oracle_rows(cfg, q, k, v, np.arange(total), b, chunk_starts=starts)
        assert_close(synth.bf16_bits_to_f64(out[b][:total]), want_o, "deployed prefill, batch %d" % b)
        assert np.abs(lse[b][:, :total] - want_lse).max() <= ATOL_LSE
        # the decode steps after it see the ordinary cache contents
        want_d, _ = oracle_rows(cfg, q, k, v, np.arange(total, total + 4), b)
        assert_close(synth.bf16_bits_to_f64(out[b][total:]), want_d, "decode after deployed prefill")


@pytest.mark.parametrize("kv_dtype", [1, 2, 3])
@pytest.mark.parametrize("hq,hkv,d,sink,recent,chunks,batch,deployed", [
    (8, 2, 128, 4, 32, [300, 1, 77, 130], 2, False),     # GQA 4, ragged chunks
    (4, 4, 64, 16, 64, [129, 513, 64], 1, False),        # head_dim 64, tile tails
    (8, 8, 128, 64, 256, [700, 300], 1, True),           # deployment constants, chunk-causal streaming heads
])
def test_prefill_over_a_quantised_cache(hq, hkv, d, sink, recent, chunks, batch, deployed, kv_dtype):
    # cached positions are seen through the codec (as the cache holds them), the chunk's own positions
    # as given; the decode steps afterwards see every position through the codec
    total, n_decode = sum(chunks), 3
    mask = np.array([(h + 1) % 2 for h in range(hkv)], dtype=np.uint8)
    cfg = dict(batch=batch, hq=hq, hkv=hkv, d=d, sink=sink, recent=recent, mask=mask, max_seq=total + n_decode,
               kv_dtype=kv_dtype)
    q, k, v = make_qkv(77 + kv_dtype, batch, total + n_decode, hq, hkv, d)
    out, lse, handle = run_scenario(duo, cfg, q, k, v, chunks, n_decode, deployed=deployed, fused_decode="step")
    duo.duo_cache_destroy(handle)
    from helpers import ATOL_LSE_IMAGE, oracle_kv
    for b in range(batch):
        kq, vq = oracle_kv(k[b], v[b], kv_dtype)          # every position through the codec, float64
        # the library's pre-filling reads the cached rows from a bf16 image of these values
        ki, vi = (synth.bf16_bits_to_f64(synth.f32_to_bf16_bits(x.astype(np.float32))) for x in (kq, vq))
        kf, vf = synth.bf16_bits_to_f64(k[b]), synth.bf16_bits_to_f64(v[b])
        p0 = 0
        for n in chunks:
            pos = np.arange(p0, p0 + n)
            qf = synth.bf16_bits_to_f64(q[b][pos])
            starts = np.full(n, p0) if deployed else None
            # the definition: float64 attention over the codec's exact output for the cached positions
            want_o, want_lse = oracle.attention_rows(qf, np.concatenate([kq[:p0], kf[p0:p0 + n]]),
                                                     np.concatenate([vq[:p0], vf[p0:p0 + n]]), pos, mask, sink,
                                                     recent, None, chunk_starts=starts)
            assert_close(synth.bf16_bits_to_f64(out[b][pos]), want_o, "chunk at %d, batch %d" % (p0, b))
            assert np.abs(lse[b][:, pos] - want_lse).max() <= ATOL_LSE_IMAGE
            # secondary, tighter: against the same attention over the bf16-rounded image the kernel reads
            img_o, img_lse = oracle.attention_rows(qf, np.concatenate([ki[:p0], kf[p0:p0 + n]]),
                                                   np.concatenate([vi[:p0], vf[p0:p0 + n]]), pos, mask, sink,
                                                   recent, None, chunk_starts=starts)
            assert_close(synth.bf16_bits_to_f64(out[b][pos]), img_o, "chunk at %d, batch %d (image)" % (p0, b))
            assert np.abs(lse[b][:, pos] - img_lse).max() <= ATOL_LSE
            p0 += n
        want_d, _ = oracle_rows(cfg, q, k, v, np.arange(total, total + n_decode), b)
        assert_close(synth.bf16_bits_to_f64(out[b][total:]), want_d, "decode after the quantised prefill")
