"""Shared helpers of the GPU parity tests: input staging and the scenario runner."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2410_10819_amd import synth

ATOL_MAX = 2e-2     # max-abs bound on bf16 attention outputs vs the float64 oracle
ATOL_MEAN = 2e-3    # mean-abs bound
# log-sum-exp: the kernels form the scores with fp32 accumulation of exact bf16 products and sum the
# unrounded fp32 probabilities, so the error is fp32 noise on numbers of order 10 plus the hardware
# exp2 / log2 approximations (about 1e-5 in all); 1e-3 absolute
ATOL_LSE = 1e-3
# pre-filling over a QUANTISED cache reads the cached rows from a bf16 image of code * scale (+ lo):
# every cached key is off by a relative rounding error <= 2^-9 (uniform, standard deviation 2^-9 / sqrt(3)
# = 1.1e-3), so a score of head_dim products of unit-variance factors, scaled by 1/sqrt(head_dim), is off
# by about 1.1e-3 (standard deviation) and the log-sum-exp, a softmax-weighted mean of the score errors, by
# at most that: four standard deviations on top of ATOL_LSE
ATOL_LSE_IMAGE = 1e-3 + 4.5e-3


def to_dev(bits: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def from_dev_bits(t) -> np.ndarray:
    import torch
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def from_dev_f64(t) -> np.ndarray:
    return synth.bf16_bits_to_f64(from_dev_bits(t))


def make_qkv(seed, batch, n_tok, hq, hkv, d, generator="counter", layer=0):
    """bf16 bit patterns q [B,T,Hq,D], k, v [B,T,Hkv,D]."""
    if generator == "counter":
        q = synth.counter_bf16_batch(seed, layer, synth.TENSOR_Q, batch, 0, n_tok, hq, d)
        k = synth.counter_bf16_batch(seed, layer, synth.TENSOR_K, batch, 0, n_tok, hkv, d)
        v = synth.counter_bf16_batch(seed, layer, synth.TENSOR_V, batch, 0, n_tok, hkv, d)
    else:
        rng = np.random.default_rng(seed)
        q = synth.randn_bf16(rng, (batch, n_tok, hq, d))
        k = synth.randn_bf16(rng, (batch, n_tok, hkv, d))
        v = synth.randn_bf16(rng, (batch, n_tok, hkv, d))
    return q, k, v


def assert_close(got_f64, want_f64, what=""):
    diff = np.abs(got_f64 - want_f64)
    assert np.isfinite(got_f64).all(), "%s: non-finite output" % what
    assert diff.max() <= ATOL_MAX, "%s: max-abs %.4g > %.4g" % (what, diff.max(), ATOL_MAX)
    assert diff.mean() <= ATOL_MEAN, "%s: mean-abs %.4g > %.4g" % (what, diff.mean(), ATOL_MEAN)
    return diff.max(), diff.mean()


def oracle_kv(k_bits, v_bits, kv_dtype):
    """float64 K/V history the oracle attends over (after the fp8 (1) or int4 (2) codec if enabled)."""
    k = synth.bf16_bits_to_f64(k_bits)
    v = synth.bf16_bits_to_f64(v_bits)
    if kv_dtype == 1:
        kc, ks = oracle.quantize_rows(k.astype(np.float32))
        vc, vs = oracle.quantize_rows(v.astype(np.float32))
        k, v = oracle.dequantize_rows(kc, ks), oracle.dequantize_rows(vc, vs)
    elif kv_dtype == 2:
        k = oracle.dequantize_rows_int4(*oracle.quantize_rows_int4(k.astype(np.float32)))
        v = oracle.dequantize_rows_int4(*oracle.quantize_rows_int4(v.astype(np.float32)))
    elif kv_dtype == 3:
        k = oracle.dequantize_rows_int8(*oracle.quantize_rows_int8(k.astype(np.float32)))
        v = oracle.dequantize_rows_int8(*oracle.quantize_rows_int8(v.astype(np.float32)))
    return k, v


def run_scenario(duo, cfg, q_bits, k_bits, v_bits, chunks, n_decode, fused_decode=False, want_lse=True,
                 pass_params=False, deployed=False):
    """Drive the library: prefill+append per chunk, then n_decode decode steps.

    cfg: dict(batch, hq, hkv, d, sink, recent, mask [hkv], max_seq, kv_dtype, scale)
    Returns (out_bits [B,T,Hq,D], lse [B,Hq,T], handle) with T = sum(chunks) + n_decode.
    """
    import torch
    b, hq, hkv, d = cfg["batch"], cfg["hq"], cfg["hkv"], cfg["d"]
    total = sum(chunks) + n_decode
    assert q_bits.shape == (b, total, hq, d)
    handle = duo.duo_cache_create(1, b, hq, hkv, d, cfg["sink"], cfg["recent"], cfg["max_seq"],
                                  np.asarray(cfg["mask"], dtype=np.uint8)[None], cfg.get("kv_dtype", 0),
                                  cfg.get("scale", 0.0))
    params = (np.asarray(cfg["mask"], dtype=np.uint8), cfg["sink"], cfg["recent"]) if pass_params else None
    out = np.zeros((b, total, hq, d), dtype=np.uint16)
    lse = np.zeros((b, hq, total), dtype=np.float64)
    pos = 0
    for n in chunks:
        qd, kd, vd = (to_dev(x[:, pos:pos + n]) for x in (q_bits, k_bits, v_bits))
        od = torch.empty((b, n, hq, d), dtype=torch.bfloat16, device="cuda")
        ld = torch.empty((b, hq, n), dtype=torch.float32, device="cuda") if want_lse else None
        (duo.duo_attn_prefill_deployed if deployed else duo.duo_attn_prefill)(handle, 0, qd, kd, vd, n, od, lse=ld,
                                                                              params=params)
        duo.duo_kv_append(handle, 0, kd, vd, n, params=params)
        torch.cuda.synchronize()
        out[:, pos:pos + n] = from_dev_bits(od)
        if want_lse:
            lse[:, :, pos:pos + n] = ld.cpu().numpy()
        pos += n
        assert duo.duo_cache_len(handle, 0) == pos
    for _ in range(n_decode):
        qd, kd, vd = (to_dev(x[:, pos:pos + 1]) for x in (q_bits, k_bits, v_bits))
        od = torch.empty((b, 1, hq, d), dtype=torch.bfloat16, device="cuda")
        ld = torch.empty((b, hq), dtype=torch.float32, device="cuda") if want_lse else None
        if fused_decode == "step":
            duo.duo_decode_step(handle, 0, qd, kd, vd, od, lse=ld, params=params)
        elif fused_decode:
            duo.duo_attn_decode(handle, 0, qd, od, k=kd, v=vd, lse=ld, params=params)
            duo.duo_kv_append(handle, 0, kd, vd, 1, params=params)
        else:
            duo.duo_kv_append(handle, 0, kd, vd, 1, params=params)
            duo.duo_attn_decode(handle, 0, qd, od, lse=ld, params=params)
        torch.cuda.synchronize()
        assert duo.duo_cache_len(handle, 0) == pos + 1
        out[:, pos] = from_dev_bits(od)[:, 0]
        if want_lse:
            lse[:, :, pos] = ld.cpu().numpy()
        pos += 1
    return out, lse, handle


def oracle_rows(cfg, q_bits, k_bits, v_bits, positions, batch_idx=0, chunk_starts=None):
    """Oracle output/lse of the given positions of one sequence: (o [n,Hq,D], lse [Hq,n]).
    chunk_starts (one per position) selects the deployed chunk-causal streaming attention."""
    kf, vf = oracle_kv(k_bits[batch_idx], v_bits[batch_idx], int(cfg.get("kv_dtype", 0)))
    qf = synth.bf16_bits_to_f64(q_bits[batch_idx][np.asarray(positions)])
    scale = cfg.get("scale", 0.0) or None
    return oracle.attention_rows(qf, kf, vf, positions, cfg["mask"], cfg["sink"], cfg["recent"], scale,
                                 chunk_starts=chunk_starts)


# ---- full-size cases: inputs generated on the device, the CPU regenerates the slices it checks

def device_table():
    import torch
    return torch.from_numpy(synth.normal_table_bf16().view(np.int16)).cuda()


def device_fill(table, seed, layer, tensor, batch, pos_start, n_pos, heads, d):
    """bf16 [batch, n_pos, heads, d] on the device: the counter generator's bits."""
    import torch
    from paper_2410_10819_amd import binding as duo
    t = torch.empty((batch, n_pos, heads, d), dtype=torch.bfloat16, device="cuda")
    for b in range(batch):
        duo.duo_synth_fill_bf16(t[b], table, synth.stream_key(seed, layer, tensor, b), pos_start, n_pos, heads, d)
    return t


def fill_cache_by_append(duo, handle, table, seed, layer, batch, hkv, d, n_tokens, chunk=65536):
    """Append positions 0 .. n_tokens-1 of the seeded K/V streams of `layer` to the cache."""
    for p in range(0, n_tokens, chunk):
        n = min(chunk, n_tokens - p)
        k = device_fill(table, seed, layer, synth.TENSOR_K, batch, p, n, hkv, d)
        v = device_fill(table, seed, layer, synth.TENSOR_V, batch, p, n, hkv, d)
        duo.duo_kv_append(handle, layer, k, v, n)


def cpu_history_bits(seed, layer, tensor, batch_idx, n_tokens, n_heads, d, heads=None, workers=8):
    """bf16 bits [n_tokens, len(heads), d] of one sequence, regenerated on the CPU in parallel blocks."""
    sel = list(range(n_heads)) if heads is None else list(heads)
    out = np.empty((n_tokens, len(sel), d), dtype=np.uint16)
    step = 1 << 15

    def job(p0):
        n = min(step, n_tokens - p0)
        out[p0:p0 + n] = synth.counter_bf16(seed, layer, tensor, batch_idx, p0, n, n_heads, d, heads=sel)

    synth.normal_table_bf16()
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(workers) as pool:
        list(pool.map(job, range(0, n_tokens, step)))
    return out


def oracle_history_f64(bits, kv_dtype, workers=8):
    """float64 history the oracle attends over: the bf16 values, or their round trip through the
    oracle's fp8 (1) or int4 (2) codec (applied block by block; each row is coded independently)."""
    kv_dtype = int(kv_dtype)
    if not kv_dtype:
        return synth.bf16_bits_to_f64(bits)
    out = np.empty(bits.shape, dtype=np.float64)
    step = 1 << 14

    def job(p0):
        x = synth.bf16_bits_to_f32(bits[p0:p0 + step])
        if kv_dtype == 2:
            out[p0:p0 + step] = oracle.dequantize_rows_int4(*oracle.quantize_rows_int4(x))
        elif kv_dtype == 3:
            out[p0:p0 + step] = oracle.dequantize_rows_int8(*oracle.quantize_rows_int8(x))
        else:
            codes, scales = oracle.quantize_rows(x)
            out[p0:p0 + step] = oracle.dequantize_rows(codes, scales)

    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(workers) as pool:
        list(pool.map(job, range(0, bits.shape[0], step)))
    return out
