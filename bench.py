#!/usr/bin/env python3
"""Benchmark of the DuoAttention hot path on one MI355X.  Prints ONE JSON line.

Default (no --workload): the suite.  The headline - `value`, `config`, `roofline`, `cpu_baseline`, and the
K steps that --steps / --warmup count - is the largest single-GPU decode configuration: a
Llama-3-8B-shaped stack of 32 attention layers (32 query / 8 KV heads x 128, half of the KV heads
retrieval per layer, 64 sink + 256 recent tokens) decoding at 3 300 000 tokens of context over an fp8
E4M3 KV cache with per-row fp32 scales (111.5 GB).  One "step" is one pass of the whole decode path over
one batch of synthetic input: 4 new tokens, each through all 32 layers (append to both caches + attention
over them, one launch per token and layer).  After it the other configurations run as short timed loops
of their own and are reported under `sub` (the 1M-token bf16 stack, the 3.3M-token 4-bit stack, the
128K-context GQA layer at batch 1 / 4 / 16 and through 32 distinct layers, the 32K-context MHA layer with
its chunked pre-filling and through 32 distinct layers), and `roofline_prefill` is the 128K-token
pre-filling in 32K-token chunks.  All inputs are synthetic bf16 N(0,1) tensors generated on the device
before the timed regions.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]     (one workload alone, e.g. under rocprofv3)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM bytes per launch RECORDED from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of `bench.py --workload NAME`,
# scaled by a 1 GiB device copy (summaries under profiles/): constants of the build they were taken on, not
# measured by the run that prints them; known for these workloads only.
MEASURED_TRAFFIC = {"c2": {"decode": 139.06e6 + 0.17e6, "prefill": 165.4e6 + 33.6e6},
                    "c3_prefill": {"prefill": 2528.1e6 + 268.7e6},
                    "c3_decode_b1": {"decode": 270.34e6 + 0.60e6},
                    "c3_decode_b16": {"decode": 4307.9e6 + 0.65e6},
                    "c4": {"decode": 2149.3e6 + 0.6e6},
                    "c5": {"decode": 3549.4e6 + 0.6e6},
                    "c6": {"decode": 1917.4e6 + 0.6e6}}
HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 MFMA rate

WORKLOADS = {
    # name: (hq, hkv, d, ratio, sink, recent, prefill_tokens, chunk, decode_steps, batch, kv_dtype, append_only_fill)
    "c1": dict(hq=8, hkv=8, d=64, ratio=0.5, sink=16, recent=256, prefill=2048, chunk=2048, decode=64, batch=1,
               desc="toy MHA 8x64, prefill 2048 + 64 decode"),
    "c2": dict(hq=32, hkv=32, d=128, ratio=0.25, sink=64, recent=256, prefill=32768, chunk=4096, decode=256, batch=1,
               desc="Llama-2-7B-shaped MHA layer, 25% retrieval heads, sink 64, recent 256, "
                    "prefill 32768 in 4096-token chunks + 256 decode steps, batch 1"),
    "c3_prefill": dict(hq=32, hkv=8, d=128, ratio=0.5, sink=64, recent=256, prefill=131072, chunk=32768, decode=0,
                       batch=1, desc="Llama-3-8B-shaped GQA layer, 50% retrieval KV heads, prefill 131072 in "
                                     "32768-token chunks, batch 1"),
    "c3_decode_b1": dict(hq=32, hkv=8, d=128, ratio=0.5, sink=64, recent=256, prefill=131072, chunk=0, decode=64,
                         batch=1, desc="Llama-3-8B-shaped GQA layer decode at 131072 context, batch 1"),
    "c3_decode_b4": dict(hq=32, hkv=8, d=128, ratio=0.5, sink=64, recent=256, prefill=131072, chunk=0, decode=64,
                         batch=4, desc="Llama-3-8B-shaped GQA layer decode at 131072 context, batch 4"),
    "c3_decode_b16": dict(hq=32, hkv=8, d=128, ratio=0.5, sink=64, recent=256, prefill=131072, chunk=0, decode=32,
                          batch=16, desc="Llama-3-8B-shaped GQA layer decode at 131072 context, batch 16"),
    "c2_stack": dict(hq=32, hkv=32, d=128, ratio=0.25, sink=64, recent=256, prefill=32768, chunk=0, decode=16, batch=1,
                     layers=32, desc="Llama-2-7B-shaped MHA decode at 32768 context through 32 distinct layers "
                                     "(4.4 GB per token: beyond the memory-side cache), batch 1"),
    "c3_stack": dict(hq=32, hkv=8, d=128, ratio=0.5, sink=64, recent=256, prefill=131072, chunk=0, decode=16, batch=1,
                     layers=32, desc="Llama-3-8B-shaped GQA decode at 131072 context through 32 distinct layers "
                                     "(8.6 GB per token: beyond the memory-side cache), batch 1"),
    "c4": dict(hq=32, hkv=8, d=128, ratio=0.5, sink=64, recent=256, prefill=1 << 20, chunk=0, decode=4, batch=1,
               layers=32, desc="Llama-3-8B-shaped GQA decode at 1048576 context, 32 layers (attention op only), "
                               "bf16 KV, batch 1"),
    "c5": dict(hq=32, hkv=8, d=128, ratio=0.5, sink=64, recent=256, prefill=3300000, chunk=0, decode=4, batch=1,
               layers=32, kv_dtype=1, desc="Llama-3-8B-shaped GQA decode at 3300000 context, 32 layers, fp8 e4m3 KV "
                                           "+ fp32 scales per (token, KV head), batch 1"),
    "c6": dict(hq=32, hkv=8, d=128, ratio=0.5, sink=64, recent=256, prefill=3300000, chunk=0, decode=4, batch=1,
               layers=32, kv_dtype=2, desc="Llama-3-8B-shaped GQA decode at 3300000 context, 32 layers, 4-bit KV "
                                           "(asymmetric codes + fp32 scale and minimum per (token, KV head)), batch 1"),
}


def visible_pairs(pos0, n, sink, recent, retrieval):
    """Number of unmasked (query, key) pairs of a chunk of n queries starting at position pos0."""
    i = np.arange(pos0, pos0 + n, dtype=np.int64)
    if retrieval:
        return int((i + 1).sum())
    return int(np.minimum(i + 1, sink + recent).sum())


# the suite: (workload, steps, warmup) of the short loops reported under "sub"
HEADLINE = "c5"
SUITE = [("c3_prefill", 3, 1), ("c2", 10, 2), ("c4", 3, 1), ("c6", 3, 1), ("c3_decode_b1", 5, 2),
         ("c3_decode_b4", 5, 2), ("c3_decode_b16", 5, 2), ("c3_stack", 5, 2), ("c2_stack", 5, 2)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="suite", choices=["suite"] + sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--splits", type=int, default=0, help="key splits per retrieval head in decode (0 = automatic)")
    ap.add_argument("--sweep", default=None, choices=["decode_ratio", "decode_context", "prefill_chunk", "gate_mixed"],
                    help="instead of the benchmark line, print one JSON line per point of a sweep that mirrors "
                         "the shape of the paper's efficiency figures (latency against retrieval-head ratio, "
                         "context length, pre-filling chunk size), each with the all-retrieval (= full "
                         "attention) run through the same kernels beside it")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain 1 GiB device copy (reads 1 GiB, writes 1 GiB) so that rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings can be scaled by a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2410_10819_amd import binding as duo
    from paper_2410_10819_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    lib = duo.load()                      # raises if the HIP library is missing: no fallback
    if args.sweep:
        run_sweep(args.sweep, torch, duo, synth, lib, args.seed)
        return
    if args.workload != "suite":
        print(json.dumps(run_workload(args.workload, args, torch, duo, synth, lib, not args.no_cpu_baseline)))
        return
    result = run_workload(HEADLINE, args, torch, duo, synth, lib, not args.no_cpu_baseline)
    print("bench: headline %s done" % HEADLINE, file=sys.stderr, flush=True)
    sub = {}
    for name, steps, warmup in SUITE:
        sub_args = argparse.Namespace(**vars(args))
        sub_args.steps, sub_args.warmup = steps, warmup
        r = run_workload(name, sub_args, torch, duo, synth, lib, False)
        sub[name] = {"workload": r["config"]["workload"], "steps": steps, "warmup": warmup,
                     "ms_per_step": r["ms_per_step"], "dtype": r["dtype"],
                     "decode_us_per_token": r["value"] if r["unit"] == "us/token" else None,
                     "roofline_decode": r["roofline_decode"], "roofline_prefill": r["roofline_prefill"]}
        print("bench: %s done" % name, file=sys.stderr, flush=True)
    result["roofline_prefill"] = sub["c3_prefill"]["roofline_prefill"]
    result["prefill_tflops"] = result["roofline_prefill"]["achieved"]
    result["sub"] = sub
    print(json.dumps(result))


def run_workload(workload, args, torch, duo, synth, lib, with_cpu_baseline):
    """Time one workload: args.warmup untimed steps, then exactly args.steps timed steps; returns its record."""
    w = WORKLOADS[workload]
    hq, hkv, d, B = w["hq"], w["hkv"], w["d"], w["batch"]
    sink, recent = w["sink"], w["recent"]
    n_prefill, chunk, n_decode = w["prefill"], w["chunk"], w["decode"]
    n_layers, kv_dtype = w.get("layers", 1), w.get("kv_dtype", 0)
    group = hq // hkv
    attn_prefill = chunk > 0
    # with pre-filling attention a step starts from an empty cache; a decode-only workload fills its
    # caches once (by append alone) before the timed region and every step decodes n_decode more tokens
    n_dec_total = n_decode if attn_prefill else n_decode * (args.warmup + args.steps)
    total = n_prefill + n_dec_total
    mask = synth.retrieval_mask(args.seed, n_layers, hkv, w["ratio"])
    n_ret = int(mask[0].sum())
    n_str = hkv - n_ret
    stream = torch.cuda.current_stream().cuda_stream
    assert attn_prefill or n_decode > 0
    assert n_layers == 1 or not attn_prefill

    # ---- synthetic inputs, generated on the device (bit-identical to the CPU generator)
    table = torch.from_numpy(synth.normal_table_bf16().view(np.int16)).cuda()

    def fill(layer, tensor_id, heads, pos, n_pos):
        t = torch.empty((B, n_pos, heads, d), dtype=torch.bfloat16, device="cuda")
        for b in range(B):
            duo.duo_synth_fill_bf16(t[b], table, synth.stream_key(args.seed, layer, tensor_id, b), pos, n_pos,
                                    heads, d)
        return t

    handle = duo.duo_cache_create(n_layers, B, hq, hkv, d, sink, recent, total, mask, kv_dtype)
    if args.splits:
        duo.duo_set_decode_splits(handle, args.splits)
    P = lambda t: t.data_ptr()   # raw pointers: the timed loop does no Python-side tensor checks

    def check(rc):
        if rc != 0:
            raise duo.DuoError(rc, lib.duo_last_error().decode())

    chunks, keep = [], []
    if attn_prefill:
        q_all = fill(0, synth.TENSOR_Q, hq, 0, total)
        k_all = fill(0, synth.TENSOR_K, hkv, 0, total)
        v_all = fill(0, synth.TENSOR_V, hkv, 0, total)
        for p in range(0, n_prefill, chunk):
            n = min(chunk, n_prefill - p)
            qc, kc, vc = (t[:, p:p + n].contiguous() if B > 1 else t[:, p:p + n] for t in (q_all, k_all, v_all))
            keep.append((qc, kc, vc))
            chunks.append((p, n, P(qc), P(kc), P(vc)))
        dec_src = [(q_all[:, n_prefill:], k_all[:, n_prefill:], v_all[:, n_prefill:])]
    else:
        fill_chunk = 1 << 17
        for layer in range(n_layers):
            for p in range(0, n_prefill, fill_chunk):
                n = min(fill_chunk, n_prefill - p)
                kc, vc = fill(layer, synth.TENSOR_K, hkv, p, n), fill(layer, synth.TENSOR_V, hkv, p, n)
                duo.duo_kv_append(handle, layer, kc, vc, n)
            torch.cuda.synchronize()
        dec_src = [(fill(layer, synth.TENSOR_Q, hq, n_prefill, n_dec_total),
                    fill(layer, synth.TENSOR_K, hkv, n_prefill, n_dec_total),
                    fill(layer, synth.TENSOR_V, hkv, n_prefill, n_dec_total)) for layer in range(n_layers)]
    # decode-phase inputs as separate contiguous [B, 1, H, D] slices: dec_ptrs[token][layer]
    dec_ptrs = []
    for t in range(n_dec_total):
        per_layer = []
        for layer in range(n_layers):
            trio = tuple(x[:, t:t + 1].contiguous() for x in dec_src[layer])
            keep.append(trio)
            per_layer.append(tuple(P(x) for x in trio))
        dec_ptrs.append(per_layer)
    out_pre = torch.empty((B, max(chunk, 1), hq, d), dtype=torch.bfloat16, device="cuda")
    out_dec = torch.empty((B, 1, hq, d), dtype=torch.bfloat16, device="cuda")
    p_out_pre, p_out_dec = P(out_pre), P(out_dec)
    torch.cuda.synchronize()

    def prefill_phase():
        for _, n, pq, pk, pv in chunks:
            check(lib.duo_attn_prefill(handle, 0, pq, pk, pv, n, None, p_out_pre, None, stream))
            check(lib.duo_kv_append(handle, 0, pk, pv, n, None, stream))

    def decode_phase(first_token):
        # one launch per token and layer: duo_decode_step appends the token and attends
        for t in range(first_token, first_token + n_decode):
            for layer, (pq, pk, pv) in enumerate(dec_ptrs[t]):
                check(lib.duo_decode_step(handle, layer, pq, pk, pv, None, p_out_dec, None, stream))

    ev = lambda: torch.cuda.Event(enable_timing=True)
    pre_ms, dec_ms = [], []
    e0, e1, e2 = ev(), ev(), ev()
    step_no = [0]

    def one_step(timed):
        if attn_prefill:
            duo.duo_cache_reset(handle)
        if timed:
            e0.record()
        prefill_phase()
        if timed:
            e1.record()
        decode_phase(0 if attn_prefill else step_no[0] * n_decode)
        if timed:
            e2.record()
        step_no[0] += 1

    if args.calibrate:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        one_step(False)
    torch.cuda.synchronize()
    ctx_first = duo.duo_cache_len(handle, 0) if not attn_prefill else n_prefill
    t_start = time.perf_counter()
    for _ in range(args.steps):
        one_step(True)
        torch.cuda.synchronize()
        pre_ms.append(e0.elapsed_time(e1))
        dec_ms.append(e1.elapsed_time(e2))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps

    # ---- algorithmic work
    row_bytes = {0: 2 * d, 1: d + 4, 2: d // 2 + 8, 3: d + 8}[kv_dtype]
    n_timed_tokens = n_decode if attn_prefill else n_decode * args.steps
    dec_bytes = []           # per launch (one layer, one token, all sequences)
    for t in range(n_timed_tokens):
        n_ctx = ctx_first + t + 1
        dec_bytes.append(B * (n_ret * 2 * n_ctx * row_bytes + n_str * 2 * min(n_ctx, sink + recent) * row_bytes
                              + 2 * hq * d * 2))
    avg_dec_bytes = float(np.mean(dec_bytes)) if dec_bytes else 0.0
    flops = 0
    for p, n, *_ in chunks:
        pairs = group * B * (n_ret * visible_pairs(p, n, sink, recent, True)
                             + n_str * visible_pairs(p, n, sink, recent, False))
        flops += 4 * d * pairs
    pre_t = float(np.mean(pre_ms)) * 1e-3
    dec_t = float(np.mean(dec_ms)) * 1e-3
    us_per_token = dec_t / n_decode * 1e6 if n_decode else None
    # events bracket the back-to-back launches of the phase: average time per launch, launch gaps
    # included (the kernel-only figure is in the rocprofv3 summary)
    dec_call_us = dec_t / (n_decode * n_layers) * 1e6 if n_decode else None
    dec_gbps = avg_dec_bytes / (dec_call_us * 1e-6) / 1e9 if dec_call_us else None
    pre_tflops = flops / pre_t / 1e12 if attn_prefill and pre_t > 0 else None

    roof_dec = None
    if dec_gbps:
        roof_dec = {"bound": "hbm", "achieved": round(dec_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(dec_gbps / HBM_PEAK_GBPS, 4),
                    "traffic": MEASURED_TRAFFIC.get(workload, {}).get("decode"),
                    "traffic_source": "recorded constant: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary under profiles/",
                    "kernel": "duo::decode_kernel" if (group == 1 and not kv_dtype) else "duo::decode_sk_kernel",
                    "bytes_per_launch": int(avg_dec_bytes),
                    "avg_launch_us": round(dec_call_us, 2)}
    roof_pre = None
    if pre_tflops:
        roof_pre = {"bound": "mfma", "achieved": round(pre_tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(pre_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                    "traffic": MEASURED_TRAFFIC.get(workload, {}).get("prefill"),
                    "traffic_source": "recorded constant: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary under profiles/",
                    "kernel": "duo::prefill_kernel", "flops_per_step": int(flops),
                    "avg_chunk_ms": round(pre_t * 1e3 / max(len(chunks), 1), 3)}
    dominant = roof_dec if (roof_pre is None or (roof_dec is not None and dec_t >= pre_t)) else roof_pre

    # ---- the oracle on the host cores, bounded sample of the same workload
    cpu = None
    if with_cpu_baseline and n_decode:
        cpu = cpu_baseline(synth, args.seed, w, mask, n_prefill, B)

    result = {
        "metric": "decode_attn_us_per_token" if n_decode else "prefill_attn_tflops",
        "value": round(us_per_token, 3) if n_decode else round(pre_tflops, 2),
        "unit": "us/token" if n_decode else "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": False if n_decode else True, "scaling": "weak", "vs_baseline": None,
        "dtype": {0: "bf16", 1: "bf16 (fp8 e4m3 KV, fp32 accumulate)",
                  2: "bf16 (int4 KV, fp32 accumulate)", 3: "bf16 (int8 KV, fp32 accumulate)"}[kv_dtype], "data": "synthetic",
        "config": {"workload": w["desc"], "name": workload, "n_layers": n_layers, "n_q_heads": hq,
                   "n_kv_heads": hkv, "head_dim": d, "retrieval_kv_heads": n_ret, "sink": sink, "recent": recent,
                   "batch": B, "prefill_tokens": n_prefill, "chunk": chunk, "decode_steps": n_decode,
                   "cache_bytes": duo.duo_cache_bytes(handle)},
        "decode_hbm_GBps": round(dec_gbps, 1) if dec_gbps else None,
        "decode_call_us": round(dec_call_us, 2) if dec_call_us else None,
        "prefill_tflops": round(pre_tflops, 1) if pre_tflops else None,
        "prefill_ms": round(pre_t * 1e3, 3), "decode_ms": round(dec_t * 1e3, 3),
        "roofline": dominant, "roofline_decode": roof_dec, "roofline_prefill": roof_pre,
        "cpu_baseline": cpu,
    }
    duo.duo_cache_destroy(handle)
    del keep, dec_ptrs, dec_src, chunks, out_pre, out_dec, table
    torch.cuda.empty_cache()
    return result


def run_sweep(name, torch, duo, synth, lib, seed):
    """Latency sweeps on synthetic layers of the paper's two shapes (Section 3.4 and its figures on decoding
    and pre-filling efficiency): MHA = 32 heads x 128 (Llama-2-7B-shaped), GQA = 32 query / 8 KV heads x 128
    (Llama-3-8B-shaped); sink 64, recent 256.  Every point is also run with all heads retrieval, which is
    full attention through the same kernels, and the ratio of the two times is reported."""
    sink, recent, d = 64, 256, 128
    table = torch.from_numpy(synth.normal_table_bf16().view(np.int16)).cuda()
    stream = torch.cuda.current_stream().cuda_stream

    def fill(tensor_id, heads, pos, n_pos):
        t = torch.empty((1, n_pos, heads, d), dtype=torch.bfloat16, device="cuda")
        duo.duo_synth_fill_bf16(t[0], table, synth.stream_key(seed, 0, tensor_id, 0), pos, n_pos, heads, d)
        return t

    def timed(fn, iters):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    def decode_us(hq, hkv, n_ret, n_ctx):
        mask = np.zeros((1, hkv), dtype=np.uint8)
        mask[0, np.random.default_rng(seed).permutation(hkv)[:n_ret]] = 1
        h = duo.duo_cache_create(1, 1, hq, hkv, d, sink, recent, n_ctx + 1, mask)
        for p in range(0, n_ctx, 1 << 16):
            n = min(1 << 16, n_ctx - p)
            duo.duo_kv_append(h, 0, fill(synth.TENSOR_K, hkv, p, n), fill(synth.TENSOR_V, hkv, p, n), n)
        q = fill(synth.TENSOR_Q, hq, n_ctx, 1)
        o = torch.empty_like(q)
        ms = timed(lambda: lib.duo_attn_decode(h, 0, q.data_ptr(), None, None, None, o.data_ptr(), None, stream), 50)
        duo.duo_cache_destroy(h)
        return ms * 1e3

    def prefill_ms(hq, hkv, n_ret, n_ctx, chunk, deployed=False):
        call = lib.duo_attn_prefill_deployed if deployed else lib.duo_attn_prefill
        mask = np.zeros((1, hkv), dtype=np.uint8)
        mask[0, np.random.default_rng(seed).permutation(hkv)[:n_ret]] = 1
        h = duo.duo_cache_create(1, 1, hq, hkv, d, sink, recent, n_ctx, mask)
        out = torch.empty((1, chunk, hq, d), dtype=torch.bfloat16, device="cuda")
        total = 0.0
        for p in range(0, n_ctx, chunk):
            n = min(chunk, n_ctx - p)
            q, k, v = fill(synth.TENSOR_Q, hq, p, n), fill(synth.TENSOR_K, hkv, p, n), fill(synth.TENSOR_V, hkv, p, n)
            total += timed(lambda: call(h, 0, q.data_ptr(), k.data_ptr(), v.data_ptr(), n, None, out.data_ptr(), None,
                                        stream), 1)
            duo.duo_kv_append(h, 0, k, v, n)
        duo.duo_cache_destroy(h)
        return total

    shapes = {"mha": (32, 32), "gqa": (32, 8)}
    if name == "decode_ratio":
        for shape, n_ctx in (("mha", 32768), ("gqa", 131072)):
            hq, hkv = shapes[shape]
            full = decode_us(hq, hkv, hkv, n_ctx)
            for n_ret in sorted({0, hkv // 8, hkv // 4, 3 * hkv // 8, hkv // 2, 3 * hkv // 4, hkv}):
                us = full if n_ret == hkv else decode_us(hq, hkv, n_ret, n_ctx)
                print(json.dumps({"sweep": name, "shape": shape, "context": n_ctx, "retrieval_ratio": n_ret / hkv,
                                  "decode_us": round(us, 2), "full_attention_us": round(full, 2),
                                  "speedup_vs_full": round(full / us, 3)}), flush=True)
    elif name == "decode_context":
        for shape, n_ret, ctxs in (("mha", 8, (8192, 16384, 32768, 65536, 131072, 262144)),
                                   ("gqa", 4, (32768, 131072, 524288, 1048576))):
            hq, hkv = shapes[shape]
            for n_ctx in ctxs:
                us, full = decode_us(hq, hkv, n_ret, n_ctx), decode_us(hq, hkv, hkv, n_ctx)
                print(json.dumps({"sweep": name, "shape": shape, "context": n_ctx, "retrieval_ratio": n_ret / hkv,
                                  "decode_us": round(us, 2), "full_attention_us": round(full, 2),
                                  "speedup_vs_full": round(full / us, 3)}), flush=True)
    elif name == "gate_mixed":
        # identification-phase forward (Section 2.2): alpha * full + (1 - alpha) * streaming over whole
        # sequences of the training lengths (appendix, Training Hyperparameters), sink 128 / recent 256 as in
        # Section 3.1, the streaming term with the Lambda mask and with the block-aligned mask (block 128)
        g_sink, g_recent = 128, 256
        for shape, lengths in (("mha", (4096, 32000)), ("gqa", (8192, 32000))):
            hq, hkv = shapes[shape]
            alpha = np.random.default_rng(seed).uniform(0, 1, hkv).astype(np.float32)
            h = duo.duo_cache_create(1, 1, hq, hkv, d, g_sink, g_recent, 64, np.ones((1, hkv), dtype=np.uint8))
            for n in lengths:
                q, k, v = fill(synth.TENSOR_Q, hq, 0, n), fill(synth.TENSOR_K, hkv, 0, n), fill(synth.TENSOR_V, hkv, 0, n)
                out = torch.empty_like(q)
                full_pairs = hq * n * (n + 1) // 2
                for block in (0, 128):
                    ms = timed(lambda: duo.duo_attn_gate_mixed(h, 0, q, k, v, n, alpha, out, block=block), 3)
                    if block:
                        n_sb, n_lb = -(-g_sink // block), -(-(g_recent - 1) // block) + 1
                        i = np.arange(n, dtype=np.int64)
                        vis = np.minimum(i + 1, np.minimum(n_sb * block, i + 1)
                                         + np.maximum(0, i + 1 - np.maximum((i // block - n_lb + 1) * block,
                                                                             np.minimum(n_sb * block, i + 1))))
                        str_pairs = hq * int(vis.sum())
                    else:
                        str_pairs = hq * visible_pairs(0, n, g_sink, g_recent, False)
                    # the streaming term's keys are a subset of the causal ones and the library computes every
                    # score once: `tflops` counts the causal pairs only, `tflops_two_terms` what two separate
                    # attentions (full, then streaming) would have to compute
                    print(json.dumps({"sweep": name, "shape": shape, "tokens": n, "block": block,
                                      "gate_mixed_ms": round(ms, 3),
                                      "tflops": round(4 * d * full_pairs / ms / 1e9, 1),
                                      "tflops_two_terms": round(4 * d * (full_pairs + str_pairs) / ms / 1e9, 1),
                                      "streaming_share_of_pairs": round(str_pairs / full_pairs, 4)}),
                          flush=True)
            duo.duo_cache_destroy(h)
    else:
        for shape, n_ret, n_ctx, chunks in (("mha", 8, 102400, (4096, 8192, 16384, 32768, 102400)),
                                            ("gqa", 4, 327680, (16384, 32768, 65536, 163840))):
            hq, hkv = shapes[shape]
            for chunk in chunks:
                ms, full = prefill_ms(hq, hkv, n_ret, n_ctx, chunk), prefill_ms(hq, hkv, hkv, n_ctx, chunk)
                dep = prefill_ms(hq, hkv, n_ret, n_ctx, chunk, deployed=True)
                print(json.dumps({"sweep": name, "shape": shape, "context": n_ctx, "chunk": chunk,
                                  "retrieval_ratio": n_ret / hkv, "prefill_ms": round(ms, 2),
                                  "deployed_chunk_causal_ms": round(dep, 2), "full_attention_ms": round(full, 2),
                                  "speedup_vs_full": round(full / ms, 3),
                                  "deployed_speedup_vs_full": round(full / dep, 3)}), flush=True)


def cpu_baseline(synth, seed, w, mask, n_ctx, batch):
    """Time the float64 oracle (as it stands) on the host cores for a bounded sample of decode tokens:
    whole tokens of sequence 0 for a one-layer workload; for the layer stacks one retrieval KV group of
    layer 0, scaled by the number of retrieval KV groups of all layers (a streaming group costs
    (sink + recent) / context of that, which is left out)."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    hq, hkv, d, sink, recent = w["hq"], w["hkv"], w["d"], w["sink"], w["recent"]
    n_layers, kv_dtype = w.get("layers", 1), w.get("kv_dtype", 0)
    group = hq // hkv
    n_sample = 4 if n_ctx <= 40000 else 1
    t_hist = n_ctx + n_sample
    whole = n_layers == 1
    heads = list(range(hkv)) if whole else [int(np.flatnonzero(mask[0] == 1)[0])]

    def history(tensor_id):
        out = np.empty((t_hist, len(heads), d), dtype=np.uint16)
        step = 1 << 15

        def job(p0):
            n = min(step, t_hist - p0)
            out[p0:p0 + n] = synth.counter_bf16(seed, 0, tensor_id, 0, p0, n, hkv, d, heads=heads)

        with ThreadPoolExecutor(8) as pool:
            list(pool.map(job, range(0, t_hist, step)))
        if not kv_dtype:
            return synth.bf16_bits_to_f64(out)
        deq = np.empty(out.shape, dtype=np.float64)
        qstep = 1 << 14

        def qjob(p0):
            x = synth.bf16_bits_to_f32(out[p0:p0 + qstep])
            if kv_dtype == 2:
                deq[p0:p0 + qstep] = oracle.dequantize_rows_int4(*oracle.quantize_rows_int4(x))
            elif kv_dtype == 3:
                deq[p0:p0 + qstep] = oracle.dequantize_rows_int8(*oracle.quantize_rows_int8(x))
            else:
                codes, scales = oracle.quantize_rows(x)
                deq[p0:p0 + qstep] = oracle.dequantize_rows(codes, scales)

        with ThreadPoolExecutor(8) as pool:
            list(pool.map(qjob, range(0, t_hist, qstep)))
        return deq

    kh, vh = history(synth.TENSOR_K), history(synth.TENSOR_V)
    q_heads = slice(0, hq) if whole else slice(heads[0] * group, (heads[0] + 1) * group)
    qh = synth.bf16_bits_to_f64(synth.counter_bf16(seed, 0, synth.TENSOR_Q, 0, n_ctx, n_sample, hq, d))[:, q_heads]
    sub_mask = mask[0] if whole else np.array([1], dtype=np.uint8)

    def timed_tokens():
        t0 = time.perf_counter()
        for t in range(n_sample):
            oracle.decode_step(qh[t], kh[:n_ctx + t + 1], vh[:n_ctx + t + 1], sub_mask, sink, recent)
        return (time.perf_counter() - t0) / n_sample

    # the oracle as it stands, (a) with the numerical library's threads limited to one, (b) with all of them
    from threadpoolctl import threadpool_info, threadpool_limits
    with threadpool_limits(limits=1):
        cpu_s_one = timed_tokens()
    cpu_s = timed_tokens()
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    if whole:
        factor, what = batch, "%d decode tokens of sequence 0 at context %d, scaled by batch %d" % (
            n_sample, n_ctx, batch)
    else:
        n_groups = int(mask.sum())
        factor, what = n_groups * batch, ("one retrieval KV group (%d query heads) of layer 0 for one token at "
                                          "context %d, scaled by the %d retrieval KV groups of the %d layers"
                                          % (group, n_ctx, n_groups, n_layers))
    return {"value": round(cpu_s * factor * 1e6, 1), "unit": "us/token", "cores": int(threads), "kind": "oracle",
            "one_thread": {"value": round(cpu_s_one * factor * 1e6, 1), "unit": "us/token", "cores": 1},
            "host_cores_available": len(os.sched_getaffinity(0)),
            "sample": what + " (float64 numpy oracle; inputs regenerated on the CPU, not timed)"}


if __name__ == "__main__":
    main()
