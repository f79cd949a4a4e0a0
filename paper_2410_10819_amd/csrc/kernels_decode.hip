// Decode attention on the vector unit: one query per sequence against the split KV
// cache (paper, Section 2.3, Decoding; attention definitions of Section 2.2).
// This kernel serves one query head per KV head on a bf16 cache; query groups and
// quantised caches go to the matrix-core kernel in kernels_decode_sk.hip, which
// handles them with far fewer instructions per byte.
//
// The step is bound by HBM bandwidth: every cached K and V row of a retrieval
// head is read once per token, while a streaming head reads at most
// sink + recent rows.  Work decomposition:
//   - one work item (workgroup) per (sequence, retrieval KV head, key split) and
//     one per (sequence, streaming KV head);
//   - inside an item the head_dim/8 lanes of a "row group" each own one 16-byte
//     piece of a row, so a wavefront load covers 1 KiB of consecutive cache
//     memory; two register buffers of loads alternate, the next one being issued
//     before the current one is consumed, and the very first loads go out before
//     the query is read; each row group keeps its own running (max, sum, output)
//     softmax state, merged once at the end of the item;
//   - the split partials of a head are merged by the last workgroup of that head
//     to finish (an integer ticket per head decides who is last; the merge order
//     is fixed, so results are deterministic) - one launch per token;
//   - optionally the same launch writes the new token's K/V rows into the caches
//     (append fused into the step).
#include "duo_internal.h"

namespace duo {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ inline uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Cache rows are read once per launch: non-temporal loads stream them past the caches, which on
// this part moves a plain read of a large buffer from 6.3 to 7.1 TB/s (stand-alone probe).  Every
// wavefront load of this kernel covers 1 KiB of consecutive memory, whole cache lines.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ inline uint4 stream_load16(const void* p) {
  const u32x4_t x = __builtin_nontemporal_load((const u32x4_t*)p);
  return make_uint4(x[0], x[1], x[2], x[3]);
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Load of a table entry whose address is the same for the whole workgroup and
// whose memory no kernel writes: through the constant address space, i.e. the
// scalar unit, so the dependent address arithmetic does not wait for a vector load.
__device__ inline int uniform_load(const int32_t* p) {
  return *(const __attribute__((address_space(4))) int32_t*)(uintptr_t)p;
}

// Device-scope accesses for data exchanged between workgroups inside one launch.
__device__ inline void coherent_store(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Their counterpart: device-scope loads are served from the memory side of the per-die L2
// caches, so what another die stored this way is seen without invalidating a cache first.
__device__ inline float2 coherent_load2(const float2* p) {
  const uint64_t v = __hip_atomic_load((const uint64_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((uint32_t)v), __uint_as_float((uint32_t)(v >> 32)));
}
__device__ inline float4 coherent_load4(const float4* p) {
  const float2 lo = coherent_load2((const float2*)p), hi = coherent_load2((const float2*)p + 1);
  return make_float4(lo.x, lo.y, hi.x, hi.y);
}


// Sum over the LPR adjacent lanes of a row group with DPP cross-lane moves
// (quad permutes, then half-row and row mirrors: every lane of an already
// reduced sub-group holds the same value, so a mirror acts as an exchange).
template <int LPR>
__device__ inline float group_sum(float x) {
  static_assert(LPR == 4 || LPR == 8 || LPR == 16, "row group width");
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));
  if constexpr (LPR >= 8)
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));
  if constexpr (LPR >= 16)
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));
  return x;
}
// Widen one 16-byte piece of a row (8 bf16 values) to floats.
__device__ inline void widen(const uint4& c, float (&f)[8]) {
  const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) { f[2 * i] = bf16_lo(w[i]); f[2 * i + 1] = bf16_hi(w[i]); }
}

template <int D>
__global__ __launch_bounds__(256) void decode_kernel(DecodeArgs a) {
  constexpr int LPR = D / 8;           // lanes per row (8 bf16 values per lane)
  constexpr int RPL = 64 / LPR;        // rows per wavefront load
  constexpr int RPB = 4 * RPL;         // rows per block iteration (4 wavefronts)
  constexpr int U = 4;                 // row iterations per register buffer
  constexpr int STEP = RPB * U;        // rows per buffer
  const LayerView& lv = a.lv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, grp = lane / LPR;
  const int b = blockIdx.y;
  const int n_ret_items = lv.n_ret * a.splits;
  const bool retrieval = (int)blockIdx.x < n_ret_items;

  int kvh, split = 0, nsplit;
  int64_t j0, j1, exclude = -1, new_row;
  uint8_t *kbase, *vbase;
  bool with_new = a.k_new != nullptr;
  if (retrieval) {
    const int slot = blockIdx.x / a.splits;
    split = blockIdx.x % a.splits;
    nsplit = a.splits;
    kvh = uniform_load(lv.ret_heads + slot);
    int64_t chunk = (a.cache_len + nsplit - 1) / nsplit;
    chunk = (chunk + RPB - 1) / RPB * RPB;
    j0 = (int64_t)split * chunk;
    j1 = j0 + chunk < a.cache_len ? j0 + chunk : a.cache_len;
    if (j0 > j1) j0 = j1;
    const int64_t head_row0 = ((int64_t)b * lv.n_ret + slot) * lv.max_seq;
    kbase = lv.k_ret + head_row0 * lv.row_bytes;
    vbase = lv.v_ret + head_row0 * lv.row_bytes;
    with_new = with_new && split == nsplit - 1;
    new_row = a.cache_len;
  } else {
    const int slot = blockIdx.x - n_ret_items;
    nsplit = 1;
    kvh = uniform_load(lv.str_heads + slot);
    const int64_t cap = (int64_t)lv.sink + lv.recent;
    j0 = 0;
    j1 = streaming_rows(a.cache_len, lv.sink, lv.recent);
    // The slot the new token goes to: while it is not yet written, that slot of a
    // full ring still holds the token the append evicts, which the query at
    // position cache_len must not see.
    new_row = a.cache_len < lv.sink ? a.cache_len : lv.sink + (a.cache_len - lv.sink) % lv.recent;
    if (with_new && a.cache_len >= cap) exclude = new_row;
    const int64_t head_row0 = ((int64_t)b * lv.n_str + slot) * cap;
    kbase = lv.k_str + head_row0 * lv.row_bytes;
    vbase = lv.v_str + head_row0 * lv.row_bytes;
  }

  struct Buf { uint4 k[U], v[U]; };
  const int row_in_block = wave * RPL + grp;
  // Loads past the item's end are redirected to its last row (row 0 of the head's
  // cache for an empty item: allocated memory whose value is then ignored).
  const int64_t last_row = j1 > 0 ? j1 - 1 : 0;
  auto issue = [&](Buf& buf, int64_t base) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = base + u * RPB + row_in_block;
      const int64_t rc = r < j1 ? r : last_row;
      buf.k[u] = stream_load16(kbase + rc * lv.row_bytes + sub * 16);
      buf.v[u] = stream_load16(vbase + rc * lv.row_bytes + sub * 16);
    }
  };
  // Raw query piece and the new token's pieces first (they are waited for first),
  // then the first K/V rows; the barrier keeps that issue order.
  const uint4 q_raw = *(const uint4*)((const uint16_t*)a.q + ((int64_t)b * lv.n_q_heads + kvh) * D + sub * 8);
  uint4 new_k = make_uint4(0, 0, 0, 0), new_v = new_k;   // the new token's piece
  if (with_new) {
    new_k = *(const uint4*)((const uint16_t*)a.k_new + ((int64_t)b * lv.n_kv_heads + kvh) * D + sub * 8);
    new_v = *(const uint4*)((const uint16_t*)a.v_new + ((int64_t)b * lv.n_kv_heads + kvh) * D + sub * 8);
  }
  __builtin_amdgcn_sched_barrier(0);
  Buf buf_a;
  issue(buf_a, j0);
  __builtin_amdgcn_sched_barrier(0);

  // Query piece, pre-multiplied by scale * log2(e).
  float q[8];
  {
    const float c = lv.scale * kLog2e;
    widen(q_raw, q);
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] *= c;
  }
  __builtin_amdgcn_sched_barrier(0);
  float m = -INFINITY, l = 0.f, o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = 0.f;

  auto consume = [&](const Buf& buf, int64_t base) {
    float s[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = base + u * RPB + row_in_block;
      const bool ok = r < j1 && r != exclude;
      float kf[8];
      widen(buf.k[u], kf);
      float d = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) d = fmaf(q[i], kf[i], d);
      d = group_sum<LPR>(d);
      s[u] = ok ? d : -INFINITY;
    }
    float mn = m;
#pragma unroll
    for (int u = 0; u < U; ++u) mn = fmaxf(mn, s[u]);
    const float mu = mn == -INFINITY ? 0.f : mn;
    const float alpha = fast_exp2(m - mu);
    float p[U], sum = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) { p[u] = fast_exp2(s[u] - mu); sum += p[u]; }
    l = l * alpha + sum;
    m = mn;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] *= alpha;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float vf[8];
      widen(buf.v[u], vf);
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = fmaf(p[u], vf[i], o[i]);
    }
  };

  // Two register buffers: the loads of the next STEP rows are in flight while the
  // current buffer is consumed.  Inside the loop every issue is unconditional (a
  // conditional one would make the compiler's wait counts assume the shorter queue
  // and drain it); the scheduling barriers keep the loads from being sunk below the
  // arithmetic.  Nothing is loaded past the item's last row.  (Three and four buffers, with
  // the issues running past the end of the item so that all of them stay unconditional, were
  // measured: 0.9 and 1.3 us slower per launch at 32K context, with and without the memory-side
  // cache - the bytes in flight are not what limits this loop.)
  if (j0 < j1) {
    int64_t base = j0;
    Buf buf_b;
    while (base + 2 * STEP < j1) {
      issue(buf_b, base + STEP);
      __builtin_amdgcn_sched_barrier(0);
      consume(buf_a, base);
      __builtin_amdgcn_sched_barrier(0);
      issue(buf_a, base + 2 * STEP);
      __builtin_amdgcn_sched_barrier(0);
      consume(buf_b, base + STEP);
      __builtin_amdgcn_sched_barrier(0);
      base += 2 * STEP;
    }
    if (base + STEP < j1) {
      issue(buf_b, base + STEP);
      __builtin_amdgcn_sched_barrier(0);
      consume(buf_a, base);
      __builtin_amdgcn_sched_barrier(0);
      consume(buf_b, base + STEP);
    } else {
      consume(buf_a, base);
    }
  }

  // The new token, handled by row group 0 of wavefront 0 of the item that owns it;
  // with a.commit its rows are also written into the cache.
  if (with_new && wave == 0 && grp == 0) {
    float kf[8], vf[8];
    widen(new_k, kf);
    widen(new_v, vf);
    if (a.commit) {
      *(uint4*)(kbase + new_row * lv.row_bytes + sub * 16) = new_k;
      *(uint4*)(vbase + new_row * lv.row_bytes + sub * 16) = new_v;
    }
    float d = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) d = fmaf(q[i], kf[i], d);
    d = group_sum<LPR>(d);
    const float mn = fmaxf(m, d);
    const float alpha = fast_exp2(m - mn);
    const float pw = fast_exp2(d - mn);
    l = l * alpha + pw;
    m = mn;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = fmaf(pw, vf[i], o[i] * alpha);
  }

  // Merge the row groups of a wavefront.
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
    const float mo = __shfl_xor(m, off), lo = __shfl_xor(l, off);
    const float mn = fmaxf(m, mo);
    const float mu = mn == -INFINITY ? 0.f : mn;
    const float a1 = fast_exp2(m - mu), a2 = fast_exp2(mo - mu);
    l = l * a1 + lo * a2;
    m = mn;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = o[i] * a1 + __shfl_xor(o[i], off) * a2;
  }
  // Merge the four wavefronts through LDS.
  __shared__ float sm_o[1024];   // [wave][d] during the wavefront merge, [slot][d] in the split merge
  __shared__ float sm_m[4], sm_l[4];
  __shared__ float sm_m2[16], sm_l2[16];   // per merge slot, in the split merge
  __shared__ int sm_last;
  if (grp == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) sm_o[wave * D + sub * 8 + i] = o[i];
    if (sub == 0) { sm_m[wave] = m; sm_l[wave] = l; }
  }
  __syncthreads();
  if (tid < D) {
    const int d = tid;
    float mn = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) mn = fmaxf(mn, sm_m[w]);
    const float mu = mn == -INFINITY ? 0.f : mn;
    float acc = 0.f, ls = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = fast_exp2(sm_m[w] - mu);
      acc += wgt * sm_o[w * D + d];
      ls += wgt * sm_l[w];
    }
    if (nsplit == 1) {
      ((uint16_t*)a.out)[((int64_t)b * lv.n_q_heads + kvh) * D + d] = f32_to_bf16(acc / ls);
      if (a.lse && d == 0) a.lse[(int64_t)b * lv.n_q_heads + kvh] = (mn + log2f(ls)) * kLn2;
    } else {
      const int64_t pi = ((int64_t)b * lv.n_q_heads + kvh) * nsplit + split;
      coherent_store(a.part_o + pi * D + d, acc);
      if (d == 0) { coherent_store(a.part_ml + pi * 2, mn); coherent_store(a.part_ml + pi * 2 + 1, ls); }
    }
  }
  if (nsplit == 1) return;

  // Ticket: the last item of this (sequence, KV head) to get here merges the partials.
  // Hand-off protocol (the same in the matrix-core kernel): the partials are written with
  // device-scope stores, which go through to the memory side of the per-die L2 caches; every
  // thread waits until its stores are acknowledged (s_waitcnt 0), the workgroup barrier collects
  // those waits, and only then does one thread take the ticket, so whoever sees the final ticket
  // value finds every partial in memory.  The compiler fences keep the three steps in that order
  // in the instruction stream.  (A device-scope release fence per workgroup would add a write-back
  // of the die's L2, about a microsecond each here, for data that is already written through.)
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (tid == 0) {
    int* ticket = a.tickets + (int64_t)b * lv.n_kv_heads + kvh;
    const int prev = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sm_last = prev == nsplit - 1;
    if (sm_last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next launch
  }
  __syncthreads();
  if (!sm_last) return;
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  // The partials are read with device-scope loads (after the ticket, on which this branch
  // depends): they are served from the memory side of the L2 caches, so no stale cached copy
  // (of an earlier launch's partials, say) can be hit and no cache invalidation is needed.
  // One memory round trip: the 256 threads form SLOTS rows of TPR threads (one float4 of a
  // partial row each); slot `part` sums the partials part, part + SLOTS, ... in that order with
  // a running maximum, and the slot results are merged through LDS in slot order - a fixed
  // order, so the result is deterministic.
  constexpr int TPR = D / 4;
  constexpr int SLOTS = 256 / TPR;
  const int dq = tid % TPR, part = tid / TPR;
  {
    const int64_t p0 = ((int64_t)b * lv.n_q_heads + kvh) * nsplit;
    const float2* ml = (const float2*)a.part_ml + p0;
    const float4* po = (const float4*)(a.part_o + p0 * D) + dq;
    float mr = -INFINITY, lr = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    constexpr int B4 = 4;   // partial rows fetched together
    for (int s0 = part; s0 < nsplit; s0 += SLOTS * B4) {
      float2 mlv[B4];
      float4 x[B4];
#pragma unroll
      for (int j = 0; j < B4; ++j) {
        const int sidx = s0 + j * SLOTS;
        const int sc = sidx < nsplit ? sidx : nsplit - 1;
        mlv[j] = coherent_load2(ml + sc);
        x[j] = coherent_load4(po + (int64_t)sc * TPR);
      }
#pragma unroll
      for (int j = 0; j < B4; ++j) {
        // rows past the end count as empty; decided here, after every load of the batch has
        // been issued, so that no load waits for the one before it
        const bool there = s0 + j * SLOTS < nsplit;
        const float mj = there ? mlv[j].x : -INFINITY, lj = there ? mlv[j].y : 0.f;
        const float mn = fmaxf(mr, mj);
        const float mu = mn == -INFINITY ? 0.f : mn;
        const float a1 = fast_exp2(mr - mu), a2 = fast_exp2(mj - mu);
        lr = lr * a1 + lj * a2;
        acc.x = acc.x * a1 + x[j].x * a2; acc.y = acc.y * a1 + x[j].y * a2;
        acc.z = acc.z * a1 + x[j].z * a2; acc.w = acc.w * a1 + x[j].w * a2;
        mr = mn;
      }
    }
    __syncthreads();   // sm_o / sm_m / sm_l are free again
    *(float4*)(sm_o + part * D + 4 * dq) = acc;
    if (dq == 0) { sm_m2[part] = mr; sm_l2[part] = lr; }
  }
  __syncthreads();
  if (tid < D) {
    const int d = tid;
    float mn = -INFINITY;
#pragma unroll
    for (int pp = 0; pp < SLOTS; ++pp) mn = fmaxf(mn, sm_m2[pp]);
    float tot = 0.f, ls = 0.f;
#pragma unroll
    for (int pp = 0; pp < SLOTS; ++pp) {
      const float wgt = fast_exp2(sm_m2[pp] - mn);
      tot += wgt * sm_o[pp * D + d];
      ls += wgt * sm_l2[pp];
    }
    ((uint16_t*)a.out)[((int64_t)b * lv.n_q_heads + kvh) * D + d] = f32_to_bf16(tot / ls);
    if (a.lse && d == 0) a.lse[(int64_t)b * lv.n_q_heads + kvh] = (mn + log2f(ls)) * kLn2;
  }
}

}  // namespace

hipError_t launch_decode(const DecodeArgs& a, hipStream_t stream) {
  const LayerView& lv = a.lv;
  // this kernel serves one query head per KV head on a bf16 cache; everything else goes to the
  // matrix-core kernel
  if (lv.group != 1 || lv.kv_mode != 0) return hipErrorInvalidValue;
  if (a.splits < 1 || a.splits > kMaxDecodeSplits) return hipErrorInvalidValue;
  dim3 grid(lv.n_ret * a.splits + lv.n_str, lv.batch);
  if (lv.head_dim == 128) decode_kernel<128><<<grid, 256, 0, stream>>>(a);
  else decode_kernel<64><<<grid, 256, 0, stream>>>(a);
  return hipGetLastError();
}

}  // namespace duo
