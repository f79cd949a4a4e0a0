// Decode attention on the vector unit: one query per sequence against the split KV
// cache (paper, Section 2.3, Decoding; attention definitions of Section 2.2).
// This kernel serves one query head per KV head on a bf16 cache (its templates
// also cover query groups and fp8 rows, which the matrix-core kernel in
// kernels_decode_sk.hip handles with far fewer instructions per byte).
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


// fp32 -> OCP E4M3 (finite-only) code, round to nearest even, saturating at 448.
__device__ inline uint32_t e4m3_encode(float x) {
  uint32_t u = __float_as_uint(x);
  uint32_t sign = (u >> 24) & 0x80u;
  u &= 0x7FFFFFFFu;
  float a = __uint_as_float(u);
  uint32_t code;
  if (a >= 448.0f) {
    code = 0x7Eu;
  } else if (a < 0.015625f) {
    code = (uint32_t)rintf(a * 512.0f);
  } else {
    uint32_t r = u + 0x7FFFFu + ((u >> 20) & 1u);
    code = (r >> 20) - ((127u - 7u) << 3);
  }
  return code | sign;
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
template <int LPR>
__device__ inline float group_max(float x) {
  x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true)));
  x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true)));
  if constexpr (LPR >= 8)
    x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true)));
  if constexpr (LPR >= 16)
    x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true)));
  return x;
}

typedef float f32x2_t __attribute__((ext_vector_type(2)));

// Widen one 16-byte piece of a row to floats: 8 bf16 values or 16 E4M3 codes.
template <bool FP8>
struct Piece {
  static constexpr int N = FP8 ? 16 : 8;
  __device__ static inline void widen(const uint4& c, float (&f)[N]) {
    const uint32_t w[4] = {c.x, c.y, c.z, c.w};
    if constexpr (FP8) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        f32x2_t a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);
        f32x2_t b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
        f[4 * i] = a[0]; f[4 * i + 1] = a[1]; f[4 * i + 2] = b[0]; f[4 * i + 3] = b[1];
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) { f[2 * i] = bf16_lo(w[i]); f[2 * i + 1] = bf16_hi(w[i]); }
    }
  }
};

template <int D, int G, bool FP8>
__global__ __launch_bounds__(256) void decode_kernel(DecodeArgs a) {
  constexpr int EPL = Piece<FP8>::N;   // elements per lane
  constexpr int LPR = D / EPL;         // lanes per row
  constexpr int RPL = 64 / LPR;        // rows per wavefront load
  constexpr int RPB = 4 * RPL;         // rows per block iteration (4 wavefronts)
  // row iterations per register buffer: as many as fit beside the per-head state
  constexpr int U = (FP8 && G == 2) ? 2 : 4;
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
  float *ksbase = nullptr, *vsbase = nullptr;
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
    if (FP8) { ksbase = lv.ks_ret + head_row0; vsbase = lv.vs_ret + head_row0; }
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
    if (FP8) { ksbase = lv.ks_str + head_row0; vsbase = lv.vs_str + head_row0; }
  }

  struct Buf { uint4 k[U], v[U]; float ks[U], vs[U]; };
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
      if constexpr (FP8) { buf.ks[u] = ksbase[rc]; buf.vs[u] = vsbase[rc]; }
    }
  };
  // Raw query pieces and the new token's pieces first (they are waited for first),
  // then the first K/V rows; the barrier keeps that issue order.
  uint4 q_raw[G][EPL / 8];
  {
    const uint4* qp = (const uint4*)((const uint16_t*)a.q + ((int64_t)b * lv.n_q_heads + (int64_t)kvh * G) * D + sub * EPL);
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int i = 0; i < EPL / 8; ++i) q_raw[g][i] = qp[g * (D / 8) + i];
  }
  uint4 new_k[EPL / 8], new_v[EPL / 8];   // the new token's piece: EPL bf16 values
  if (with_new) {
    const uint4* kin = (const uint4*)((const uint16_t*)a.k_new + ((int64_t)b * lv.n_kv_heads + kvh) * D + sub * EPL);
    const uint4* vin = (const uint4*)((const uint16_t*)a.v_new + ((int64_t)b * lv.n_kv_heads + kvh) * D + sub * EPL);
#pragma unroll
    for (int i = 0; i < EPL / 8; ++i) { new_k[i] = kin[i]; new_v[i] = vin[i]; }
  }
  __builtin_amdgcn_sched_barrier(0);
  Buf buf_a;
  issue(buf_a, j0);
  __builtin_amdgcn_sched_barrier(0);

  // Query pieces of the group's heads, pre-multiplied by scale * log2(e).
  float q[G][EPL];
  {
    const float c = lv.scale * kLog2e;
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int i = 0; i < EPL / 8; ++i) {
        float f[8];
        Piece<false>::widen(q_raw[g][i], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) q[g][8 * i + e] = f[e] * c;
      }
  }
  __builtin_amdgcn_sched_barrier(0);
  float m[G], l[G], o[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
    for (int i = 0; i < EPL; ++i) o[g][i] = 0.f;
  }

  auto consume = [&](const Buf& buf, int64_t base) {
    float s[U][G];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = base + u * RPB + row_in_block;
      const bool ok = r < j1 && r != exclude;
      float kf[EPL];
      Piece<FP8>::widen(buf.k[u], kf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) d = fmaf(q[g][i], kf[i], d);
        d = group_sum<LPR>(d);
        if constexpr (FP8) d *= buf.ks[u];
        s[u][g] = ok ? d : -INFINITY;
      }
    }
    float p[U][G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mn = m[g];
#pragma unroll
      for (int u = 0; u < U; ++u) mn = fmaxf(mn, s[u][g]);
      const float mu = mn == -INFINITY ? 0.f : mn;
      const float alpha = fast_exp2(m[g] - mu);
      float sum = 0.f;
#pragma unroll
      for (int u = 0; u < U; ++u) { p[u][g] = fast_exp2(s[u][g] - mu); sum += p[u][g]; }
      l[g] = l[g] * alpha + sum;
      m[g] = mn;
#pragma unroll
      for (int i = 0; i < EPL; ++i) o[g][i] *= alpha;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float vf[EPL];
      Piece<FP8>::widen(buf.v[u], vf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float pw = FP8 ? p[u][g] * buf.vs[u] : p[u][g];
#pragma unroll
        for (int i = 0; i < EPL; ++i) o[g][i] = fmaf(pw, vf[i], o[g][i]);
      }
    }
  };

  // Two register buffers: the loads of the next STEP rows are in flight while the
  // current buffer is consumed.  Inside the loop every issue is unconditional (a
  // conditional one would make the compiler's wait counts assume the shorter queue
  // and drain it); the scheduling barriers keep the loads from being sunk below the
  // arithmetic.  Nothing is loaded past the item's last row.  The variants with the
  // most per-head state have no registers for a second buffer.
  constexpr bool kTwoBuffers = !((FP8 && G >= 4) || G >= 8);
  if (j0 < j1) {
    int64_t base = j0;
    if constexpr (kTwoBuffers) {
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
    } else {
      consume(buf_a, base);
      for (base += STEP; base < j1; base += STEP) {
        issue(buf_a, base);
        consume(buf_a, base);
      }
    }
  }

  // The new token, handled by row group 0 of wavefront 0 of the item that owns it;
  // with a.commit its rows are also written into the cache.
  if (with_new && wave == 0 && grp == 0) {
    float kf[EPL], vf[EPL];
    float ksc = 1.f, vsc = 1.f;
    if constexpr (!FP8) {
      Piece<false>::widen(new_k[0], kf);
      Piece<false>::widen(new_v[0], vf);
      if (a.commit) {
        *(uint4*)(kbase + new_row * lv.row_bytes + sub * 16) = new_k[0];
        *(uint4*)(vbase + new_row * lv.row_bytes + sub * 16) = new_v[0];
      }
    } else {
      // quantise exactly as the append kernel does, then attend to the dequantised row
      float kmax = 0.f, vmax = 0.f;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        float f[8];
        Piece<false>::widen(new_k[i], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) { kf[8 * i + e] = f[e]; kmax = fmaxf(kmax, fabsf(f[e])); }
        Piece<false>::widen(new_v[i], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) { vf[8 * i + e] = f[e]; vmax = fmaxf(vmax, fabsf(f[e])); }
      }
      kmax = group_max<LPR>(kmax);
      vmax = group_max<LPR>(vmax);
      ksc = kmax == 0.f ? 1.0f : kmax / 448.0f;
      vsc = vmax == 0.f ? 1.0f : vmax / 448.0f;
      uint32_t kq[4] = {0, 0, 0, 0}, vq[4] = {0, 0, 0, 0};
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        kq[i / 4] |= e4m3_encode(kf[i] / ksc) << (8 * (i % 4));
        vq[i / 4] |= e4m3_encode(vf[i] / vsc) << (8 * (i % 4));
      }
      const uint4 kc = make_uint4(kq[0], kq[1], kq[2], kq[3]);
      const uint4 vc = make_uint4(vq[0], vq[1], vq[2], vq[3]);
      Piece<true>::widen(kc, kf);
      Piece<true>::widen(vc, vf);
      if (a.commit) {
        *(uint4*)(kbase + new_row * lv.row_bytes + sub * 16) = kc;
        *(uint4*)(vbase + new_row * lv.row_bytes + sub * 16) = vc;
        if (sub == 0) { ksbase[new_row] = ksc; vsbase[new_row] = vsc; }
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float d = 0.f;
#pragma unroll
      for (int i = 0; i < EPL; ++i) d = fmaf(q[g][i], kf[i], d);
      d = group_sum<LPR>(d) * ksc;
      const float mn = fmaxf(m[g], d);
      const float alpha = fast_exp2(m[g] - mn);
      const float pw = fast_exp2(d - mn);
      l[g] = l[g] * alpha + pw;
      m[g] = mn;
      const float pv = pw * vsc;
#pragma unroll
      for (int i = 0; i < EPL; ++i) o[g][i] = fmaf(pv, vf[i], o[g][i] * alpha);
    }
  }

  // Merge the row groups of a wavefront.
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mo = __shfl_xor(m[g], off), lo = __shfl_xor(l[g], off);
      const float mn = fmaxf(m[g], mo);
      const float mu = mn == -INFINITY ? 0.f : mn;
      const float a1 = fast_exp2(m[g] - mu), a2 = fast_exp2(mo - mu);
      l[g] = l[g] * a1 + lo * a2;
      m[g] = mn;
#pragma unroll
      for (int i = 0; i < EPL; ++i) o[g][i] = o[g][i] * a1 + __shfl_xor(o[g][i], off) * a2;
    }
  }
  // Merge the four wavefronts through LDS.
  constexpr int kSmO = 4 * G * D > 1024 ? 4 * G * D : 1024;
  __shared__ float sm_o[kSmO];   // [wave][g][d] during the wavefront merge, [part][d] in the split merge
  __shared__ float sm_m[4][G], sm_l[4][G];
  __shared__ float sm_m2[16], sm_l2[16];   // per merge slot, in the split merge
  __shared__ int sm_last;
  if (grp == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int i = 0; i < EPL; ++i) sm_o[(wave * G + g) * D + sub * EPL + i] = o[g][i];
      if (sub == 0) { sm_m[wave][g] = m[g]; sm_l[wave][g] = l[g]; }
    }
  }
  __syncthreads();
  for (int idx = tid; idx < G * D; idx += 256) {
    const int g = idx / D, d = idx % D;
    float mn = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) mn = fmaxf(mn, sm_m[w][g]);
    const float mu = mn == -INFINITY ? 0.f : mn;
    float acc = 0.f, ls = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = fast_exp2(sm_m[w][g] - mu);
      acc += wgt * sm_o[(w * G + g) * D + d];
      ls += wgt * sm_l[w][g];
    }
    const int h = kvh * G + g;
    if (nsplit == 1) {
      ((uint16_t*)a.out)[((int64_t)b * lv.n_q_heads + h) * D + d] = f32_to_bf16(acc / ls);
      if (a.lse && d == 0) a.lse[(int64_t)b * lv.n_q_heads + h] = (mn + log2f(ls)) * kLn2;
    } else {
      const int64_t pi = ((int64_t)b * lv.n_q_heads + h) * nsplit + split;
      coherent_store(a.part_o + pi * D + d, acc);
      if (d == 0) { coherent_store(a.part_ml + pi * 2, mn); coherent_store(a.part_ml + pi * 2 + 1, ls); }
    }
  }
  if (nsplit == 1) return;

  // Ticket: the last item of this (sequence, KV head) to get here merges the partials.
  // The partials are written and read with device-scope atomic accesses, which go
  // to the memory side of the per-XCD L2 caches; waiting for the stores to be
  // acknowledged before taking the ticket orders them without a cache write-back
  // (a device-scope fence per workgroup costs about a microsecond each here).
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
  // The partials are read with device-scope loads (after the ticket, on which this branch
  // depends), so no cached copy of an earlier launch's partials can be hit.
  // All heads of the group at once, one memory round trip: the 256 threads form
  // SLOTS rows of TPR threads (one float4 of a partial row each); head g owns NP
  // consecutive slots, slot `part` of a head sums the partials part, part + NP, ...
  // in that order with a running maximum, and the NP slot results are merged
  // through LDS in slot order - a fixed order, so the result is deterministic.
  constexpr int TPR = D / 4;
  constexpr int SLOTS = 256 / TPR;
  static_assert(SLOTS % G == 0, "group size must divide the merge slots");
  constexpr int NP = SLOTS / G;
  const int dq = tid % TPR, slot_id = tid / TPR;
  const int mg = slot_id / NP, part = slot_id % NP;
  {
    const int h = kvh * G + mg;
    const int64_t p0 = ((int64_t)b * lv.n_q_heads + h) * nsplit;
    const float2* ml = (const float2*)a.part_ml + p0;
    const float4* po = (const float4*)(a.part_o + p0 * D) + dq;
    float mr = -INFINITY, lr = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    constexpr int B4 = 4;   // partial rows fetched together
    for (int s0 = part; s0 < nsplit; s0 += NP * B4) {
      float2 mlv[B4];
      float4 x[B4];
#pragma unroll
      for (int j = 0; j < B4; ++j) {
        const int sidx = s0 + j * NP;
        const int sc = sidx < nsplit ? sidx : nsplit - 1;
        mlv[j] = coherent_load2(ml + sc);
        x[j] = coherent_load4(po + (int64_t)sc * TPR);
      }
#pragma unroll
      for (int j = 0; j < B4; ++j) {
        // rows past the end count as empty; decided here, after every load of the batch has
        // been issued, so that no load waits for the one before it
        const bool there = s0 + j * NP < nsplit;
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
    *(float4*)(sm_o + slot_id * D + 4 * dq) = acc;
    if (dq == 0) { sm_m2[slot_id] = mr; sm_l2[slot_id] = lr; }
  }
  __syncthreads();
  for (int idx = tid; idx < G * D; idx += 256) {
    const int g = idx / D, d = idx % D;
    float mn = -INFINITY;
#pragma unroll
    for (int pp = 0; pp < NP; ++pp) mn = fmaxf(mn, sm_m2[g * NP + pp]);
    float tot = 0.f, ls = 0.f;
#pragma unroll
    for (int pp = 0; pp < NP; ++pp) {
      const float wgt = fast_exp2(sm_m2[g * NP + pp] - mn);
      tot += wgt * sm_o[(g * NP + pp) * D + d];
      ls += wgt * sm_l2[g * NP + pp];
    }
    const int h = kvh * G + g;
    ((uint16_t*)a.out)[((int64_t)b * lv.n_q_heads + h) * D + d] = f32_to_bf16(tot / ls);
    if (a.lse && d == 0) a.lse[(int64_t)b * lv.n_q_heads + h] = (mn + log2f(ls)) * kLn2;
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
  if (lv.head_dim == 128) decode_kernel<128, 1, false><<<grid, 256, 0, stream>>>(a);
  else decode_kernel<64, 1, false><<<grid, 256, 0, stream>>>(a);
  return hipGetLastError();
}

}  // namespace duo
