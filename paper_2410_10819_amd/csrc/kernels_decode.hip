// Decode attention: one query per sequence against the split KV cache
// (paper, Section 2.3, Decoding; attention definitions of Section 2.2).
//
// The step is bound by HBM bandwidth: every cached K and V row of a retrieval
// head is read once per token, while a streaming head reads at most
// sink + recent rows.  Work decomposition:
//   - one work item (workgroup) per (sequence, retrieval KV head, key split) and
//     one per (sequence, streaming KV head); all query heads of a GQA group share
//     the item, so K/V are read once per group;
//   - inside an item the head_dim/8 (bf16) or head_dim/16 (fp8) lanes of a "row
//     group" each own one 16-byte piece of a row, so a wavefront load covers
//     1 KiB of consecutive cache memory; loads are double-buffered in registers
//     so the next rows are in flight while the current ones are consumed; each
//     row group keeps its own running (max, sum, output) softmax state, merged
//     once at the end of the item;
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

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Device-scope accesses for data exchanged between workgroups inside one launch.
__device__ inline void coherent_store(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
#ifndef DUO_EXP_U
#define DUO_EXP_U 4
#endif
  constexpr int U = DUO_EXP_U;         // row iterations per register buffer
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
    kvh = lv.ret_heads[slot];
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
    kvh = lv.str_heads[slot];
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

  // Query pieces of the group's heads, pre-multiplied by scale * log2(e).
  float q[G][EPL];
  {
    const float c = lv.scale * kLog2e;
    const uint16_t* qp = (const uint16_t*)a.q + ((int64_t)b * lv.n_q_heads + (int64_t)kvh * G) * D + sub * EPL;
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int i = 0; i < EPL; ++i) q[g][i] = __uint_as_float((uint32_t)qp[g * D + i] << 16) * c;
  }
  float m[G], l[G], o[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
    for (int i = 0; i < EPL; ++i) o[g][i] = 0.f;
  }

  struct Buf { uint4 k[U], v[U]; float ks[U], vs[U]; };
  const int row_in_block = wave * RPL + grp;
  auto issue = [&](Buf& buf, int64_t base) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = base + u * RPB + row_in_block;
      const int64_t rc = r < j1 ? r : j1 - 1;
      buf.k[u] = *(const uint4*)(kbase + rc * lv.row_bytes + sub * 16);
      buf.v[u] = *(const uint4*)(vbase + rc * lv.row_bytes + sub * 16);
      if constexpr (FP8) { buf.ks[u] = ksbase[rc]; buf.vs[u] = vsbase[rc]; }
    }
  };
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

  for (int64_t base = j0; base < j1; base += STEP) {
    Buf buf;
    issue(buf, base);
    consume(buf, base);
  }

  // The new token, handled by row group 0 of wavefront 0 of the item that owns it;
  // with a.commit its rows are also written into the cache.
  if (with_new && wave == 0 && grp == 0) {
    const uint16_t* kin = (const uint16_t*)a.k_new + ((int64_t)b * lv.n_kv_heads + kvh) * D + sub * EPL;
    const uint16_t* vin = (const uint16_t*)a.v_new + ((int64_t)b * lv.n_kv_heads + kvh) * D + sub * EPL;
    float kf[EPL], vf[EPL];
    float ksc = 1.f, vsc = 1.f;
    if constexpr (!FP8) {
      const uint4 kc = *(const uint4*)kin;
      const uint4 vc = *(const uint4*)vin;
      Piece<false>::widen(kc, kf);
      Piece<false>::widen(vc, vf);
      if (a.commit) {
        *(uint4*)(kbase + new_row * lv.row_bytes + sub * 16) = kc;
        *(uint4*)(vbase + new_row * lv.row_bytes + sub * 16) = vc;
      }
    } else {
      // quantise exactly as the append kernel does, then attend to the dequantised row
      float kmax = 0.f, vmax = 0.f;
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        kf[i] = __uint_as_float((uint32_t)kin[i] << 16);
        vf[i] = __uint_as_float((uint32_t)vin[i] << 16);
        kmax = fmaxf(kmax, fabsf(kf[i]));
        vmax = fmaxf(vmax, fabsf(vf[i]));
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
  __shared__ float sm_w[kMaxDecodeSplits];
  __shared__ float sm_red[8];
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
  // Acquire: drop any stale cached copies of the partials before reading them.
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  constexpr int TPR = D / 4;        // threads per partial row (one float4 each)
  constexpr int NP = 256 / TPR;     // partial rows in flight
  const int dq = tid % TPR, part = tid / TPR;
  float* flat = sm_o;
  for (int g = 0; g < G; ++g) {
    const int h = kvh * G + g;
    const int64_t p0 = ((int64_t)b * lv.n_q_heads + h) * nsplit;
    // weights of the partials: w_s = 2^(m_s - M), L = sum w_s l_s
    const float2* ml = (const float2*)a.part_ml + p0;
    float2 mine = make_float2(-INFINITY, 0.f);
    if (tid < nsplit) mine = ml[tid];
    float mloc = mine.x;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mloc = fmaxf(mloc, __shfl_xor(mloc, off));
    __syncthreads();
    if (lane == 0) sm_red[wave] = mloc;
    __syncthreads();
    const float mn = fmaxf(fmaxf(sm_red[0], sm_red[1]), fmaxf(sm_red[2], sm_red[3]));
    const float wgt = fast_exp2(mine.x - mn);
    if (tid < nsplit) sm_w[tid] = wgt;
    float lloc = wgt * mine.y;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) lloc += __shfl_xor(lloc, off);
    if (lane == 0) sm_red[4 + wave] = lloc;
    __syncthreads();
    const float ls = (sm_red[4] + sm_red[5]) + (sm_red[6] + sm_red[7]);
    // output: thread (part, dq) sums the partials s = part, part + NP, ... in order
    const float4* po = (const float4*)(a.part_o + p0 * D) + dq;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = part; s < nsplit; s += NP) {
      const float4 x = po[(int64_t)s * TPR];
      const float w = sm_w[s];
      acc.x = fmaf(w, x.x, acc.x); acc.y = fmaf(w, x.y, acc.y);
      acc.z = fmaf(w, x.z, acc.z); acc.w = fmaf(w, x.w, acc.w);
    }
    __syncthreads();
    *(float4*)(flat + part * D + 4 * dq) = acc;   // NP * D = 1024 floats
    __syncthreads();
    if (tid < D) {
      float tot = 0.f;
#pragma unroll
      for (int pp = 0; pp < NP; ++pp) tot += flat[pp * D + tid];
      ((uint16_t*)a.out)[((int64_t)b * lv.n_q_heads + h) * D + tid] = f32_to_bf16(tot / ls);
      if (a.lse && tid == 0) a.lse[(int64_t)b * lv.n_q_heads + h] = (mn + log2f(ls)) * kLn2;
    }
    __syncthreads();
  }
}

template <int D, bool FP8>
hipError_t launch_dg(const DecodeArgs& a, dim3 grid, hipStream_t stream) {
  switch (a.lv.group) {
    case 1: decode_kernel<D, 1, FP8><<<grid, 256, 0, stream>>>(a); break;
    case 2: decode_kernel<D, 2, FP8><<<grid, 256, 0, stream>>>(a); break;
    case 4: decode_kernel<D, 4, FP8><<<grid, 256, 0, stream>>>(a); break;
    case 8:
      if constexpr (FP8) return hipErrorInvalidValue;
      else decode_kernel<D, 8, false><<<grid, 256, 0, stream>>>(a);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode(const DecodeArgs& a, hipStream_t stream) {
  const LayerView& lv = a.lv;
  if (a.splits < 1 || a.splits > kMaxDecodeSplits) return hipErrorInvalidValue;
  dim3 grid(lv.n_ret * a.splits + lv.n_str, lv.batch);
  if (lv.head_dim == 128) return lv.fp8 ? launch_dg<128, true>(a, grid, stream) : launch_dg<128, false>(a, grid, stream);
  return lv.fp8 ? launch_dg<64, true>(a, grid, stream) : launch_dg<64, false>(a, grid, stream);
}

}  // namespace duo
