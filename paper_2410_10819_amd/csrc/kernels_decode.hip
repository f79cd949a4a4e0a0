// Decode attention: one query per sequence against the split KV cache
// (paper, Section 2.3, Decoding; attention definitions of Section 2.2).
//
// The step is bound by HBM bandwidth: every cached K and V row of a retrieval
// head is read once per token, while a streaming head reads at most
// sink + recent rows.  Work decomposition:
//   - one work item per (sequence, retrieval KV head, key split) and one per
//     (sequence, streaming KV head); all query heads of a GQA group share the
//     item, so K/V are read once per group;
//   - inside an item the head_dim/8 (bf16) or head_dim/16 (fp8) lanes of a "row
//     group" each own one 16-byte piece of a row, so a wavefront load covers
//     1 KiB of consecutive cache memory; each row group keeps its own running
//     (max, sum, output) softmax state, merged once at the end of the item;
//   - split partials are merged by a second, tiny kernel in a fixed order, so
//     results are deterministic.
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
  constexpr int U = 4;                 // row iterations in flight
  const LayerView& lv = a.lv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, grp = lane / LPR;
  const int b = blockIdx.y;
  const int n_ret_items = lv.n_ret * a.splits;
  const bool retrieval = (int)blockIdx.x < n_ret_items;

  int kvh, split = 0, nsplit;
  int64_t j0, j1, exclude = -1;
  const uint8_t *kbase, *vbase;
  const float *ksbase = nullptr, *vsbase = nullptr;
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
  } else {
    const int slot = blockIdx.x - n_ret_items;
    nsplit = 1;
    kvh = lv.str_heads[slot];
    const int64_t cap = (int64_t)lv.sink + lv.recent;
    j0 = 0;
    j1 = streaming_rows(a.cache_len, lv.sink, lv.recent);
    // With an un-appended token the ring still holds the token that the append
    // would evict; the query at position cache_len must not see it.
    if (with_new && a.cache_len >= cap) exclude = lv.sink + (a.cache_len - lv.sink) % lv.recent;
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

  for (int64_t base = j0; base < j1; base += RPB * U) {
    uint4 kc[U], vc[U];
    float ksc[U], vsc[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = base + u * RPB + wave * RPL + grp;
      ok[u] = r < j1 && r != exclude;
      const int64_t rc = r < j1 ? r : j1 - 1;
      kc[u] = *(const uint4*)(kbase + rc * lv.row_bytes + sub * 16);
      vc[u] = *(const uint4*)(vbase + rc * lv.row_bytes + sub * 16);
      if constexpr (FP8) { ksc[u] = ksbase[rc]; vsc[u] = vsbase[rc]; }
    }
    float s[U][G];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPL];
      Piece<FP8>::widen(kc[u], kf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) d = fmaf(q[g][i], kf[i], d);
#pragma unroll
        for (int off = 1; off < LPR; off <<= 1) d += __shfl_xor(d, off);
        if constexpr (FP8) d *= ksc[u];
        s[u][g] = ok[u] ? d : -INFINITY;
      }
    }
    float p[U][G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mn = m[g];
#pragma unroll
      for (int u = 0; u < U; ++u) mn = fmaxf(mn, s[u][g]);
      const float mu = mn == -INFINITY ? 0.f : mn;
      const float alpha = exp2f(m[g] - mu);
      float sum = 0.f;
#pragma unroll
      for (int u = 0; u < U; ++u) { p[u][g] = exp2f(s[u][g] - mu); sum += p[u][g]; }
      l[g] = l[g] * alpha + sum;
      m[g] = mn;
#pragma unroll
      for (int i = 0; i < EPL; ++i) o[g][i] *= alpha;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float vf[EPL];
      Piece<FP8>::widen(vc[u], vf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float pw = FP8 ? p[u][g] * vsc[u] : p[u][g];
#pragma unroll
        for (int i = 0; i < EPL; ++i) o[g][i] = fmaf(pw, vf[i], o[g][i]);
      }
    }
  }

  // The un-appended token (bf16 caches only): handled by row group 0 of wavefront 0.
  if constexpr (!FP8) {
    if (with_new && wave == 0 && grp == 0) {
      const int64_t off = ((int64_t)b * lv.n_kv_heads + kvh) * D + sub * 8;
      const uint4 kc = *(const uint4*)((const uint16_t*)a.k_new + off);
      const uint4 vc = *(const uint4*)((const uint16_t*)a.v_new + off);
      float kf[8], vf[8];
      Piece<false>::widen(kc, kf);
      Piece<false>::widen(vc, vf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) d = fmaf(q[g][i], kf[i], d);
#pragma unroll
        for (int off2 = 1; off2 < LPR; off2 <<= 1) d += __shfl_xor(d, off2);
        const float mn = fmaxf(m[g], d);
        const float alpha = exp2f(m[g] - mn);
        const float pw = exp2f(d - mn);
        l[g] = l[g] * alpha + pw;
        m[g] = mn;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[g][i] = fmaf(pw, vf[i], o[g][i] * alpha);
      }
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
      const float a1 = exp2f(m[g] - mu), a2 = exp2f(mo - mu);
      l[g] = l[g] * a1 + lo * a2;
      m[g] = mn;
#pragma unroll
      for (int i = 0; i < EPL; ++i) o[g][i] = o[g][i] * a1 + __shfl_xor(o[g][i], off) * a2;
    }
  }
  // Merge the four wavefronts through LDS.
  __shared__ float sm_o[4][G][D];
  __shared__ float sm_m[4][G], sm_l[4][G];
  if (grp == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int i = 0; i < EPL; ++i) sm_o[wave][g][sub * EPL + i] = o[g][i];
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
      const float wgt = exp2f(sm_m[w][g] - mu);
      acc += wgt * sm_o[w][g][d];
      ls += wgt * sm_l[w][g];
    }
    const int h = kvh * G + g;
    if (nsplit == 1) {
      ((uint16_t*)a.out)[((int64_t)b * lv.n_q_heads + h) * D + d] = f32_to_bf16(acc / ls);
      if (a.lse && d == 0) a.lse[(int64_t)b * lv.n_q_heads + h] = (mn + log2f(ls)) * kLn2;
    } else {
      const int64_t pi = ((int64_t)b * lv.n_q_heads + h) * nsplit + split;
      a.part_o[pi * D + d] = acc;
      if (d == 0) { a.part_ml[pi * 2] = mn; a.part_ml[pi * 2 + 1] = ls; }
    }
  }
}

// Merge the split partials of the retrieval heads (fixed order -> deterministic).
template <int D>
__global__ __launch_bounds__(D) void combine_kernel(DecodeArgs a) {
  const LayerView& lv = a.lv;
  const int slot = blockIdx.x / lv.group, g = blockIdx.x % lv.group;
  const int h = lv.ret_heads[slot] * lv.group + g;
  const int b = blockIdx.y, d = threadIdx.x;
  const int64_t p0 = ((int64_t)b * lv.n_q_heads + h) * a.splits;
  float mn = -INFINITY;
  for (int s = 0; s < a.splits; ++s) mn = fmaxf(mn, a.part_ml[(p0 + s) * 2]);
  float acc = 0.f, ls = 0.f;
  for (int s = 0; s < a.splits; ++s) {
    const float w = exp2f(a.part_ml[(p0 + s) * 2] - mn);
    ls += w * a.part_ml[(p0 + s) * 2 + 1];
    acc += w * a.part_o[(p0 + s) * D + d];
  }
  ((uint16_t*)a.out)[((int64_t)b * lv.n_q_heads + h) * D + d] = f32_to_bf16(acc / ls);
  if (a.lse && d == 0) a.lse[(int64_t)b * lv.n_q_heads + h] = (mn + log2f(ls)) * kLn2;
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
  dim3 grid(lv.n_ret * a.splits + lv.n_str, lv.batch);
  hipError_t e;
  if (lv.head_dim == 128) e = lv.fp8 ? launch_dg<128, true>(a, grid, stream) : launch_dg<128, false>(a, grid, stream);
  else e = lv.fp8 ? launch_dg<64, true>(a, grid, stream) : launch_dg<64, false>(a, grid, stream);
  if (e != hipSuccess) return e;
  if (a.splits > 1 && lv.n_ret > 0) {
    dim3 cgrid(lv.n_ret * lv.group, lv.batch);
    if (lv.head_dim == 128) combine_kernel<128><<<cgrid, 128, 0, stream>>>(a);
    else combine_kernel<64><<<cgrid, 64, 0, stream>>>(a);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace duo
