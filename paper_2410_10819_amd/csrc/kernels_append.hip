// KV-cache append and export kernels.
//
// Append (paper, Section 2.3, Decoding / Chunked Pre-filling): a retrieval head
// stores every token, so a new row goes to its position in the dense cache; a
// streaming head keeps only the sink tokens and the most recent `recent` tokens,
// so a new row at position p goes to slot p (p < sink) or to ring slot
// sink + (p - sink) % recent, overwriting the oldest non-sink token.  When one
// call appends more than `recent` tokens only the rows that survive are written,
// so no two rows of a call ever target the same slot.
#include "duo_internal.h"

namespace duo {
namespace {

__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// One 16-byte chunk (8 bf16 values) of one row per thread; the head_dim/8 threads
// of a row sit in adjacent lanes.
// MODE: 0 bf16 rows, 1 fp8 codes + scale, 2 int4 / 3 int8 codes + (scale, minimum).
template <int D, int MODE>
__global__ __launch_bounds__(256) void append_kernel(LayerView lv, const uint4* __restrict__ k_in,
                                                     const uint4* __restrict__ v_in, int64_t pos0,
                                                     int n_new, int64_t total_rows) {
  constexpr int LPR = D / 8;  // lanes per row
  const int64_t row = (int64_t)blockIdx.x * (256 / LPR) + threadIdx.x / LPR;
  const int sub = threadIdx.x % LPR;
  const bool live = row < total_rows;
  const int64_t r = live ? row : total_rows - 1;
  // row index -> (batch, token, kv head)
  const int h = (int)(r % lv.n_kv_heads);
  const int64_t bt = r / lv.n_kv_heads;
  const int t = (int)(bt % n_new);
  const int b = (int)(bt / n_new);
  const int64_t p = pos0 + t;
  const uint32_t info = lv.head_info[h];
  const bool retrieval = (info & kRetrievalBit) != 0;
  const int slot_head = (int)(info & ~kRetrievalBit);

  bool write = live;
  int64_t dst_row;  // row index inside the class's cache
  if (retrieval) {
    dst_row = ((int64_t)b * lv.n_ret + slot_head) * lv.max_seq + p;
  } else {
    const int64_t cap = (int64_t)lv.sink + lv.recent;
    int64_t slot;
    if (p < lv.sink) {
      slot = p;
    } else {
      slot = lv.sink + (p - lv.sink) % lv.recent;
      // rows of this call that a later row of the same call would overwrite
      if (p + lv.recent < pos0 + n_new) write = false;
    }
    dst_row = ((int64_t)b * lv.n_str + slot_head) * cap + slot;
  }
  const uint4 kc = k_in[r * LPR + sub];
  const uint4 vc = v_in[r * LPR + sub];
  if constexpr (MODE == 0) {
    if (write) {
      uint4* kd = (uint4*)(retrieval ? lv.k_ret : lv.k_str);
      uint4* vd = (uint4*)(retrieval ? lv.v_ret : lv.v_str);
      kd[dst_row * LPR + sub] = kc;
      vd[dst_row * LPR + sub] = vc;
    }
  } else if constexpr (MODE == 2 || MODE == 3) {
    // asymmetric codes per row, all in fp32: lo = min, scale = (max - lo) / top (1 for a constant
    // row), code = clamp(rint((x - lo) / scale), 0, top), top = 15 or 255.  4-bit: element j of the
    // lane's eight goes to bits 4 j of its dword, so element 2 i sits in the low nibble of byte i
    // of the row; 8-bit: one byte per element.
    constexpr float kTop = MODE == 2 ? 15.0f : 255.0f;
    const uint32_t kw[4] = {kc.x, kc.y, kc.z, kc.w};
    const uint32_t vw[4] = {vc.x, vc.y, vc.z, vc.w};
    float kf[8], vf[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      kf[2 * i] = bf16_lo(kw[i]); kf[2 * i + 1] = bf16_hi(kw[i]);
      vf[2 * i] = bf16_lo(vw[i]); vf[2 * i + 1] = bf16_hi(vw[i]);
    }
    float kmin = kf[0], kmax = kf[0], vmin = vf[0], vmax = vf[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) {
      kmin = fminf(kmin, kf[i]); kmax = fmaxf(kmax, kf[i]);
      vmin = fminf(vmin, vf[i]); vmax = fmaxf(vmax, vf[i]);
    }
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) {
      kmin = fminf(kmin, __shfl_xor(kmin, off)); kmax = fmaxf(kmax, __shfl_xor(kmax, off));
      vmin = fminf(vmin, __shfl_xor(vmin, off)); vmax = fmaxf(vmax, __shfl_xor(vmax, off));
    }
    const float kspan = kmax - kmin, vspan = vmax - vmin;
    const float ks = kspan == 0.f ? 1.0f : kspan / kTop;
    const float vs = vspan == 0.f ? 1.0f : vspan / kTop;
    constexpr int kBits = MODE == 2 ? 4 : 8;
    uint32_t kq[2] = {0, 0}, vq[2] = {0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float kr = fminf(fmaxf(rintf((kf[i] - kmin) / ks), 0.f), kTop);
      const float vr = fminf(fmaxf(rintf((vf[i] - vmin) / vs), 0.f), kTop);
      kq[i * kBits / 32] |= (uint32_t)kr << (i * kBits % 32);
      vq[i * kBits / 32] |= (uint32_t)vr << (i * kBits % 32);
    }
    if (write) {
      if constexpr (MODE == 2) {
        uint32_t* kd = (uint32_t*)(retrieval ? lv.k_ret : lv.k_str);
        uint32_t* vd = (uint32_t*)(retrieval ? lv.v_ret : lv.v_str);
        kd[dst_row * LPR + sub] = kq[0];
        vd[dst_row * LPR + sub] = vq[0];
      } else {
        uint2* kd = (uint2*)(retrieval ? lv.k_ret : lv.k_str);
        uint2* vd = (uint2*)(retrieval ? lv.v_ret : lv.v_str);
        kd[dst_row * LPR + sub] = make_uint2(kq[0], kq[1]);
        vd[dst_row * LPR + sub] = make_uint2(vq[0], vq[1]);
      }
      if (sub == 0) {
        ((float2*)(retrieval ? lv.ks_ret : lv.ks_str))[dst_row] = make_float2(ks, kmin);
        ((float2*)(retrieval ? lv.vs_ret : lv.vs_str))[dst_row] = make_float2(vs, vmin);
      }
    }
  } else {
    const uint32_t kw[4] = {kc.x, kc.y, kc.z, kc.w};
    const uint32_t vw[4] = {vc.x, vc.y, vc.z, vc.w};
    float kf[8], vf[8];
    float kmax = 0.f, vmax = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      kf[2 * i] = bf16_lo(kw[i]); kf[2 * i + 1] = bf16_hi(kw[i]);
      vf[2 * i] = bf16_lo(vw[i]); vf[2 * i + 1] = bf16_hi(vw[i]);
      kmax = fmaxf(kmax, fmaxf(fabsf(kf[2 * i]), fabsf(kf[2 * i + 1])));
      vmax = fmaxf(vmax, fmaxf(fabsf(vf[2 * i]), fabsf(vf[2 * i + 1])));
    }
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) {
      kmax = fmaxf(kmax, __shfl_xor(kmax, off));
      vmax = fmaxf(vmax, __shfl_xor(vmax, off));
    }
    const float ks = kmax == 0.f ? 1.0f : kmax / 448.0f;
    const float vs = vmax == 0.f ? 1.0f : vmax / 448.0f;
    uint32_t kq[2] = {0, 0}, vq[2] = {0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      kq[i / 4] |= e4m3_encode(kf[i] / ks) << (8 * (i % 4));
      vq[i / 4] |= e4m3_encode(vf[i] / vs) << (8 * (i % 4));
    }
    if (write) {
      uint2* kd = (uint2*)(retrieval ? lv.k_ret : lv.k_str);
      uint2* vd = (uint2*)(retrieval ? lv.v_ret : lv.v_str);
      kd[dst_row * LPR + sub] = make_uint2(kq[0], kq[1]);
      vd[dst_row * LPR + sub] = make_uint2(vq[0], vq[1]);
      if (sub == 0) {
        (retrieval ? lv.ks_ret : lv.ks_str)[dst_row] = ks;
        (retrieval ? lv.vs_ret : lv.vs_str)[dst_row] = vs;
      }
    }
  }
}

// Copy the rows a head currently holds, in ascending position order.
__global__ __launch_bounds__(256) void export_kernel(LayerView lv, int batch_idx, int kv_head, int64_t len,
                                                     uint8_t* k_out, uint8_t* v_out, float* ks_out, float* vs_out,
                                                     int64_t* pos_out, int64_t count) {
  const int words_per_row = lv.row_bytes / 4;
  const int rows_per_block = 256 / words_per_row;
  const int64_t idx = (int64_t)blockIdx.x * rows_per_block + threadIdx.x / words_per_row;
  const int w = threadIdx.x % words_per_row;
  if (threadIdx.x / words_per_row >= rows_per_block || idx >= count) return;
  const uint32_t info = lv.head_info[kv_head];
  const bool retrieval = (info & kRetrievalBit) != 0;
  const int slot_head = (int)(info & ~kRetrievalBit);
  int64_t p, src_row;
  if (retrieval) {
    p = idx;
    src_row = ((int64_t)batch_idx * lv.n_ret + slot_head) * lv.max_seq + p;
  } else {
    const int64_t cap = (int64_t)lv.sink + lv.recent;
    const int64_t n_sink = len < lv.sink ? len : lv.sink;
    if (idx < n_sink) {
      p = idx;
    } else {
      const int64_t first = (len - lv.recent > lv.sink) ? len - lv.recent : lv.sink;
      p = first + (idx - n_sink);
    }
    const int64_t slot = p < lv.sink ? p : lv.sink + (p - lv.sink) % lv.recent;
    src_row = ((int64_t)batch_idx * lv.n_str + slot_head) * cap + slot;
  }
  const uint32_t* ks = (const uint32_t*)(retrieval ? lv.k_ret : lv.k_str);
  const uint32_t* vs = (const uint32_t*)(retrieval ? lv.v_ret : lv.v_str);
  ((uint32_t*)k_out)[idx * words_per_row + w] = ks[src_row * words_per_row + w];
  ((uint32_t*)v_out)[idx * words_per_row + w] = vs[src_row * words_per_row + w];
  if (w == 0) {
    pos_out[idx] = p;
    const float* ksrc = retrieval ? lv.ks_ret : lv.ks_str;
    const float* vsrc = retrieval ? lv.vs_ret : lv.vs_str;
    for (int j = 0; j < lv.sc_per_row; ++j) {
      ks_out[idx * lv.sc_per_row + j] = ksrc[src_row * lv.sc_per_row + j];
      vs_out[idx * lv.sc_per_row + j] = vsrc[src_row * lv.sc_per_row + j];
    }
  }
}

// bf16 image of quantised rows: value = code * scale (fp8) or code * scale + minimum (int4, int8),
// in fp32, rounded to nearest even.  One 16-byte piece of output (8 values) per thread; a segment
// is one (sequence, head) run of `seg_stride` rows of which `rows` rows from `first_row` on are widened.
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
  a += 0x7FFFu + ((a >> 16) & 1u);
  b += 0x7FFFu + ((b >> 16) & 1u);
  return (a >> 16) | (b & 0xFFFF0000u);
}

template <int MODE>
__global__ __launch_bounds__(256) void dequant_kernel(const uint8_t* __restrict__ codes, const float* __restrict__ params,
                                                      uint4* __restrict__ out, int head_dim, int64_t n_seg,
                                                      int64_t seg_stride, int64_t first_row, int64_t rows) {
  const int ppr = head_dim / 8;   // pieces per row
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n_seg * rows * ppr) return;
  const int piece = (int)(idx % ppr);
  const int64_t r = idx / ppr;
  const int64_t row = (r / rows) * seg_stride + first_row + r % rows;
  float f[8];
  if constexpr (MODE == 2) {
    const uint32_t w = *(const uint32_t*)(codes + row * (head_dim / 2) + piece * 4);
    const float2 sl = *(const float2*)(params + row * 2);
#pragma unroll
    for (int j = 0; j < 8; ++j) f[j] = fmaf((float)((w >> (4 * j)) & 0xFu), sl.x, sl.y);
  } else {
    const uint2 w = *(const uint2*)(codes + row * head_dim + piece * 8);
    const uint32_t ww[2] = {w.x, w.y};
    if constexpr (MODE == 3) {
      const float2 sl = *(const float2*)(params + row * 2);
#pragma unroll
      for (int j = 0; j < 8; ++j) f[j] = fmaf((float)((ww[j / 4] >> (8 * (j % 4))) & 0xFFu), sl.x, sl.y);
    } else {
      const float sc = params[row];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const auto a = __builtin_amdgcn_cvt_pk_f32_fp8((int)ww[i], false);
        const auto b = __builtin_amdgcn_cvt_pk_f32_fp8((int)ww[i], true);
        f[4 * i] = a[0] * sc; f[4 * i + 1] = a[1] * sc; f[4 * i + 2] = b[0] * sc; f[4 * i + 3] = b[1] * sc;
      }
    }
  }
  out[row * ppr + piece] = make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                                      pack_bf16x2(f[6], f[7]));
}

}  // namespace

hipError_t launch_dequant(const LayerView& lv, int64_t first_ret_row, int64_t len, void* k_ret_out, void* v_ret_out,
                          void* k_str_out, void* v_str_out, hipStream_t stream) {
  if (lv.kv_mode < 1 || lv.kv_mode > 3) return hipErrorInvalidValue;
  if (first_ret_row < 0 || first_ret_row > len) return hipErrorInvalidValue;
  const int64_t cap = (int64_t)lv.sink + lv.recent;
  const int64_t str_rows = streaming_rows(len, lv.sink, lv.recent);
  struct { const uint8_t* codes; const float* params; void* out; int64_t n_seg, stride, first, rows; } parts[] = {
      {lv.k_ret, lv.ks_ret, k_ret_out, (int64_t)lv.batch * lv.n_ret, lv.max_seq, first_ret_row, len - first_ret_row},
      {lv.v_ret, lv.vs_ret, v_ret_out, (int64_t)lv.batch * lv.n_ret, lv.max_seq, first_ret_row, len - first_ret_row},
      {lv.k_str, lv.ks_str, k_str_out, (int64_t)lv.batch * lv.n_str, cap, 0, str_rows},
      {lv.v_str, lv.vs_str, v_str_out, (int64_t)lv.batch * lv.n_str, cap, 0, str_rows}};
  for (auto& p : parts) {
    const int64_t pieces = p.n_seg * p.rows * (lv.head_dim / 8);
    if (pieces <= 0) continue;
    if (!p.out) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((pieces + 255) / 256)), block(256);
    uint4* out = (uint4*)p.out;
    if (lv.kv_mode == 1) dequant_kernel<1><<<grid, block, 0, stream>>>(p.codes, p.params, out, lv.head_dim, p.n_seg, p.stride, p.first, p.rows);
    else if (lv.kv_mode == 2) dequant_kernel<2><<<grid, block, 0, stream>>>(p.codes, p.params, out, lv.head_dim, p.n_seg, p.stride, p.first, p.rows);
    else dequant_kernel<3><<<grid, block, 0, stream>>>(p.codes, p.params, out, lv.head_dim, p.n_seg, p.stride, p.first, p.rows);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_append(const LayerView& lv, const void* k, const void* v, int64_t pos0, int n_new,
                         hipStream_t stream) {
  const int64_t total_rows = (int64_t)lv.batch * n_new * lv.n_kv_heads;
  const int lpr = lv.head_dim / 8;
  const int rows_per_block = 256 / lpr;
  const int64_t blocks = (total_rows + rows_per_block - 1) / rows_per_block;
  dim3 grid((unsigned)blocks), block(256);
  const uint4* kk = (const uint4*)k;
  const uint4* vv = (const uint4*)v;
#define DUO_APPEND(D_, M_) append_kernel<D_, M_><<<grid, block, 0, stream>>>(lv, kk, vv, pos0, n_new, total_rows)
  if (lv.kv_mode < 0 || lv.kv_mode > 3) return hipErrorInvalidValue;
  if (lv.head_dim == 128) {
    if (lv.kv_mode == 3) DUO_APPEND(128, 3);
    else if (lv.kv_mode == 2) DUO_APPEND(128, 2);
    else if (lv.kv_mode == 1) DUO_APPEND(128, 1);
    else DUO_APPEND(128, 0);
  } else {
    if (lv.kv_mode == 3) DUO_APPEND(64, 3);
    else if (lv.kv_mode == 2) DUO_APPEND(64, 2);
    else if (lv.kv_mode == 1) DUO_APPEND(64, 1);
    else DUO_APPEND(64, 0);
  }
#undef DUO_APPEND
  return hipGetLastError();
}

hipError_t launch_export(const LayerView& lv, int batch_idx, int kv_head, int64_t len, void* k_out, void* v_out,
                         float* ks_out, float* vs_out, int64_t* pos_out, int64_t count, hipStream_t stream) {
  const int words_per_row = lv.row_bytes / 4;
  const int rows_per_block = 256 / words_per_row;
  const int64_t blocks = (count + rows_per_block - 1) / rows_per_block;
  export_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(lv, batch_idx, kv_head, len, (uint8_t*)k_out,
                                                                   (uint8_t*)v_out, ks_out, vs_out, pos_out, count);
  return hipGetLastError();
}

}  // namespace duo
