// Chunked pre-filling attention (paper, Section 2.3, Chunked Pre-filling; masks
// of Section 2.2): the chunk's queries attend to [cached tokens || chunk tokens].
// Retrieval heads use the causal mask; streaming heads the exact Lambda mask
// (sink tokens + a window of `recent` positions ending at the query), so K/V
// tiles outside the mask are never loaded.
//
// Flash-style kernel for CDNA4: one workgroup = 128 query rows of one query head
// (4 wavefronts x 32 rows); K/V tiles of 64 keys staged in LDS; bf16 MFMA
// 32x32x16 for both contractions with fp32 accumulation; online softmax in
// registers.  The score tile is produced transposed (S^T = K Q^T) so that each
// lane owns one query column: row statistics need a single cross-lane exchange,
// and the accumulator registers of S^T are, after conversion to bf16, exactly
// the B operand of O^T += V^T P^T.  V^T fragments come from LDS transpose reads.
//
// Keys are addressed through a "virtual key list" so that both head classes
// share the code: for a retrieval head it is positions 0 .. pos0+n-1 (cache
// rows, then chunk rows); for a streaming head it is the retained sink slots,
// the retained ring slots in position order, then the chunk rows.
#include "duo_internal.h"

namespace duo {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int BM = 128;  // query rows per workgroup
constexpr int BN = 64;   // keys per tile

// Where the keys of one (sequence, KV head) come from.
struct KeySource {
  const uint8_t* k_cache;  // first cache row of this head
  const uint8_t* v_cache;
  const uint8_t* k_chunk;  // chunk row 0 of this head
  const uint8_t* v_chunk;
  int64_t chunk_stride;    // bytes between chunk rows
  int64_t pos0;
  int64_t n_head;          // list entries [0, n_head) are positions 0 .. n_head-1
  int64_t tail_pos;        // list entry n_head + x is position tail_pos + x
  int64_t total;           // list length
  int32_t sink, recent;
  bool retrieval;

  __device__ inline int64_t position(int64_t u) const { return u < n_head ? u : tail_pos + (u - n_head); }
  __device__ inline void rows(int64_t p, int row_bytes, const uint8_t*& kr, const uint8_t*& vr) const {
    if (p >= pos0) {
      kr = k_chunk + (p - pos0) * chunk_stride;
      vr = v_chunk + (p - pos0) * chunk_stride;
    } else {
      int64_t slot = p;
      if (!retrieval && p >= sink) slot = sink + (p - sink) % recent;
      kr = k_cache + slot * row_bytes;
      vr = v_cache + slot * row_bytes;
    }
  }
};

template <int D>
__global__ __launch_bounds__(256) void prefill_kernel(PrefillArgs a) {
  constexpr int KSTR = D * 2 + 16;  // LDS row strides chosen against bank conflicts
  constexpr int VSTR = D * 2 + 64;
  constexpr int NKK = D / 16;       // MFMA k-steps of the QK^T contraction
  constexpr int NMB = D / 32;       // 32-row blocks of O^T
  constexpr int CPR = D / 8;        // 16-byte pieces per row
  __shared__ __attribute__((aligned(16))) uint8_t k_lds[BN * KSTR];
  __shared__ __attribute__((aligned(16))) uint8_t v_lds[BN * VSTR];

  const LayerView& lv = a.lv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int n_rb = (a.n + BM - 1) / BM;
  const int h = lv.q_order[blockIdx.x / n_rb];
  const int rb = n_rb - 1 - (int)(blockIdx.x % n_rb);   // longest rows first
  const int b = blockIdx.y;
  const int kvh = h / lv.group;
  const uint32_t info = lv.head_info[kvh];
  const int slot_head = (int)(info & ~kRetrievalBit);

  KeySource ks;
  ks.retrieval = (info & kRetrievalBit) != 0;
  ks.pos0 = a.pos0;
  ks.sink = lv.sink; ks.recent = lv.recent;
  ks.chunk_stride = (int64_t)lv.n_kv_heads * D * 2;
  ks.k_chunk = (const uint8_t*)a.k + ((int64_t)b * a.n * lv.n_kv_heads + kvh) * D * 2;
  ks.v_chunk = (const uint8_t*)a.v + ((int64_t)b * a.n * lv.n_kv_heads + kvh) * D * 2;
  if (ks.retrieval) {
    const int64_t row0 = ((int64_t)b * lv.n_ret + slot_head) * lv.max_seq;
    ks.k_cache = lv.k_ret + row0 * lv.row_bytes;
    ks.v_cache = lv.v_ret + row0 * lv.row_bytes;
    ks.n_head = a.pos0 + a.n; ks.tail_pos = ks.n_head; ks.total = ks.n_head;
  } else {
    const int64_t row0 = ((int64_t)b * lv.n_str + slot_head) * ((int64_t)lv.sink + lv.recent);
    ks.k_cache = lv.k_str + row0 * lv.row_bytes;
    ks.v_cache = lv.v_str + row0 * lv.row_bytes;
    const int64_t n_head = a.pos0 < lv.sink ? a.pos0 : lv.sink;
    const int64_t tail = a.pos0 - lv.recent > n_head ? a.pos0 - lv.recent : n_head;
    ks.n_head = n_head; ks.tail_pos = tail; ks.total = n_head + (a.pos0 + a.n - tail);
  }

  // Rows of this workgroup / wavefront / lane.
  const int i_first = rb * BM;
  const int i_last = (i_first + BM < a.n ? i_first + BM : a.n) - 1;
  const int64_t qpos_first = a.pos0 + i_first, qpos_last = a.pos0 + i_last;
  const int ci = i_first + wave * 32 + col;         // chunk index of this lane's query
  const int ci_c = ci < a.n ? ci : a.n - 1;
  const int64_t qpos = a.pos0 + ci_c;
  const int64_t wave_qpos0 = a.pos0 + i_first + wave * 32;

  // Tile ranges: [0, tA_end) covers the sink part, [tB_begin, t_end) the window.
  int64_t tA_end, tB_begin, t_end;
  if (ks.retrieval) {
    tA_end = 0; tB_begin = 0; t_end = qpos_last / BN + 1;
  } else {
    const int64_t usink = (int64_t)lv.sink < qpos_last + 1 ? lv.sink : qpos_last + 1;
    tA_end = (usink + BN - 1) / BN;
    int64_t plo = qpos_first - lv.recent + 1;
    if (plo < 0) plo = 0;
    const int64_t u_lo = plo < ks.tail_pos ? (plo < ks.n_head ? plo : ks.n_head) : ks.n_head + (plo - ks.tail_pos);
    const int64_t u_hi = qpos_last < ks.n_head ? qpos_last : ks.n_head + (qpos_last - ks.tail_pos);
    tB_begin = u_lo / BN;
    if (tB_begin < tA_end) tB_begin = tA_end;
    t_end = u_hi / BN + 1;
    if (t_end < tA_end) t_end = tA_end;
  }

  // Q^T fragments (B operand): lane (col, half) holds q[ci][16*kk + 8*half .. +7].
  bf16x8 qf[NKK];
  {
    const uint8_t* qrow = (const uint8_t*)a.q + (((int64_t)b * a.n + ci_c) * lv.n_q_heads + h) * D * 2;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) qf[kk] = *(const bf16x8*)(qrow + (16 * kk + 8 * half) * 2);
  }
  f32x16 o_acc[NMB];
#pragma unroll
  for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[mb][r] = 0.f;
  float m_i = -INFINITY, l_i = 0.f;
  const float sc = lv.scale * kLog2e;

  for (int64_t t = 0; t < t_end; ++t) {
    if (t == tA_end && t < tB_begin) t = tB_begin;
    __syncthreads();
    // Stage the tile: each thread moves 16-byte pieces of K and V rows.
#pragma unroll
    for (int pass = 0; pass < BN * CPR / 256; ++pass) {
      const int row = pass * (256 / CPR) + tid / CPR, piece = tid % CPR;
      int64_t u = t * BN + row;
      if (u >= ks.total) u = ks.total - 1;
      const uint8_t *kr, *vr;
      ks.rows(ks.position(u), lv.row_bytes, kr, vr);
      const uint4 kc = *(const uint4*)(kr + piece * 16);
      const uint4 vc = *(const uint4*)(vr + piece * 16);
      *(uint4*)(k_lds + row * KSTR + piece * 16) = kc;
      *(uint4*)(v_lds + row * VSTR + piece * 16) = vc;
    }
    __syncthreads();

    // S^T = K Q^T : two 32-key blocks x 32 queries.
    f32x16 s_acc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s_acc[kb][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        const bf16x8 kf = *(const bf16x8*)(k_lds + (32 * kb + col) * KSTR + (16 * kk + 8 * half) * 2);
        s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s_acc[kb], 0, 0, 0);
      }
    }
    // Mask (only tiles that touch the mask boundary or the end of the list).
    const bool need_mask = !ks.retrieval || (t * BN + BN - 1 > wave_qpos0) || (t * BN + BN > ks.total);
    if (need_mask) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t u = t * BN + 32 * kb + 8 * (r / 4) + 4 * half + (r % 4);
          const int64_t p = ks.position(u);
          const bool vis = u < ks.total && p <= qpos && (ks.retrieval || p < lv.sink || qpos - p < lv.recent);
          if (!vis) s_acc[kb][r] = -INFINITY;
        }
    }
    // Online softmax for this lane's query column.
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_acc[kb][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_i, mx * sc);
    const float mu = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = exp2f(m_i - mu);
    m_i = m_new;
    float psum = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = exp2f(fmaf(s_acc[kb][r], sc, -mu));
        psum += p;
        pf[kb * 2 + r / 8][r % 8] = (__bf16)p;
      }
    l_i = l_i * alpha + psum;
    if (__ballot(alpha != 1.0f) != 0) {
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[mb][r] *= alpha;
    }
    // O^T += V^T P^T.  Slab sl covers keys 16*sl + {4*half + t, 8 + 4*half + t}.
    {
      const int blk = lane >> 4, l16 = lane & 15;
      const int e = l16 >> 2, i4 = l16 & 3;
      const int dcol = 16 * (blk & 1) + 4 * i4;   // within the 32-row block of O^T
#pragma unroll
      for (int sl = 0; sl < 4; ++sl) {
        const int key0 = 16 * sl + 4 * half + e;
#pragma unroll
        for (int mb = 0; mb < NMB; ++mb) {
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              LDS_PTR(s16x4, v_lds + key0 * VSTR + (32 * mb + dcol) * 2));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              LDS_PTR(s16x4, v_lds + (key0 + 8) * VSTR + (32 * mb + dcol) * 2));
          const s16x8 vv = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o_acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), pf[sl], o_acc[mb], 0, 0, 0);
        }
      }
    }
  }

  // Normalise and store.  Lane (col, half) holds O^T rows 32*mb + 8*bq + 4*half + t.
  const float l_tot = l_i + __shfl_xor(l_i, 32);
  const float inv = 1.0f / l_tot;
  if (ci < a.n) {
    uint8_t* orow = (uint8_t*)a.out + (((int64_t)b * a.n + ci) * lv.n_q_heads + h) * D * 2;
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
      for (int bq = 0; bq < 4; ++bq) {
        bf16x4 w;
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) w[t4] = (__bf16)(o_acc[mb][4 * bq + t4] * inv);
        *(bf16x4*)(orow + (32 * mb + 8 * bq + 4 * half) * 2) = w;
      }
    if (a.lse && half == 0) a.lse[((int64_t)b * lv.n_q_heads + h) * a.n + ci] = (m_i + log2f(l_tot)) * kLn2;
  }
}

}  // namespace

hipError_t launch_prefill(const PrefillArgs& a, hipStream_t stream) {
  const int n_rb = (a.n + BM - 1) / BM;
  dim3 grid((unsigned)(n_rb * a.lv.n_q_heads), a.lv.batch);
  if (a.lv.head_dim == 128) prefill_kernel<128><<<grid, 256, 0, stream>>>(a);
  else prefill_kernel<64><<<grid, 256, 0, stream>>>(a);
  return hipGetLastError();
}

}  // namespace duo
