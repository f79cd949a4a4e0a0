// Decode attention on the matrix cores, with an even split of all cache rows
// over the workgroups (paper, Section 2.3, Decoding; attention definitions of
// Section 2.2).
//
// One decoding step reads every cached K and V row of the retrieval heads and at
// most sink + recent rows of the streaming heads once: HBM-bound.  The design
// keeps the arithmetic per byte small and the number of bytes in flight large:
//   - Work split.  The rows of all retrieval (sequence, KV head) "segments" are cut
//     into units of 32 rows and the units are dealt out evenly and contiguously
//     to W workgroups, whatever the head count, batch and context length.  A
//     workgroup whose range crosses a segment border handles both pieces; a
//     segment handled by several workgroups is merged by the last of them to
//     finish (ticket per segment, fixed merge order: deterministic).  Every
//     streaming segment (at most sink + recent rows) has a workgroup of its own.
//   - Arithmetic.  The G query heads of a KV head form the (padded) 16-wide side
//     of 16x16x32 bf16 matrix-core products: S^T = K Q^T for 16 keys at a time,
//     O^T += V^T P^T for 32 keys at a time.  A lane owns one head column, so the
//     scores come out exactly where the probabilities are needed as the second
//     product's operand, and a lane's accumulators all belong to one head.
//     The running maximum is only re-synchronised across lanes when some score
//     exceeds it (rare after the first blocks).
//   - Data movement.  K goes from global memory straight into the matrix-core
//     operand registers; V is staged through a wavefront-private LDS buffer
//     (swizzled rows) and read back transposed.  Each wavefront works on its own
//     32-row blocks with the loads of the next three blocks in flight (one
//     workgroup per compute unit, registers instead of occupancy); no workgroup
//     barrier in the main loop.
//   - fp8 caches: codes are widened to bf16 on the way (exact), the K scale
//     multiplies the score and the V scale the probability of its key.
//   - int4 caches (value = code * scale + lo per row): a code c becomes the bf16
//     value 128 + c by OR-ing its nibble into 0x4300, two codes per instruction.
//     The K product starts from -128 sum_d q_d, so it yields A = sum_d q_d c_d and
//     the score is scale_k A + lo_k sum_d q_d.  With p' = bf16(p scale_v) the
//     output is sum_key p' (128 + c) (matrix core) + sum_key p (lo_v + 7.5 scale_v)
//     - 135.5 sum_key p', the last two one scalar per head (the sum of p' as
//     rounded comes from a product with a row of ones): taking the codes' midpoint
//     out this way leaves the rounding of p' acting on c - 7.5 only.  The nibble
//     extraction leaves the eight values of a dword in the order 0 4 1 5 2 6 3 7;
//     the query operand (for K) and the probability operand (for V) are permuted
//     to match, so no instruction is spent on order.  V rows are staged in LDS as
//     codes and come back through the 4-bit transposing read, sixteen d by sixteen
//     (key, row block) pairs per lane group and read.
//   - int8 caches: the same algebra with the codes 0 .. 255 themselves as bf16
//     operands (exact), widened like the fp8 codes, and 127.5 as the midpoint.
#include "duo_internal.h"

#include <type_traits>

namespace duo {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kUnit = kDecodeUnitRows;   // rows per unit = rows per wavefront block

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// Cache rows are read once per launch.  Non-temporal loads stream them past the caches, which on
// this part moves a plain read of a large buffer from 6.3 to 7.1 TB/s (stand-alone probe) - for
// loads that cover whole cache lines.  The V rows of a block are one contiguous run (1 KiB per
// wavefront load) and take them; a K load fetches 32 or 64 bytes of each of 16 rows, two loads
// share a line, and streaming those was slower than caching them (measured both ways), so K
// loads stay ordinary.  The per-row parameters are small contiguous runs and stream as well.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2s_t __attribute__((ext_vector_type(2)));
__device__ inline uint4 stream_load16(const void* p) {
  const u32x4_t x = __builtin_nontemporal_load((const u32x4_t*)p);
  return make_uint4(x[0], x[1], x[2], x[3]);
}
__device__ inline float2 stream_load_f2(const float2* p) {
  const f32x2s_t x = __builtin_nontemporal_load((const f32x2s_t*)p);
  return make_float2(x[0], x[1]);
}
__device__ inline float stream_load_f(const float* p) { return __builtin_nontemporal_load(p); }

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ inline uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ inline int uniform_load(const int32_t* p) {
  return *(const __attribute__((address_space(4))) int32_t*)(uintptr_t)p;
}
__device__ inline void coherent_store(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Four E4M3 codes (one dword) -> four bf16 values (two dwords); exact (every E4M3 value has at
// most 4 significant bits).  The scaled conversion of this architecture turns two codes into a
// bf16 pair in one instruction; with a scale of one it gives, for every code, the bits of the
// conversion through fp32 (checked over all code pairs).
__device__ inline uint2 e4m3x4_to_bf16x4(uint32_t w) {
  const bf16x2 lo = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
  const bf16x2 hi = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true);
  uint2 r;
  r.x = __builtin_bit_cast(uint32_t, lo);
  r.y = __builtin_bit_cast(uint32_t, hi);
  return r;
}

// Eight 4-bit codes (one dword, code j at bits 4 j) -> eight bf16 values 128 + code as four
// dwords holding the code pairs (0,4) (1,5) (2,6) (3,7).
__device__ inline uint4 int4x8_to_bf16x8(uint32_t w) {
  constexpr uint32_t kMask = 0x000F000Fu;
  // bf16 0x4300 = 128, one ulp = 1.  The bias passes through an empty asm statement so that the
  // compiler keeps it in a vector register and can fuse each mask-and-bias into one v_and_or_b32
  // (with two literal constants it emits the two operations separately).  The fused instruction
  // itself is left to the compiler: it knows the wait states between it and the matrix-core
  // instructions that read its result, which it cannot know for an instruction inside an asm.
  uint32_t bias = 0x43004300u;
  asm volatile("" : "+v"(bias));
  uint4 r;
  r.x = (w & kMask) | bias;
  r.y = ((w >> 4) & kMask) | bias;
  r.z = ((w >> 8) & kMask) | bias;
  r.w = ((w >> 12) & kMask) | bias;
  return r;
}

// Four 8-bit codes (one dword) -> four bf16 values 0 .. 255 (two dwords); exact: an integer below
// 256 has at most 8 significant bits, so the upper half of its float is the bf16 value.
__device__ inline uint2 u8x4_to_bf16x4(uint32_t w) {
  const float f0 = (float)(w & 0xFFu), f1 = (float)((w >> 8) & 0xFFu);
  const float f2 = (float)((w >> 16) & 0xFFu), f3 = (float)(w >> 24);
  uint2 r;
  r.x = __builtin_amdgcn_perm(__float_as_uint(f1), __float_as_uint(f0), 0x07060302u);
  r.y = __builtin_amdgcn_perm(__float_as_uint(f3), __float_as_uint(f2), 0x07060302u);
  return r;
}

// MODE: 0 bf16 rows, 1 fp8 codes + scale, 2 int4 / 3 int8 codes + (scale, lo).
template <int D, int MODE>
struct Shape {
  static constexpr int NKK = D / 32;                 // matrix-core k-steps of K Q^T
  static constexpr int NMB = D / 16;                 // 16-row blocks of O^T
  static constexpr int LROW = D * 2;                 // bytes of a (bf16) V row in LDS
  static constexpr int CPR = D / 8;                  // 16-byte pieces per LDS row
  static constexpr int GROW = MODE == 2 ? D / 2 : (MODE == 0 ? D * 2 : D);   // bytes of a row in the cache
  static constexpr int VPR = GROW / 16;              // 16-byte pieces per cache row
  static constexpr int VRPI = 64 / VPR;              // V rows covered by one wavefront load
  static constexpr int NV = kUnit / VRPI;            // V loads per lane and block
  static constexpr int KB = MODE == 2 ? 4 : (MODE == 0 ? 16 : 8);   // bytes of K per lane, 16-key group and k-step
  static constexpr int NSC = MODE >= 2 ? 2 : 1;      // floats per row in the scale arrays
  __device__ static inline int v_swz(int row) { return (2 * row) % CPR; }
  // Slot (16-byte unit within the LDS row) of piece `piece` of staged V row `row`.  bf16 rows: the piece
  // index XOR an even row swizzle, which spreads the four rows one transposing read touches over the
  // banks.  One-byte codes at D = 128 are widened by the lane that loaded them into two neighbouring
  // pieces (2 pc, 2 pc + 1), written by two stores; with the plain layout each store of the eight lanes
  // of a row hits every second slot, i.e. half the banks twice (36 % of this mode's LDS cycles were
  // bank conflicts).  Here piece 2 pc + h goes to slot (pc ^ 4h) + 8h, XOR a row term: a store covers
  // eight neighbouring slots, a read's two pieces (h = 0, 1) still differ in the bank-selecting bits,
  // the row term's low bits separate the four rows of a read and its bit 3 alternates between
  // neighbouring rows.  Conflict-free for 32 banks x 4 bytes and for 64.
  __device__ static inline int v_slot(int row, int piece) {
    if constexpr ((MODE == 1 || MODE == 3) && D == 128) {
      const int rterm = (row & 3) | (((row ^ (row >> 2)) & 1) << 3);
      return (piece >> 1) ^ (12 * (piece & 1)) ^ rterm;
    } else {
      return piece ^ v_swz(row);
    }
  }
  // int4: V rows are staged as codes (GROW bytes a row); 16-byte pieces swizzled so that the rows one
  // transposing read touches (keys 4 qd + r and 16 + 4 qd + r) spread over the banks
  __device__ static inline int c_swz(int row) { return (((row >> 2) & 1) * 2 + ((row >> 4) & 1)) % VPR; }
};

// Raw registers of one 32-row block as loaded from the cache.
template <int D, int MODE>
struct RawBlock {
  using S = Shape<D, MODE>;
  uint32_t k[2][S::NKK][S::KB / 4];
  uint4 v[S::NV];
  float sc[S::NSC];   // quantised: K parameters of row `lane` (lanes 0..31) or V parameters of row `lane - 32`
};

// Per-key dequantisation parameters of a block in the lane's key order (keys 16 t + 4 qd + r at
// index 4 t + r), with the softmax scale c = scale * log2(e) folded in.  fp8: ks = c * scale_k,
// vs = scale_v.  int4: ks = c * scale_k, klo = c * lo_k, vs = scale_v, vlo = lo_v + 7.5 scale_v.
struct KeyParams {
  float ks[8], klo[8], vs[8], vlo[8];
};

template <int D, int MODE>
__global__ __launch_bounds__(256, 1) void decode_sk_kernel(DecodeArgs a) {
  using S = Shape<D, MODE>;
  constexpr bool FP8 = MODE == 1, INT4 = MODE == 2, INT8 = MODE == 3, QUANT = MODE != 0;
  constexpr bool ASYM = INT4 || INT8;    // integer codes with (scale, lo) per row
  constexpr bool BYTES = FP8 || INT8;    // one byte per element
  // the matrix-core operands of integer codes are kOff + code (128 + nibble by the OR trick, the
  // byte itself); kMid is the middle of the code range
  constexpr float kOff = INT4 ? 128.f : 0.f, kMid = INT4 ? 7.5f : 127.5f;
  constexpr int NKK = S::NKK, NMB = S::NMB, LROW = S::LROW, GROW = S::GROW;
  constexpr int NBUF = INT4 ? 6 : 3;   // blocks of loads in flight per wavefront
  const LayerView& lv = a.lv;
  const int G = lv.group;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: block addresses stay uniform
  const int hd = lane & 15, qd = lane >> 4;
  const bool head_ok = hd < G;

  // LDS: per-wavefront V staging; later reused for the merges.
  __shared__ __attribute__((aligned(16))) uint8_t sm_v[4][kUnit * LROW];
  __shared__ __attribute__((aligned(16))) float sm_sc[4][64 * S::NSC];
  __shared__ __attribute__((aligned(16))) uint16_t sm_new[2][D];
  __shared__ float sm_m[4][16], sm_l[4][16], sm_m2[16], sm_l2[16];
  __shared__ int sm_last;
  float* sm_o = (float*)&sm_v[0][0];   // [wave][head][D] or [slot][D]: 4 * 16 * D floats at most
  uint8_t* my_v = &sm_v[wave][0];

  // Workgroups 0 .. W-1 share the units of the retrieval segments evenly; each streaming segment
  // (at most sink + recent rows) has a workgroup of its own after them.
  const int64_t n_ret_seg = (int64_t)lv.batch * lv.n_ret;
  const int64_t ret_units_all = n_ret_seg * a.units_ret;
  const int64_t T = ret_units_all, W = a.ret_workers;
  int64_t u_lo, u_hi;
  if ((int64_t)blockIdx.x < W) {
    u_lo = (int64_t)blockIdx.x * T / W;
    u_hi = ((int64_t)blockIdx.x + 1) * T / W;
  } else {
    u_lo = ret_units_all + ((int64_t)blockIdx.x - W) * a.units_str;
    u_hi = u_lo + a.units_str;
  }
  const float c_scale = lv.scale * kLog2e;

  for (int64_t u = u_lo; u < u_hi;) {
    // ---- the segment that owns unit u
    int64_t seg, seg_a;
    int seg_units, b, slot, kvh;
    int64_t n_rows, exclude = -1, new_row;
    uint8_t *kbase, *vbase;
    float *ksbase = nullptr, *vsbase = nullptr;
    const bool retrieval = u < ret_units_all;
    if (retrieval) {
      seg = u / a.units_ret;
      seg_a = seg * a.units_ret;
      seg_units = a.units_ret;
      b = (int)(seg / lv.n_ret); slot = (int)(seg % lv.n_ret);
      kvh = uniform_load(lv.ret_heads + slot);
      n_rows = a.cache_len;
      new_row = a.cache_len;
      const int64_t head_row0 = ((int64_t)b * lv.n_ret + slot) * lv.max_seq;
      kbase = lv.k_ret + head_row0 * GROW;
      vbase = lv.v_ret + head_row0 * GROW;
      if (QUANT) { ksbase = lv.ks_ret + head_row0 * S::NSC; vsbase = lv.vs_ret + head_row0 * S::NSC; }
    } else {
      const int64_t s2 = (u - ret_units_all) / a.units_str;
      seg = n_ret_seg + s2;
      seg_a = ret_units_all + s2 * a.units_str;
      seg_units = a.units_str;
      b = (int)(s2 / lv.n_str); slot = (int)(s2 % lv.n_str);
      kvh = uniform_load(lv.str_heads + slot);
      const int64_t cap = (int64_t)lv.sink + lv.recent;
      n_rows = streaming_rows(a.cache_len, lv.sink, lv.recent);
      // The slot the new token goes to: while it is not yet written, that slot of a
      // full ring still holds the token the append evicts, which the query at
      // position cache_len must not see.
      new_row = a.cache_len < lv.sink ? a.cache_len : lv.sink + (a.cache_len - lv.sink) % lv.recent;
      if (a.k_new != nullptr && a.cache_len >= cap) exclude = new_row;
      const int64_t head_row0 = ((int64_t)b * lv.n_str + slot) * cap;
      kbase = lv.k_str + head_row0 * GROW;
      vbase = lv.v_str + head_row0 * GROW;
      if (QUANT) { ksbase = lv.ks_str + head_row0 * S::NSC; vsbase = lv.vs_str + head_row0 * S::NSC; }
    }
    const int64_t seg_e = seg_a + seg_units;
    const int64_t part_e = u_hi < seg_e ? u_hi : seg_e;
    const int64_t row0 = (u - seg_a) * kUnit;                      // first row of this workgroup's part
    int64_t row1 = (part_e - seg_a) * kUnit;                       // end of the part, clipped to the rows present
    if (row1 > n_rows) row1 = n_rows;
    const int nb = row1 > row0 ? (int)((row1 - row0 + kUnit - 1) / kUnit) : 0;
    const bool with_new = a.k_new != nullptr && part_e == seg_e;   // the part that ends the segment owns the new token
    const int64_t last_row = n_rows > 0 ? n_rows - 1 : 0;

    // ---- query operand: lane (hd, qd) holds q[head hd][32 kk + 8 qd .. + 7]; for an int4 cache,
    // whose lanes load D/4 consecutive codes of a key, q[head hd][(D/4) qd + 8 kk + sigma(0..7)]
    bf16x8 qf[NKK];
    float qsum = 0.f;   // integer codes: sum_d q[head hd][d]
    {
      const uint16_t* qrow = (const uint16_t*)a.q + ((int64_t)b * lv.n_q_heads + (int64_t)kvh * G + (head_ok ? hd : 0)) * D;
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        uint4 raw = *(const uint4*)(qrow + (INT4 ? (D / 4) * qd + 8 * kk : 32 * kk + 8 * qd));
        if (!head_ok) raw = make_uint4(0, 0, 0, 0);
        if constexpr (ASYM) {
          const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) qsum += __uint_as_float(w[i] << 16) + __uint_as_float(w[i] & 0xFFFF0000u);
        }
        if constexpr (INT4) {
          raw = make_uint4(__builtin_amdgcn_perm(raw.z, raw.x, 0x05040100u), __builtin_amdgcn_perm(raw.z, raw.x, 0x07060302u),
                           __builtin_amdgcn_perm(raw.w, raw.y, 0x05040100u), __builtin_amdgcn_perm(raw.w, raw.y, 0x07060302u));
        }
        qf[kk] = __builtin_bit_cast(bf16x8, raw);
      }
      if constexpr (ASYM) {
        qsum += __shfl_xor(qsum, 16);
        qsum += __shfl_xor(qsum, 32);
      }
    }

    // ---- per-wavefront online-softmax state
    f32x4 oacc[NMB];
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb) oacc[mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m_ref = -INFINITY, l_lane = 0.f;
    // int4: corr_lane = sum over the lane's keys of p (lo_v + 7.5 scale_v); pb_sum = sum over all
    // keys of the head of bf16(p scale_v) as rounded (a matrix-core product with a row of ones)
    float corr_lane = 0.f;
    f32x4 pb_sum = (f32x4){0.f, 0.f, 0.f, 0.f};

    using Raw = RawBlock<D, MODE>;
    // Loads of a block whose 32 rows are all present: a uniform block address plus per-lane
    // offsets that never change (K: row hd of each 16-key group, piece qd + 4 kk; V: the block's
    // rows are one contiguous run, 16 bytes per lane and load).
    const uint32_t k_off = (uint32_t)(hd * GROW + qd * (INT4 ? D / 8 : S::KB));
    const uint32_t v_off = (uint32_t)(lane * 16);
    // int4: the D/8 bytes of one key that belong to this lane, all k-steps in one load
    auto load_k_int4 = [&](Raw& rb, int t, const uint8_t* p) {
      if constexpr (D == 128) {
        const uint4 x = *(const uint4*)p;
        rb.k[t][0][0] = x.x; rb.k[t][1][0] = x.y; rb.k[t][2][0] = x.z; rb.k[t][3][0] = x.w;
      } else {
        const uint2 x = *(const uint2*)p;
        rb.k[t][0][0] = x.x; rb.k[t][1][0] = x.y;
      }
    };
    auto issue = [&](Raw& rb, int blk) {
      const int64_t r0 = row0 + (int64_t)blk * kUnit;
      const uint8_t* kb = kbase + r0 * GROW;
      const uint8_t* vb = vbase + r0 * GROW;
#pragma unroll
      for (int t = 0; t < 2; ++t)
        if constexpr (INT4) {
          load_k_int4(rb, t, kb + (k_off + (uint32_t)(16 * t * GROW)));
        } else {
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
          const uint8_t* p = kb + (k_off + (uint32_t)(16 * t * GROW + 4 * kk * S::KB));
          if constexpr (BYTES) {
            const uint2 x = *(const uint2*)p;
            rb.k[t][kk][0] = x.x; rb.k[t][kk][1] = x.y;
          } else {
            const uint4 x = *(const uint4*)p;
            rb.k[t][kk][0] = x.x; rb.k[t][kk][1] = x.y; rb.k[t][kk][2] = x.z; rb.k[t][kk][3] = x.w;
          }
        }
        }
#pragma unroll
      for (int j = 0; j < S::NV; ++j) rb.v[j] = stream_load16(vb + (v_off + (uint32_t)(j * 1024)));
      if constexpr (FP8) rb.sc[0] = stream_load_f((lane < 32 ? ksbase : vsbase) + (r0 + (lane & 31)));
      if constexpr (ASYM) {
        const float2 x = stream_load_f2((const float2*)(lane < 32 ? ksbase : vsbase) + (r0 + (lane & 31)));
        rb.sc[0] = x.x; rb.sc[1] = x.y;
      }
    };
    // The same for the last, partly filled block of a segment: rows past the end are redirected
    // to the last row present (and masked later).
    auto issue_tail = [&](Raw& rb, int blk) {
      const int64_t r0 = row0 + (int64_t)blk * kUnit;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        int64_t r = r0 + 16 * t + hd;
        r = r < n_rows ? r : last_row;
        const uint8_t* kr = kbase + r * GROW;
        if constexpr (INT4) load_k_int4(rb, t, kr + qd * (D / 8));
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
          if constexpr (INT4) {
          } else if constexpr (BYTES) {
            const uint2 x = *(const uint2*)(kr + (qd + 4 * kk) * 8);
            rb.k[t][kk][0] = x.x; rb.k[t][kk][1] = x.y;
          } else {
            const uint4 x = *(const uint4*)(kr + (qd + 4 * kk) * 16);
            rb.k[t][kk][0] = x.x; rb.k[t][kk][1] = x.y; rb.k[t][kk][2] = x.z; rb.k[t][kk][3] = x.w;
          }
        }
      }
#pragma unroll
      for (int j = 0; j < S::NV; ++j) {
        int64_t r = r0 + j * S::VRPI + lane / S::VPR;
        r = r < n_rows ? r : last_row;
        rb.v[j] = stream_load16(vbase + r * GROW + (lane % S::VPR) * 16);
      }
      if constexpr (QUANT) {
        int64_t r = r0 + (lane & 31);
        r = r < n_rows ? r : last_row;
        if constexpr (ASYM) {
          const float2 x = ((const float2*)(lane < 32 ? ksbase : vsbase))[r];
          rb.sc[0] = x.x; rb.sc[1] = x.y;
        } else {
          rb.sc[0] = (lane < 32 ? ksbase : vsbase)[r];
        }
      }
    };

    // S^T = K Q^T for the two 16-key groups of a block.
    auto qk = [&](const bf16x8 (&kf)[2][NKK], f32x4 (&sacc)[2]) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        // int4 operands are 128 + code: start from -128 sum(q), so the result is sum(q code)
        const float s0 = -kOff * qsum;
        sacc[t] = (f32x4){s0, s0, s0, s0};
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
          sacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][kk], qf[kk], sacc[t], 0, 0, 0);
      }
    };
    // Softmax update and O^T += V^T P^T of one block whose V rows are staged in my_v (bf16).
    // key_base: row index of the block's first key; with `masked`, keys >= valid_end, the excluded
    // key and the padding heads are masked; without, every key of the block is visible (the padding
    // heads then carry finite values that are never written out).
    auto finish = [&](auto masked, const f32x4 (&sacc)[2], const KeyParams& kp, int64_t key_base, int64_t valid_end) {
      float sv[8];
      float lmax = -INFINITY;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float s;
          if constexpr (ASYM) {
            s = sacc[t][r] * kp.ks[4 * t + r] + kp.klo[4 * t + r] * qsum;
          } else if constexpr (FP8) {
            s = sacc[t][r] * kp.ks[4 * t + r];
          } else {
            s = sacc[t][r] * c_scale;
          }
          if constexpr (decltype(masked)::value) {
            const int64_t key = key_base + 16 * t + 4 * qd + r;
            const bool ok = head_ok && key < valid_end && key != exclude;
            s = ok ? s : -INFINITY;
          }
          sv[4 * t + r] = s;
          lmax = fmaxf(lmax, s);
        }
      if (__ballot(lmax > m_ref) != 0) {
        float mx = fmaxf(lmax, __shfl_xor(lmax, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_ref, mx);
        const float mu = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = fast_exp2(m_ref - mu);
        l_lane *= alpha;
        if constexpr (ASYM) { corr_lane *= alpha; pb_sum *= alpha; }
#pragma unroll
        for (int mb = 0; mb < NMB; ++mb) oacc[mb] *= alpha;
        m_ref = m_new;
      }
      const float mu = m_ref == -INFINITY ? 0.f : m_ref;
      float p[8];
      float psum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) { p[i] = fast_exp2(sv[i] - mu); psum += p[i]; }
      l_lane += psum;
      // int4: the code expansion leaves the eight keys of an operand in the order 0 4 1 5 2 6 3 7
      bf16x8 pb;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int src = INT4 ? (i >> 1) + 4 * (i & 1) : i;
        pb[i] = (__bf16)(QUANT ? p[src] * kp.vs[src] : p[src]);
      }
      if constexpr (ASYM) {
        // the matrix core sums pb * (kOff + code) = pb * (code - kMid) + (kOff + kMid) pb: the second
        // term is taken back at the end exactly as rounded; kp.vlo holds lo + kMid scale
#pragma unroll
        for (int i = 0; i < 8; ++i) corr_lane += p[i] * kp.vlo[i];
        const uint32_t one2 = 0x3F803F80u;
        pb_sum = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, make_uint4(one2, one2, one2, one2)), pb,
                                                         pb_sum, 0, 0, 0);
      }
      if constexpr (INT4) {
        // O^T += V^T P^T from the staged codes.  The 4-bit transposing read hands lane i of a 16-lane
        // group nibble i of the 64 bits each lane e of the group points at, as its nibble e.  Lane e
        // points at the 16 codes of key 16 (j >> 2) + 4 qd + (j & 3), j = e & 7, in the 16-row block
        // 2 mbp + (e >> 3) of O^T: the first dword read is then row block 2 mbp over the lane group's
        // eight keys, the second dword row block 2 mbp + 1, and row i of a block is d = 16 block + i.
        const int j = hd & 7, half = hd >> 3;
        const int key = 16 * (j >> 2) + 4 * qd + (j & 3);
        const uint8_t* rowp = my_v + key * GROW + half * 8;
        const int sw = S::c_swz(key);
#pragma unroll
        for (int mbp = 0; mbp < NMB / 2; ++mbp) {
          const i32x2 t = __builtin_amdgcn_ds_read_tr4_b64_v2i32(LDS_PTR(i32x2, rowp + ((mbp ^ sw) * 16)));
          const bf16x8 v0 = __builtin_bit_cast(bf16x8, int4x8_to_bf16x8((uint32_t)t[0]));
          const bf16x8 v1 = __builtin_bit_cast(bf16x8, int4x8_to_bf16x8((uint32_t)t[1]));
          oacc[2 * mbp] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v0, pb, oacc[2 * mbp], 0, 0, 0);
          oacc[2 * mbp + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v1, pb, oacc[2 * mbp + 1], 0, 0, 0);
        }
        return;
      }
      // O^T += V^T P^T : lane (hd, qd) supplies the address of key 16 h + 4 qd + (hd >> 2), d 16 mb + 4 (hd & 3)
      const int e = hd >> 2, i4 = hd & 3;
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb) {
        const int piece = 2 * mb + (i4 >> 1), sub8 = (i4 & 1) * 8;
        const int key_lo = 4 * qd + e, key_hi = 16 + 4 * qd + e;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            LDS_PTR(s16x4, my_v + key_lo * LROW + (S::v_slot(key_lo, piece) * 16) + sub8));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            LDS_PTR(s16x4, my_v + key_hi * LROW + (S::v_slot(key_hi, piece) * 16) + sub8));
        const bf16x8 vt = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        oacc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, pb, oacc[mb], 0, 0, 0);
      }
    };

    // Convert / stage the raw registers of a block (V rows into the wavefront's LDS buffer, 16-byte
    // pieces swizzled by row; fp8 scales through LDS into key order) and start its arithmetic.
    // After this the raw registers are free for the next block's loads.
    // four one-byte codes -> four bf16 values
    auto widen4 = [&](uint32_t w) { return INT8 ? u8x4_to_bf16x4(w) : e4m3x4_to_bf16x4(w); };
    auto stage_qk = [&](const Raw& rb, f32x4 (&sacc)[2], KeyParams& kp) {
#pragma unroll
      for (int j = 0; j < S::NV; ++j) {
        const int row = j * S::VRPI + lane / S::VPR, pc = lane % S::VPR;
        if constexpr (INT4) {
          *(uint4*)(my_v + row * GROW + ((pc ^ S::c_swz(row)) * 16)) = rb.v[j];   // codes as they are
        } else if constexpr (BYTES) {
          const uint2 a0 = widen4(rb.v[j].x), a1 = widen4(rb.v[j].y);
          const uint2 a2 = widen4(rb.v[j].z), a3 = widen4(rb.v[j].w);
          *(uint4*)(my_v + row * LROW + (S::v_slot(row, 2 * pc) * 16)) = make_uint4(a0.x, a0.y, a1.x, a1.y);
          *(uint4*)(my_v + row * LROW + (S::v_slot(row, 2 * pc + 1) * 16)) = make_uint4(a2.x, a2.y, a3.x, a3.y);
        } else {
          *(uint4*)(my_v + row * LROW + (S::v_slot(row, pc) * 16)) = rb.v[j];
        }
      }
      bf16x8 kf[2][NKK];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
          if constexpr (INT4) {
            kf[t][kk] = __builtin_bit_cast(bf16x8, int4x8_to_bf16x8(rb.k[t][kk][0]));
          } else if constexpr (BYTES) {
            const uint2 x0 = widen4(rb.k[t][kk][0]), x1 = widen4(rb.k[t][kk][1]);
            kf[t][kk] = __builtin_bit_cast(bf16x8, make_uint4(x0.x, x0.y, x1.x, x1.y));
          } else {
            kf[t][kk] = __builtin_bit_cast(bf16x8, make_uint4(rb.k[t][kk][0], rb.k[t][kk][1], rb.k[t][kk][2], rb.k[t][kk][3]));
          }
        }
      qk(kf, sacc);
      if constexpr (ASYM) {
        // [0..31] K scale, [32..63] K lo, [64..95] V scale, [96..127] V lo, each in row order
        // the lane that loaded a row's parameters folds the constants in before sharing them
        const int at = lane < 32 ? lane : lane + 32;
        sm_sc[wave][at] = lane < 32 ? rb.sc[0] * c_scale : rb.sc[0];
        sm_sc[wave][at + 32] = lane < 32 ? rb.sc[1] * c_scale : rb.sc[1] + kMid * rb.sc[0];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const float4 s4 = *(const float4*)&sm_sc[wave][16 * t + 4 * qd];
          const float4 l4 = *(const float4*)&sm_sc[wave][32 + 16 * t + 4 * qd];
          const float4 v4 = *(const float4*)&sm_sc[wave][64 + 16 * t + 4 * qd];
          const float4 o4 = *(const float4*)&sm_sc[wave][96 + 16 * t + 4 * qd];
          kp.ks[4 * t] = s4.x; kp.ks[4 * t + 1] = s4.y; kp.ks[4 * t + 2] = s4.z; kp.ks[4 * t + 3] = s4.w;
          kp.klo[4 * t] = l4.x; kp.klo[4 * t + 1] = l4.y; kp.klo[4 * t + 2] = l4.z; kp.klo[4 * t + 3] = l4.w;
          kp.vs[4 * t] = v4.x; kp.vs[4 * t + 1] = v4.y; kp.vs[4 * t + 2] = v4.z; kp.vs[4 * t + 3] = v4.w;
          kp.vlo[4 * t] = o4.x; kp.vlo[4 * t + 1] = o4.y; kp.vlo[4 * t + 2] = o4.z; kp.vlo[4 * t + 3] = o4.w;
        }
      } else if constexpr (FP8) {
        sm_sc[wave][lane] = lane < 32 ? rb.sc[0] * c_scale : rb.sc[0];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const float4 kq = *(const float4*)&sm_sc[wave][16 * t + 4 * qd];
          const float4 vq = *(const float4*)&sm_sc[wave][32 + 16 * t + 4 * qd];
          kp.ks[4 * t] = kq.x; kp.ks[4 * t + 1] = kq.y; kp.ks[4 * t + 2] = kq.z; kp.ks[4 * t + 3] = kq.w;
          kp.vs[4 * t] = vq.x; kp.vs[4 * t + 1] = vq.y; kp.vs[4 * t + 2] = vq.z; kp.vs[4 * t + 3] = vq.w;
        }
      }
    };

    // ---- main loop: this wavefront's full blocks wave, wave + 4, ...  NBUF sets of raw
    // registers rotate: as soon as a block is staged and its K products are issued, its registers
    // take the loads of the block NBUF turns ahead, so up to NBUF blocks are in flight per
    // wavefront: three of bf16 and one-byte rows (48 and 25 KiB), six of the 4-bit rows, whose
    // blocks are a quarter of the bf16 size (six against three: 2 % faster at 3.3M tokens; four
    // instead of three for the one-byte rows: 1 % slower).  In the steady loop every issue is unconditional, which lets
    // the compiler's wait counts match the real queue; the scheduling barriers keep the loads
    // where they are written.  Then the partly filled last block, if any, by the wavefront whose
    // turn it is.
    const int n_full = (int)((row1 - row0) / kUnit) < nb ? (int)((row1 - row0) / kUnit) : nb;
    auto run_blocks = [&](auto masked) {
      Raw rb[NBUF];
      f32x4 sacc[2];
      KeyParams kp;
      const int n_my = wave < n_full ? (n_full - wave + 3) / 4 : 0;   // blocks of this wavefront
      auto blk_of = [&](int i) { return wave + 4 * i; };
      auto step = [&](Raw& r, int i, bool prefetch) {
        stage_qk(r, sacc, kp);
        __builtin_amdgcn_sched_barrier(0);
        if (prefetch) issue(r, blk_of(i + NBUF));
        __builtin_amdgcn_sched_barrier(0);
        finish(masked, sacc, kp, row0 + (int64_t)blk_of(i) * kUnit, n_rows);
        __builtin_amdgcn_sched_barrier(0);
      };
#pragma unroll
      for (int j = 0; j < NBUF; ++j)
        if (n_my > j) issue(rb[j], blk_of(j));
      __builtin_amdgcn_sched_barrier(0);
      int i = 0;
      while (i + 2 * NBUF - 1 < n_my) {
#pragma unroll
        for (int j = 0; j < NBUF; ++j) step(rb[j], i + j, true);
        i += NBUF;
      }
      while (i < n_my) {
#pragma unroll
        for (int j = 0; j < NBUF; ++j)
          if (i + j < n_my) step(rb[j], i + j, i + j + NBUF < n_my);
        i += NBUF;
      }
      Raw& r0 = rb[0];
      if (n_full < nb && wave == (n_full & 3)) {
        issue_tail(r0, n_full);
        stage_qk(r0, sacc, kp);
        finish(std::true_type{}, sacc, kp, row0 + (int64_t)n_full * kUnit, n_rows);
      }
    };
    // full blocks need no masking unless the segment has an excluded key
    if (exclude < 0) run_blocks(std::false_type{});
    else run_blocks(std::true_type{});

    // ---- the new token (wavefront 0 of the part that ends the segment); with a.commit its rows
    // are also written into the cache
    if (with_new && wave == 0) {
      // row layout: lane i < D/8 owns elements 8 i .. 8 i + 7
      const bool row_lane = lane < D / 8;
      const uint16_t* kin = (const uint16_t*)a.k_new + ((int64_t)b * lv.n_kv_heads + kvh) * D;
      const uint16_t* vin = (const uint16_t*)a.v_new + ((int64_t)b * lv.n_kv_heads + kvh) * D;
      uint4 kc = make_uint4(0, 0, 0, 0), vc = kc;
      if (row_lane) { kc = *(const uint4*)(kin + 8 * lane); vc = *(const uint4*)(vin + 8 * lane); }
      float ks1 = 1.f, vs1 = 1.f, klo1 = 0.f, vlo1 = 0.f;
      if constexpr (ASYM) {
        // quantise exactly as the append kernel does, then attend to the codes like a cached row
        constexpr float kTop = INT4 ? 15.0f : 255.0f;
        constexpr int kBits = INT4 ? 4 : 8;
        const uint32_t kw[4] = {kc.x, kc.y, kc.z, kc.w}, vw[4] = {vc.x, vc.y, vc.z, vc.w};
        float kf4[8], vf4[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          kf4[2 * i] = __uint_as_float(kw[i] << 16); kf4[2 * i + 1] = __uint_as_float(kw[i] & 0xFFFF0000u);
          vf4[2 * i] = __uint_as_float(vw[i] << 16); vf4[2 * i + 1] = __uint_as_float(vw[i] & 0xFFFF0000u);
        }
        float kmin = kf4[0], kmax = kf4[0], vmin = vf4[0], vmax = vf4[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) {
          kmin = fminf(kmin, kf4[i]); kmax = fmaxf(kmax, kf4[i]);
          vmin = fminf(vmin, vf4[i]); vmax = fmaxf(vmax, vf4[i]);
        }
        // the D/8 lanes of the row form an aligned lane group, so the exchange below stays inside it
#pragma unroll
        for (int off = 1; off < D / 8; off <<= 1) {
          kmin = fminf(kmin, __shfl_xor(kmin, off)); kmax = fmaxf(kmax, __shfl_xor(kmax, off));
          vmin = fminf(vmin, __shfl_xor(vmin, off)); vmax = fmaxf(vmax, __shfl_xor(vmax, off));
        }
        const float kspan = kmax - kmin, vspan = vmax - vmin;
        ks1 = kspan == 0.f ? 1.0f : kspan / kTop;
        vs1 = vspan == 0.f ? 1.0f : vspan / kTop;
        uint32_t kq[2] = {0, 0}, vq[2] = {0, 0};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          kq[i * kBits / 32] |= (uint32_t)fminf(fmaxf(rintf((kf4[i] - kmin) / ks1), 0.f), kTop) << (i * kBits % 32);
          vq[i * kBits / 32] |= (uint32_t)fminf(fmaxf(rintf((vf4[i] - vmin) / vs1), 0.f), kTop) << (i * kBits % 32);
        }
        if (a.commit && row_lane) {
          if constexpr (INT4) {
            *(uint32_t*)(kbase + new_row * GROW + lane * 4) = kq[0];
            *(uint32_t*)(vbase + new_row * GROW + lane * 4) = vq[0];
          } else {
            *(uint2*)(kbase + new_row * GROW + lane * 8) = make_uint2(kq[0], kq[1]);
            *(uint2*)(vbase + new_row * GROW + lane * 8) = make_uint2(vq[0], vq[1]);
          }
          if (lane == 0) {
            ((float2*)ksbase)[new_row] = make_float2(ks1, kmin);
            ((float2*)vsbase)[new_row] = make_float2(vs1, vmin);
          }
        }
        if constexpr (INT4) {
          kc = int4x8_to_bf16x8(kq[0]);
          vc.x = vq[0];   // V goes to the staging buffer as codes
        } else {
          const uint2 k0 = u8x4_to_bf16x4(kq[0]), k1 = u8x4_to_bf16x4(kq[1]);
          const uint2 v0 = u8x4_to_bf16x4(vq[0]), v1 = u8x4_to_bf16x4(vq[1]);
          kc = make_uint4(k0.x, k0.y, k1.x, k1.y);
          vc = make_uint4(v0.x, v0.y, v1.x, v1.y);
        }
        ks1 = __shfl(ks1, 0); vs1 = __shfl(vs1, 0);
        klo1 = __shfl(kmin, 0); vlo1 = __shfl(vmin, 0);
      } else if constexpr (!FP8) {
        if (a.commit && row_lane) {
          *(uint4*)(kbase + new_row * GROW + lane * 16) = kc;
          *(uint4*)(vbase + new_row * GROW + lane * 16) = vc;
        }
      } else {
        // quantise exactly as the append kernel does, then attend to the dequantised row
        const uint32_t kw[4] = {kc.x, kc.y, kc.z, kc.w}, vw[4] = {vc.x, vc.y, vc.z, vc.w};
        float kf8[8], vf8[8], kmax = 0.f, vmax = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          kf8[2 * i] = __uint_as_float(kw[i] << 16); kf8[2 * i + 1] = __uint_as_float(kw[i] & 0xFFFF0000u);
          vf8[2 * i] = __uint_as_float(vw[i] << 16); vf8[2 * i + 1] = __uint_as_float(vw[i] & 0xFFFF0000u);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) { kmax = fmaxf(kmax, fabsf(kf8[i])); vmax = fmaxf(vmax, fabsf(vf8[i])); }
#pragma unroll
        for (int off = 1; off < D / 8; off <<= 1) {
          kmax = fmaxf(kmax, __shfl_xor(kmax, off));
          vmax = fmaxf(vmax, __shfl_xor(vmax, off));
        }
        ks1 = kmax == 0.f ? 1.0f : kmax / 448.0f;
        vs1 = vmax == 0.f ? 1.0f : vmax / 448.0f;
        uint32_t kq[2] = {0, 0}, vq[2] = {0, 0};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          kq[i / 4] |= e4m3_encode(kf8[i] / ks1) << (8 * (i % 4));
          vq[i / 4] |= e4m3_encode(vf8[i] / vs1) << (8 * (i % 4));
        }
        if (a.commit && row_lane) {
          *(uint2*)(kbase + new_row * GROW + lane * 8) = make_uint2(kq[0], kq[1]);
          *(uint2*)(vbase + new_row * GROW + lane * 8) = make_uint2(vq[0], vq[1]);
          if (lane == 0) { ksbase[new_row] = ks1; vsbase[new_row] = vs1; }
        }
        const uint2 k0 = e4m3x4_to_bf16x4(kq[0]), k1 = e4m3x4_to_bf16x4(kq[1]);
        const uint2 v0 = e4m3x4_to_bf16x4(vq[0]), v1 = e4m3x4_to_bf16x4(vq[1]);
        kc = make_uint4(k0.x, k0.y, k1.x, k1.y);
        vc = make_uint4(v0.x, v0.y, v1.x, v1.y);
        ks1 = __shfl(ks1, 0); vs1 = __shfl(vs1, 0);
      }
      // the (dequantised) bf16 rows through LDS into the operand layouts: K as key 0 of a block
      // whose other keys are masked, V as every row of the staging buffer
      if (row_lane) {
        *(uint4*)&sm_new[0][8 * lane] = kc;
        if constexpr (INT4) ((uint32_t*)&sm_new[1][0])[lane] = vc.x;
        else *(uint4*)&sm_new[1][8 * lane] = vc;
      }
      bf16x8 kf[2][NKK];
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        uint4 x = *(const uint4*)&sm_new[0][INT4 ? (D / 4) * qd + 8 * kk : 32 * kk + 8 * qd];
        if (hd != 0) x = make_uint4(0, 0, 0, 0);
        kf[0][kk] = __builtin_bit_cast(bf16x8, x);
        kf[1][kk] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
      }
      if constexpr (INT4) {
#pragma unroll
        for (int j = 0; j < S::NV; ++j) {
          const int row = j * S::VRPI + lane / S::VPR, pc = lane % S::VPR;
          *(uint4*)(my_v + row * GROW + ((pc ^ S::c_swz(row)) * 16)) = *(const uint4*)&sm_new[1][8 * pc];
        }
      } else {
#pragma unroll
        for (int j = 0; j < kUnit * S::CPR / 64; ++j) {
          const int row = j * (64 / S::CPR) + lane / S::CPR, pc = lane % S::CPR;
          *(uint4*)(my_v + row * LROW + (S::v_slot(row, pc) * 16)) = *(const uint4*)&sm_new[1][8 * pc];
        }
      }
      KeyParams kp;
#pragma unroll
      for (int i = 0; i < 8; ++i) { kp.ks[i] = ks1 * c_scale; kp.vs[i] = vs1; kp.klo[i] = klo1 * c_scale; kp.vlo[i] = vlo1 + kMid * vs1; }
      const int64_t saved = exclude;
      exclude = -1;
      f32x4 sacc[2];
      qk(kf, sacc);
      finish(std::true_type{}, sacc, kp, 0, 1);   // keys 0 .. 31 of a virtual block, only key 0 valid
      exclude = saved;
    }

    // ---- merge the four wavefronts through LDS
    float l_head = l_lane + __shfl_xor(l_lane, 16);
    l_head += __shfl_xor(l_head, 32);
    float corr_head = 0.f;
    if constexpr (ASYM) {
      corr_head = corr_lane + __shfl_xor(corr_lane, 16);
      corr_head += __shfl_xor(corr_head, 32);
      corr_head -= (kOff + kMid) * pb_sum[0];
    }
    __syncthreads();   // every wavefront is done with its V staging buffer
    if (head_ok) {
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          sm_o[(wave * 16 + hd) * D + 16 * mb + 4 * qd + r] = oacc[mb][r] + corr_head;
        }
      if (qd == 0) { sm_m[wave][hd] = m_ref; sm_l[wave][hd] = l_head; }
    }
    __syncthreads();
    // retrieval workgroups that share this segment: those owning its first and last unit
    const int64_t w_first = retrieval ? ((seg_a + 1) * W + T - 1) / T - 1 : 0;
    const int64_t w_last = retrieval ? (seg_e * W + T - 1) / T - 1 : 0;
    const int n_parts = (int)(w_last - w_first + 1);
    const int64_t part_row = (int64_t)blockIdx.x + seg;   // unique per (workgroup, segment) pair
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
        acc += wgt * sm_o[(w * 16 + g) * D + d];
        ls += wgt * sm_l[w][g];
      }
      const int h = kvh * G + g;
      if (n_parts == 1) {
        ((uint16_t*)a.out)[((int64_t)b * lv.n_q_heads + h) * D + d] = f32_to_bf16(acc / ls);
        if (a.lse && d == 0) a.lse[(int64_t)b * lv.n_q_heads + h] = (mn + log2f(ls)) * kLn2;
      } else {
        const int64_t pi = part_row * G + g;
        coherent_store(a.part_o + pi * D + d, acc);
        if (d == 0) { coherent_store(a.part_ml + pi * 2, mn); coherent_store(a.part_ml + pi * 2 + 1, ls); }
      }
    }
    if (n_parts > 1) {
      // Ticket: the last workgroup of this segment to get here merges the partials.  Hand-off
      // protocol (the same in the vector-unit kernel): the partials are written with device-scope
      // stores, which go through to the memory side of the per-die L2 caches; every thread waits
      // until its stores are acknowledged (s_waitcnt 0), the workgroup barrier collects those
      // waits, and only then does one thread take the ticket, so whoever sees the final ticket
      // value finds every partial in memory.  The compiler fences keep the steps in that order in
      // the instruction stream.  (A device-scope release fence per workgroup would add a
      // write-back of the die's L2 for data that is already written through.)
      __atomic_signal_fence(__ATOMIC_SEQ_CST);
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      if (tid == 0) {
        int* ticket = a.tickets + seg;
        const int prev = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sm_last = prev == n_parts - 1;
        if (sm_last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next launch
      }
      __syncthreads();
      if (sm_last) {
        // Reader side: an acquire fence (invalidates this compute unit's and die's cached copies,
        // e.g. of an earlier launch's partials), then plain 16-byte loads: with dozens of partial
        // rows per head the merge is bound by what one compute unit can fetch, and device-scope
        // loads (8 bytes at most), which the vector-unit kernel uses for its few rows, were slower.
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        // All heads of the group at once: 256 threads = SLOTS rows of TPR threads (one float4 of a
        // partial row each); head g owns NP consecutive slots; slot `part` of a head folds the
        // partials part, part + NP, ... in that order, then the NP slot results are merged in
        // slot order - a fixed order, so the result is deterministic.
        constexpr int TPR = D / 4, SLOTS = 256 / TPR;
        const int NP = SLOTS / G;                       // G in {1, 2, 4, 8} divides SLOTS
        const int dq = tid % TPR, slot_id = tid / TPR;
        const int mg = slot_id / NP, part = slot_id % NP;
        {
          const float2* ml = (const float2*)a.part_ml;
          const float4* po = (const float4*)a.part_o;
          const int64_t first = (w_first + seg) * G + mg;   // partial row of part 0, stride G rows per part
          float mr = -INFINITY, lr = 0.f;
          float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
          constexpr int B4 = 16;   // partial rows fetched together: one memory round trip per batch
          for (int s0 = part; s0 < n_parts; s0 += NP * B4) {
            float2 mlv[B4];
            float4 x[B4];
#pragma unroll
            for (int j = 0; j < B4; ++j) {
              const int sidx = s0 + j * NP;
              const int sc = sidx < n_parts ? sidx : n_parts - 1;
              const int64_t pr = first + (int64_t)sc * G;
              mlv[j] = ml[pr];
              x[j] = po[pr * TPR + dq];
            }
#pragma unroll
            for (int j = 0; j < B4; ++j) {
              // rows past the end count as empty; decided here, after every load of the batch has
              // been issued, so that no load waits for the one before it
              const bool there = s0 + j * NP < n_parts;
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
          __syncthreads();   // sm_o is free again
          *(float4*)(sm_o + slot_id * D + 4 * dq) = acc;
          if (dq == 0) { sm_m2[slot_id] = mr; sm_l2[slot_id] = lr; }
        }
        __syncthreads();
        for (int idx = tid; idx < G * D; idx += 256) {
          const int g = idx / D, d = idx % D;
          float mn = -INFINITY;
          for (int pp = 0; pp < NP; ++pp) mn = fmaxf(mn, sm_m2[g * NP + pp]);
          float tot = 0.f, ls = 0.f;
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
    }
    u = part_e;
    __syncthreads();   // LDS is reused by the next segment
  }
}

}  // namespace

hipError_t launch_decode_sk(const DecodeArgs& a, hipStream_t stream) {
  const LayerView& lv = a.lv;
  const int64_t ret_units = (int64_t)lv.batch * lv.n_ret * a.units_ret;
  if (a.ret_workers < 0 || a.ret_workers > kMaxDecodeWorkers || (int64_t)a.ret_workers > ret_units ||
      (ret_units > 0 && a.ret_workers < 1) || a.units_ret < 1 || a.units_str < 1)
    return hipErrorInvalidValue;
  dim3 grid((unsigned)(a.ret_workers + lv.batch * lv.n_str));
  if (lv.kv_mode < 0 || lv.kv_mode > 3) return hipErrorInvalidValue;
  if (lv.head_dim == 128) {
    if (lv.kv_mode == 3) decode_sk_kernel<128, 3><<<grid, 256, 0, stream>>>(a);
    else if (lv.kv_mode == 2) decode_sk_kernel<128, 2><<<grid, 256, 0, stream>>>(a);
    else if (lv.kv_mode == 1) decode_sk_kernel<128, 1><<<grid, 256, 0, stream>>>(a);
    else decode_sk_kernel<128, 0><<<grid, 256, 0, stream>>>(a);
  } else {
    if (lv.kv_mode == 3) decode_sk_kernel<64, 3><<<grid, 256, 0, stream>>>(a);
    else if (lv.kv_mode == 2) decode_sk_kernel<64, 2><<<grid, 256, 0, stream>>>(a);
    else if (lv.kv_mode == 1) decode_sk_kernel<64, 1><<<grid, 256, 0, stream>>>(a);
    else decode_sk_kernel<64, 0><<<grid, 256, 0, stream>>>(a);
  }
  return hipGetLastError();
}

}  // namespace duo
