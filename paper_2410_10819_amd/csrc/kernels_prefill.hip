// Chunked pre-filling attention (paper, Section 2.3, Chunked Pre-filling; masks
// of Section 2.2): the chunk's queries attend to [cached tokens || chunk tokens].
// Retrieval heads use the causal mask; streaming heads the exact Lambda mask
// (sink tokens + a window of `recent` positions ending at the query), so K/V
// tiles outside the mask are never loaded.
//
// Flash-style kernel for CDNA4.  A workgroup of eight wavefronts owns a block of
// query rows of one query head; every wavefront owns 32 rows and two wavefronts
// share a SIMD.  The wavefronts form NG "key groups": with NG = 1 all eight share
// each 64-key K/V tile (256 rows per workgroup); with NG = 2 the two groups take
// alternate tiles of the same 128 rows and their partial results are merged
// through LDS at the end, which doubles the number of workgroups when a chunk has
// few row blocks.  K/V tiles are loaded straight from global memory into LDS (the
// lane-ordered LDS-direct load; rows are stored with their 16-byte pieces
// XOR-swizzled so the fragment reads are free of bank conflicts), K one tile
// ahead of V, the next tile's loads being in flight while the current tile is
// computed.  Both contractions use the bf16 MFMA 32x32x16 with fp32 accumulation;
// the softmax is online, in registers.  The score tile is produced transposed
// (S^T = K Q^T) so that each lane owns one query column: row statistics need one
// cross-lane exchange, and the accumulator registers of S^T are, after conversion
// to bf16, exactly the B operand of O^T += V^T P^T.  V^T fragments come from LDS
// transpose reads.  A wavefront alternates a matrix-core block (PV of the previous
// tile, QK^T of the current one, operand reads pipelined ahead of the products)
// with the softmax of the current tile; the two wavefronts of a SIMD do the two in
// opposite order between two workgroup barriers, so that one's softmax runs beside
// the other's matrix-core block (see the main loop).
//
// Keys are addressed through a "virtual key list" so that both head classes
// share the code: for a retrieval head it is positions 0 .. pos0+n-1 (cache
// rows, then chunk rows); for a streaming head it is the retained sink slots,
// the retained ring slots in position order, then the chunk rows.
#include <type_traits>

#include "duo_internal.h"

namespace duo {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int BN = 64;   // keys per tile
constexpr int kDies = 8;      // accelerator dies (XCDs), each with its own L2
constexpr int kBundle = 32;   // workgroups per bundle = compute units per die

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// The values of lane l and lane l ^ 32, in some order, with one vector instruction and no LDS
// round trip: v_permlane32_swap exchanges the upper half of its first operand with the lower half
// of its second.  Written as assembly because this compiler's builtin returns the first result
// twice; the no-ops cover the wait states around a lane swap whose operands come from, and go to,
// ordinary vector instructions (never to a matrix-core instruction directly).
struct HalfPair { float a, b; };
__device__ inline HalfPair both_halves(float x) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  return HalfPair{a, b};
}
// Wavefronts per workgroup with 32 query rows each (two per SIMD), and 32-row sub-blocks per
// wavefront in the instantiations that are launched.
constexpr int kWaves = 8;
constexpr int kSubBlocks = 1;
// LDS reads of the matrix-core phase are written as inline assembly with hand-placed waits:
// the compiler would tie them to the outstanding LDS-direct loads of later tiles (draining the
// prefetch) and would not keep reads several products ahead of their use.  The wait helpers
// name the registers they release so that no use can be scheduled above them.
template <int OFF>
__device__ inline s16x4 lds_read_tr16(uint32_t addr) {   // transposed 8-byte read, see pv_phase
  s16x4 r;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
  return r;
}
template <int OFF>
__device__ inline bf16x8 lds_read_b128(uint32_t addr) {
  bf16x8 r;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
  return r;
}
template <int N>
__device__ inline void lds_wait(s16x4& a, s16x4& b, s16x4& c, s16x4& d, s16x4& e, s16x4& f, s16x4& g, s16x4& h) {
  asm volatile("s_waitcnt lgkmcnt(%8)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(e), "+v"(f), "+v"(g), "+v"(h) : "n"(N) : "memory");
}
template <int N>
__device__ inline void lds_wait(s16x4& a, s16x4& b, s16x4& c, s16x4& d) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N) : "memory");
}
template <int N>
__device__ inline void lds_wait(bf16x8& a, bf16x8& b) {
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}
__device__ inline uint32_t lds_addr(const uint8_t* p) { return (uint32_t)(uintptr_t)LDS_PTR(const uint8_t, p); }
__device__ inline int clamp_i32(int64_t x) {
  const int64_t lim = 1 << 30;
  return (int)(x < -lim ? -lim : (x > lim ? lim : x));
}

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
  int32_t ring0;           // ring index (slot - sink) of position tail_pos
  int32_t row_bytes;
  bool retrieval;

  __device__ inline int64_t position(int64_t u) const { return u < n_head ? u : tail_pos + (u - n_head); }
  // Branch-free row addresses of position p (< pos0: cache slot; otherwise chunk row).
  __device__ inline void rows(int64_t p, const uint8_t*& kr, const uint8_t*& vr) const {
    const bool in_chunk = p >= pos0;
    // cached ring positions are tail_pos .. pos0-1, fewer than `recent` of them
    int64_t x = ring0 + (p - tail_pos);
    if (x >= recent) x -= recent;
    const int64_t slot = (retrieval || p < sink) ? p : sink + x;
    const int64_t off = in_chunk ? (p - pos0) * chunk_stride : slot * row_bytes;
    kr = (in_chunk ? k_chunk : k_cache) + off;
    vr = (in_chunk ? v_chunk : v_cache) + off;
  }
};

#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

template <int N>
using template_int = std::integral_constant<int, N>;

template <int D>
struct Geometry {
  static constexpr int ROW = D * 2;                   // bytes per K or V row in LDS
  static constexpr int TILE = BN * ROW;               // bytes of one K (or V) tile
  static constexpr int BUF_BYTES = 2 * TILE;          // K tile then V tile
  static constexpr int CPR = D / 8;                   // 16-byte pieces per row
  // piece p of row r lives in slot p ^ swizzle(r).  The LDS serves 256 bytes a cycle (64 banks of
  // 4 bytes): 16 lanes of a 16-byte read, 32 lanes of an 8-byte read.  K fragments: 16 neighbouring
  // rows read the same piece, so the swizzle takes 256 / ROW-row groups through all slots.  V^T
  // fragments (transposing 8-byte reads): 32 lanes read four neighbouring pieces of four neighbouring
  // rows, so the swizzle moves each row by four slots.  (Counters on an earlier layout, 2 * row for V,
  // which is free of conflicts only for 16 lanes a cycle: a third of the LDS-active cycles of this
  // kernel were bank conflicts.)
  __device__ static inline int k_swz(int row) { return (row / (256 / ROW)) % CPR; }
  __device__ static inline int v_swz(int row) { return (row * (CPR / 4)) % CPR; }
};

// DUAL: the gate-mixed forward's pass (PrefillArgs::dual), an instantiation of its own so that the
// chunked pre-filling loop carries none of its bookkeeping.
template <int D, int NG, int NSB, bool DUAL>
__global__ __launch_bounds__(NSB == 2 ? 256 : kWaves * 64, 1) void prefill_kernel(PrefillArgs a) {
  static_assert(!DUAL || NG == 1, "the dual pass hands one running state from its streaming part to its middle part");
  using Geo = Geometry<D>;
  constexpr int ROW = Geo::ROW, TILE = Geo::TILE, BUF_BYTES = Geo::BUF_BYTES;
  constexpr int NKK = D / 16;          // MFMA k-steps of the QK^T contraction
  constexpr int NMB = D / 32;          // 32-row blocks of O^T
  constexpr int CPR = D / 8;           // 16-byte pieces per row
  constexpr int NW = NSB == 2 ? 4 : kWaves; // wavefronts per workgroup: 64 rows each, or 32 rows each at two per SIMD
  constexpr int WPG = NW / NG;         // wavefronts per key group
  constexpr int RW = 32 * NSB;         // query rows per wavefront
  constexpr int BM = RW * WPG;         // query rows per workgroup
  constexpr int RPWL = 1024 / ROW;     // rows covered by one wavefront-wide 1 KiB load
  constexpr int NLOAD = TILE / 1024 / WPG;  // loads of K (and of V) per wavefront per tile
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

  const LayerView& lv = a.lv;
  const int tid = threadIdx.x, lane = tid & 63;
  // in a scalar register: everything derived from it (row ranges, the mask test) stays uniform
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave / WPG, wig = wave % WPG;
  const int col = lane & 31, half = lane >> 5;
  const int n_rb = (a.n + BM - 1) / BM;
  // Work list.  Workgroups are dealt to the 8 accelerator dies (each with its own L2) round-robin
  // by block index.  The work is cut into "bundles" of kBundle workgroups that read the same K/V:
  // the G query heads of one KV head times kBundle / G neighbouring row blocks; a die runs one
  // bundle at a time, so the workgroups on it stream the same tiles at about the same time and
  // share them through that die's L2.  Bundles are ranked by length - causal (retrieval) heads
  // before streaming heads, longest rows first, heads of equal length next to each other - and
  // dealt to the dies eight at a time in alternating direction, so that every die gets the same
  // amount of long and short work whatever the number of row blocks and heads is.
  int h, rb;
  {
    const int die = (int)blockIdx.x % kDies, idx = (int)blockIdx.x / kDies;
    const int round = idx / kBundle, w = idx % kBundle;
    const int rank = round * kDies + ((round & 1) ? kDies - 1 - die : die);
    const int rb_per_bundle = kBundle / lv.group;
    const int bundles_per_head = (n_rb + rb_per_bundle - 1) / rb_per_bundle;
    if (rank >= lv.n_kv_heads * bundles_per_head) return;
    const int n_heavy = DUAL ? lv.n_kv_heads : lv.n_ret;   // the dual pass is causal for every head
    int kv_slot, c;
    if (rank < n_heavy * bundles_per_head) {
      c = rank / n_heavy; kv_slot = rank % n_heavy;
    } else {
      const int r2 = rank - n_heavy * bundles_per_head, n_light = lv.n_kv_heads - n_heavy;
      c = r2 / n_light; kv_slot = n_heavy + r2 % n_light;
    }
    const int rbi = c * rb_per_bundle + w / lv.group;
    if (rbi >= n_rb) return;
    const int kv = kv_slot < lv.n_ret ? lv.ret_heads[kv_slot] : lv.str_heads[kv_slot - lv.n_ret];
    h = kv * lv.group + w % lv.group;
    rb = n_rb - 1 - rbi;   // longest rows first
  }
  const int b = blockIdx.y;
  const int kvh = h / lv.group;
  const uint32_t info = lv.head_info[kvh];
  const int slot_head = (int)(info & ~kRetrievalBit);

  KeySource ks;
  constexpr bool dual = DUAL;
  // the dual pass reads no cache (pos0 = 0): its key list is that of a retrieval head, the chunk's positions
  ks.retrieval = dual || (info & kRetrievalBit) != 0;
  // sink positions of the streaming list; the block-aligned mask widens them to whole blocks
  const int sink_k = a.win_block ? a.sink_eff : lv.sink;
  ks.pos0 = a.pos0;
  ks.sink = lv.sink; ks.recent = lv.recent; ks.row_bytes = lv.row_bytes; ks.ring0 = 0;
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
    ks.ring0 = tail >= lv.sink ? (int32_t)((tail - lv.sink) % lv.recent) : 0;
  }
  const int gap32 = (int)(ks.tail_pos - ks.n_head);
  // list entries below sink_u are sink positions
  const int64_t sink_u = gap32 == 0 ? (sink_k < ks.total ? (int64_t)sink_k : ks.total) : ks.n_head;

  // Rows of this workgroup / wavefront / lane: sub-block sb covers chunk rows row_w + 32*sb + col.
  const int i_first = rb * BM;
  const int i_last = (i_first + BM < a.n ? i_first + BM : a.n) - 1;
  const int64_t qpos_first = a.pos0 + i_first, qpos_last = a.pos0 + i_last;
  const int row_w = i_first + wig * RW;
  int ci[NSB];
  int64_t qpos[NSB];
#pragma unroll
  for (int sb = 0; sb < NSB; ++sb) {
    ci[sb] = row_w + 32 * sb + col;
    const int c = ci[sb] < a.n ? ci[sb] : a.n - 1;
    qpos[sb] = a.pos0 + c;
  }

  // A list that is attended causally as a whole: every retrieval head, and a streaming head in
  // the deployed chunk-causal mode (causal attention over [retained cache || chunk]).  The list
  // entry of a chunk position p is p - gap.
  // The dual pass orders and masks its tiles itself: streaming part under the Lambda mask first.
  const bool causal_list = !dual && (ks.retrieval || a.chunk_causal != 0);
  const int64_t gap = ks.tail_pos - ks.n_head;
  // Tile list of the workgroup: [0, tA_end) covers the sink part, [tB_begin, t_end) the window.
  int64_t tA_end, tB_begin, t_end;
  if (causal_list) {
    tA_end = 0; tB_begin = 0; t_end = (qpos_last - gap) / BN + 1;
  } else {
    const int64_t usink = (int64_t)sink_k < qpos_last + 1 ? sink_k : qpos_last + 1;
    tA_end = (usink + BN - 1) / BN;
    // first window position of the workgroup's first query (window starts never decrease with the query)
    int64_t plo = a.win_block ? (qpos_first / a.win_block - a.n_local_blocks + 1) * (int64_t)a.win_block
                              : qpos_first - lv.recent + 1;
    if (plo < 0) plo = 0;
    const int64_t u_lo = plo < ks.tail_pos ? (plo < ks.n_head ? plo : ks.n_head) : ks.n_head + (plo - ks.tail_pos);
    const int64_t u_hi = qpos_last < ks.n_head ? qpos_last : ks.n_head + (qpos_last - ks.tail_pos);
    tB_begin = u_lo / BN;
    if (tB_begin < tA_end) tB_begin = tA_end;
    t_end = u_hi / BN + 1;
    if (t_end < tA_end) t_end = tA_end;
  }
  // Dual pass: after the n_lambda tiles of the streaming part come the tiles [tM_begin, tM_end) that hold
  // "middle" keys - causal, but neither sink nor in the window - of some row of the workgroup: positions
  // sink .. (first window position of the last row) - 1.  Tiles that hold keys of both kinds are visited
  // in both parts, with complementary masks.
  const int n_lambda = (int)(tA_end + (t_end - tB_begin));
  int64_t tM_begin = 0, tM_end = 0;
  if (dual) {
    int64_t wfirst = a.win_block ? (qpos_last / a.win_block - a.n_local_blocks + 1) * (int64_t)a.win_block
                                 : qpos_last - lv.recent + 1;
    if (wfirst > (int64_t)sink_k) { tM_begin = sink_k / BN; tM_end = (wfirst - 1) / BN + 1; }
  }
  const int n_middle = (int)(tM_end - tM_begin);
  const int n_tiles = n_lambda + n_middle;
  const int n_iter = (n_tiles + NG - 1) / NG;
  // Tile indices fit 32 bits; the per-iteration bookkeeping below is 32-bit scalar arithmetic.
  const int tA = (int)tA_end, tB = (int)tB_begin, tM = (int)tM_begin;
  auto tile_of = [&](int s) -> int { return s < tA ? s : (s < n_lambda ? tB + (s - tA) : tM + (s - n_lambda)); };
  // Classes of tiles, by index: [0, t_dense_end) lie wholly in the dense cache of a retrieval head;
  // [t_chunk_begin, t_whole_end) lie wholly in the chunk; tiles from t_whole_end on are cut by
  // the end of the list; the others straddle regions and take the general load path.
  const int64_t u_chunk0 = ks.n_head + (ks.pos0 - ks.tail_pos);   // list entry of the chunk's first row
  const int t_whole_end = (int)(ks.total / BN);
  const int t_dense_end = ks.retrieval ? (int)(ks.pos0 / BN) : 0;
  const int t_chunk_begin = (int)((u_chunk0 + BN - 1) / BN);
  // First tile that needs the causal mask for sub-block sb of this wavefront (causal lists).
  int t_mask[NSB];
#pragma unroll
  for (int sb = 0; sb < NSB; ++sb) {
    const int64_t x = a.pos0 + row_w + 32 * sb - gap - BN + 1;
    const int64_t tm = x < 0 ? 0 : x / BN + 1;
    t_mask[sb] = tm < t_whole_end ? (int)tm : t_whole_end;
  }

  // Q^T fragments (B operand): lane (col, half) holds q[row][16*kk + 8*half .. +7].
  bf16x8 qf[NSB][NKK];
#pragma unroll
  for (int sb = 0; sb < NSB; ++sb) {
    const int c = ci[sb] < a.n ? ci[sb] : a.n - 1;
    const uint8_t* qrow = (const uint8_t*)a.q + (((int64_t)b * a.n + c) * lv.n_q_heads + h) * D * 2;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) qf[sb][kk] = *(const bf16x8*)(qrow + (16 * kk + 8 * half) * 2);
  }
  f32x16 o_acc[NSB][NMB];
#pragma unroll
  for (int sb = 0; sb < NSB; ++sb)
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[sb][mb][r] = 0.f;
  float m_i[NSB], l_i[NSB];
#pragma unroll
  for (int sb = 0; sb < NSB; ++sb) { m_i[sb] = -INFINITY; l_i[sb] = 0.f; }
  const float sc = lv.scale * kLog2e;

  // Issue the LDS-direct loads of tile t into a buffer: each wavefront-wide load
  // fills 1 KiB (RPWL rows); lane (row, slot) fetches piece slot ^ swizzle(row).
  // A tile whose 64 keys are consecutive rows of one region (the dense cache of a
  // retrieval head, or the chunk) is addressed as a wavefront-uniform base plus
  // per-lane offsets that never change; other tiles take the general path.
  // (Successive loads of a wavefront are WPG * RPWL rows apart; the swizzles repeat after SWZ_PERIOD
  // rows, so a wavefront needs NPH sets of lane offsets, one per swizzle phase its loads fall in.)
  constexpr int XROWS = WPG * RPWL;    // rows between successive loads of one wavefront
  constexpr int SWZ_PERIOD = CPR * (256 / ROW);
  constexpr int NPH = XROWS % SWZ_PERIOD == 0 ? 1 : SWZ_PERIOD / XROWS;
  static_assert(NPH == 1 || (SWZ_PERIOD % XROWS == 0 && NLOAD % NPH == 0), "unsupported tile load geometry");
  int lin_k_cache[NPH], lin_v_cache[NPH], lin_k_chunk[NPH], lin_v_chunk[NPH];
#pragma unroll
  for (int ph = 0; ph < NPH; ++ph) {
    const int row = (wig + WPG * ph) * RPWL + lane / CPR, slot = lane % CPR;
    lin_k_cache[ph] = row * ROW + ((slot ^ Geo::k_swz(row)) * 16);
    lin_v_cache[ph] = row * ROW + ((slot ^ Geo::v_swz(row)) * 16);
    lin_k_chunk[ph] = row * (int)ks.chunk_stride + ((slot ^ Geo::k_swz(row)) * 16);
    lin_v_chunk[ph] = row * (int)ks.chunk_stride + ((slot ^ Geo::v_swz(row)) * 16);
  }
  // Issue the LDS-direct loads of one tensor (K or V) of tile t into an LDS tile buffer.
  auto fetch_one = [&](int t, uint8_t* dst, auto is_v_tag) {
    constexpr bool IS_V = decltype(is_v_tag)::value;
    const int64_t u0 = (int64_t)t * BN;
    if (t < t_dense_end) {                                      // dense cache rows u0 .. u0+63
      const uint8_t* base = (IS_V ? ks.v_cache : ks.k_cache) + u0 * ROW;
#pragma unroll
      for (int x = 0; x < NLOAD; ++x) {
        const int lin = IS_V ? lin_v_cache[x % NPH] : lin_k_cache[x % NPH];
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(base + (x / NPH) * (NPH * XROWS * ROW) + lin), LDS_PTR(void, dst + (wig + WPG * x) * 1024), 16, 0, 0);
      }
    } else if (t >= t_chunk_begin && t < t_whole_end) {         // chunk rows
      const int64_t c0 = u0 - u_chunk0;
      const uint8_t* base = (IS_V ? ks.v_chunk : ks.k_chunk) + c0 * ks.chunk_stride;
#pragma unroll
      for (int x = 0; x < NLOAD; ++x) {
        const int lin = IS_V ? lin_v_chunk[x % NPH] : lin_k_chunk[x % NPH];
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(base + (x / NPH) * (NPH * XROWS * ks.chunk_stride) + lin), LDS_PTR(void, dst + (wig + WPG * x) * 1024), 16, 0, 0);
      }
    } else {                                                    // rare: not unrolled, to keep registers free
#pragma nounroll
      for (int x = 0; x < NLOAD; ++x) {
        const int j = wig + WPG * x;
        const int row = j * RPWL + lane / CPR, slot = lane % CPR;
        int64_t u = u0 + row;
        if (u >= ks.total) u = ks.total - 1;
        const uint8_t *kr, *vr;
        ks.rows(ks.position(u), kr, vr);
        const int swz = IS_V ? Geo::v_swz(row) : Geo::k_swz(row);
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR((IS_V ? vr : kr) + ((slot ^ swz) * 16)), LDS_PTR(void, dst + j * 1024), 16, 0, 0);
      }
    }
  };

  f32x16 s_acc[NSB][2];
  bf16x8 pf[NSB][4];

  // Per-lane LDS offsets of the operand fragments inside a tile buffer (they never change).
  // K fragment (kb, kk): row 32 kb + col, piece (2 kk + half) ^ swizzle(col): one offset per kk,
  // kb adds a constant.  V^T fragment (slab sl, block mb): this lane addresses key
  // 16 sl + 4 half + e (and + 8), bytes 8 (i4 & 1) of piece (4 mb + pc0) ^ swizzle(key): one offset
  // per mb (the swizzle does not depend on sl), sl and the + 8 rows add constants.
  uint32_t k_frag_off[NKK], v_frag_off[NMB];
  {
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) k_frag_off[kk] = (uint32_t)(col * ROW + (((2 * kk + half) ^ Geo::k_swz(col)) * 16));
    const int blk = lane >> 4, l16 = lane & 15;
    const int e = l16 >> 2, i4 = l16 & 3;
    const int pc0 = 2 * (blk & 1) + (i4 >> 1), sub8 = (i4 & 1) * 8;
    const int keyl = 4 * half + e;
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb) v_frag_off[mb] = (uint32_t)(keyl * ROW + (((4 * mb + pc0) ^ Geo::v_swz(keyl)) * 16) + sub8);
  }
  struct VSlab { s16x4 lo[NMB], hi[NMB]; };
  auto read_v_slab = [&](VSlab& f, const uint32_t (&va)[NMB], auto sl_tag) {
    constexpr int SL = decltype(sl_tag)::value;
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb) {
      f.lo[mb] = lds_read_tr16<SL * 16 * ROW>(va[mb]);
      f.hi[mb] = lds_read_tr16<SL * 16 * ROW + 8 * ROW>(va[mb]);
    }
  };
  auto wait_v_slab = [&](VSlab& f, auto n_tag) {
    constexpr int N = decltype(n_tag)::value;
    if constexpr (NMB == 4) lds_wait<N>(f.lo[0], f.hi[0], f.lo[1], f.hi[1], f.lo[2], f.hi[2], f.lo[3], f.hi[3]);
    else lds_wait<N>(f.lo[0], f.hi[0], f.lo[1], f.hi[1]);
  };
  auto mma_v_slab = [&](const VSlab& f, int sl) {
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb) {
      const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(f.lo[mb], f.hi[mb], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
      for (int sb = 0; sb < NSB; ++sb)
        o_acc[sb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sb][sl], o_acc[sb][mb], 0, 0, 0);
    }
  };
  template_int<0> i0; template_int<1> i1; template_int<2> i2; template_int<3> i3;
  template_int<2 * NMB> i_slab;

  // The matrix-core block of one iteration: O^T += V^T P^T of the previous tile (slab sl covers
  // keys 16 sl + {4 half + t, 8 + 4 half + t}), then S^T = K Q^T of the current tile (two 32-key
  // blocks x NSB x 32 queries; consecutive products accumulate into different registers, so none
  // waits for the one before it).  LDS reads run one slab / two k-steps ahead of the products.
  auto m_phase = [&](const uint8_t* v_lds, const uint8_t* k_lds, bool do_pv, bool do_qk) {
    uint32_t va[NMB], ka[NKK];
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb) va[mb] = lds_addr(v_lds) + v_frag_off[mb];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) ka[kk] = lds_addr(k_lds) + k_frag_off[kk];
    if (do_pv) {
      VSlab fa, fb;
      read_v_slab(fa, va, i0);
      read_v_slab(fb, va, i1);
      wait_v_slab(fa, i_slab); mma_v_slab(fa, 0);
      read_v_slab(fa, va, i2);
      wait_v_slab(fb, i_slab); mma_v_slab(fb, 1);
      read_v_slab(fb, va, i3);
      wait_v_slab(fa, i_slab); mma_v_slab(fa, 2);
      wait_v_slab(fb, i0); mma_v_slab(fb, 3);
    }
    if (do_qk) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int sb = 0; sb < NSB; ++sb)
#pragma unroll
          for (int r = 0; r < 16; ++r) s_acc[sb][kb][r] = 0.f;
      bf16x8 kf[NKK][2];
      kf[0][0] = lds_read_b128<0>(ka[0]); kf[0][1] = lds_read_b128<32 * ROW>(ka[0]);
      kf[1][0] = lds_read_b128<0>(ka[1]); kf[1][1] = lds_read_b128<32 * ROW>(ka[1]);
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        if (kk + 2 < NKK) {
          kf[kk + 2][0] = lds_read_b128<0>(ka[kk + 2]); kf[kk + 2][1] = lds_read_b128<32 * ROW>(ka[kk + 2]);
          lds_wait<4>(kf[kk][0], kf[kk][1]);
        } else if (kk + 1 < NKK) {
          lds_wait<2>(kf[kk][0], kf[kk][1]);
        } else {
          lds_wait<0>(kf[kk][0], kf[kk][1]);
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int sb = 0; sb < NSB; ++sb)
            s_acc[sb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk][kb], qf[sb][kk], s_acc[sb][kb], 0, 0, 0);
      }
    }
  };

  // Dual pass: first window position of the wavefront's first row, per sub-block.
  int64_t mid_w0[NSB];
#pragma unroll
  for (int sb = 0; sb < NSB; ++sb) {
    const int64_t q0 = a.pos0 + (row_w + 32 * sb < a.n ? row_w + 32 * sb : a.n - 1);
    mid_w0[sb] = !dual ? 0 : (a.win_block ? (q0 / a.win_block - a.n_local_blocks + 1) * (int64_t)a.win_block : q0 - lv.recent + 1);
  }
  // Online softmax of the tile whose first key is list entry ub: s_acc -> pf, m_i, l_i; rescales o_acc.
  auto softmax_phase = [&](int t, bool middle) {
    const int64_t ub = (int64_t)t * BN;
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      // Mask (only tiles that touch the mask boundary or the end of the list).  A tile of the middle
      // part needs none if it starts after the sinks and ends before the window of the wavefront's
      // first row of this sub-block (window starts never decrease with the query).
      bool need_mask = !causal_list || t >= t_mask[sb];
      if (middle) need_mask = !(ub >= (int64_t)sink_k && ub + BN - 1 < mid_w0[sb]);
      // Online softmax for this lane's query column; `score(kb, r)` yields the masked score.
      auto softmax_block = [&](auto&& score) {
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, score(kb, r));
        {
          const HalfPair hp = both_halves(mx);
          mx = fmaxf(hp.a, hp.b);
        }
        const float m_new = fmaxf(m_i[sb], mx * sc);
        const float mu = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = fast_exp2(m_i[sb] - mu);
        m_i[sb] = m_new;
        // The row sum is four chains of plain additions of the unrounded probabilities.  A
        // dot-product instruction per pair would halve the count, but dot products run on the
        // matrix pipeline and wait while the SIMD's other wavefront has MFMAs in flight, whereas
        // v_add / v_fma / v_exp / v_max3 / v_cvt_pk issue beside them (measured with a probe).
        float psum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; r += 2) {
            const float p0 = fast_exp2(fmaf(score(kb, r), sc, -mu));
            const float p1 = fast_exp2(fmaf(score(kb, r + 1), sc, -mu));
            const bf16x2 pp = {(__bf16)p0, (__bf16)p1};
            psum[(r / 2) & 1] += p0;
            psum[2 + ((r / 2) & 1)] += p1;
            pf[sb][kb * 2 + r / 8][r % 8] = pp[0];
            pf[sb][kb * 2 + r / 8][r % 8 + 1] = pp[1];
          }
        l_i[sb] = l_i[sb] * alpha + ((psum[0] + psum[1]) + (psum[2] + psum[3]));
        if (__ballot(alpha != 1.0f) != 0) {
#pragma unroll
          for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[sb][mb][r] *= alpha;
        }
      };
      if (!need_mask) {
        // interior tile: the scores are read straight from the matrix-core accumulators
        softmax_block([&](int kb, int r) { return s_acc[sb][kb][r]; });
      } else {
        // Scores with the mask applied, in registers of their own: the matrix-core
        // accumulators are only read here, never overwritten.
        float sv[2][16];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) sv[kb][r] = s_acc[sb][kb][r];
        const int lim = clamp_i32(ks.total - ub);
        const int qa = clamp_i32(qpos[sb] - ub);             // query position relative to the tile
        if (causal_list) {
          const int qu = clamp_i32(qpos[sb] - gap - ub);     // the query's own list entry, relative to the tile
          const int bound = qu < lim - 1 ? qu : lim - 1;     // visible iff u_rel <= bound
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int u_rel = 32 * kb + 8 * (r / 4) + 4 * half + (r % 4);
              if (u_rel > bound) sv[kb][r] = -INFINITY;
            }
        } else {
          const int nh_rel = clamp_i32(ks.n_head - ub);
          const int sink_rel = clamp_i32(sink_u - ub);
          // keys at distance < win from the query are inside its window: `recent` for the Lambda mask,
          // up to the start of the first local block for the block-aligned one
          const int win = a.win_block ? (int)(qpos[sb] % a.win_block) + (a.n_local_blocks - 1) * a.win_block + 1
                                      : lv.recent;
          // An entry at or after n_head holds position entry + gap32, an earlier one its own index.
          // So the visible entries of the tile are two runs: sink entries [0, s_hi] (not beyond
          // the list or the query) and window entries [w_lo, w_hi] (the `win` positions ending at
          // the query; behind a gap only entries from n_head on).  A lane's entries are a
          // compile-time constant plus 4 * half, which goes into the bounds once: three
          // compares per score.
          const int qb = qa - gap32;                           // the query's own entry (from n_head on)
          int s_hi = sink_rel - 1 < lim - 1 ? sink_rel - 1 : lim - 1;
          s_hi = s_hi < qa ? s_hi : qa;
          int w_hi = lim - 1 < qb ? lim - 1 : qb;
          int w_lo = qb - win + 1;
          if (gap32 > 0 && w_lo < nh_rel) w_lo = nh_rel;
          if (middle) {
            // the complement within the causal keys: from the first position after the sinks up to
            // the one before the query's window (there is no gap in the dual pass's list)
            const int m_lo = sink_rel - 4 * half, m_hi = w_lo - 1 - 4 * half;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int c = 32 * kb + 8 * (r / 4) + (r % 4);
                if (!((c >= m_lo) & (c <= m_hi))) sv[kb][r] = -INFINITY;
              }
          } else {
            s_hi -= 4 * half; w_hi -= 4 * half; w_lo -= 4 * half;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int c = 32 * kb + 8 * (r / 4) + (r % 4);
                const bool vis = (c <= s_hi) | ((c >= w_lo) & (c <= w_hi));
                if (!vis) sv[kb][r] = -INFINITY;
              }
          }
        }
        softmax_block([&](int kb, int r) { return sv[kb][r]; });
      }
    }
  };

  // Dual pass, between its two parts: (1 - alpha) * (streaming attention of the wavefront's rows) -> out.
  // The final store reads it back (the same lane, the same addresses) and adds alpha * full attention.
  auto emit_streaming_term = [&]() {
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      if (ci[sb] >= a.n) continue;
      const HalfPair hp = both_halves(l_i[sb]);
      const float inv = (1.0f - a.mix_alpha[kvh]) / (hp.a + hp.b);
      uint8_t* orow = (uint8_t*)a.out + (((int64_t)b * a.n + ci[sb]) * lv.n_q_heads + h) * D * 2;
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
        for (int bq = 0; bq < 4; ++bq) {
          bf16x4 w;
#pragma unroll
          for (int t4 = 0; t4 < 4; ++t4) w[t4] = (__bf16)(o_acc[sb][mb][4 * bq + t4] * inv);
          *(bf16x4*)(orow + (32 * mb + 8 * bq + 4 * half) * 2) = w;
        }
    }
  };

  // Main loop.  A wavefront's work on tile t is M_t = [O += P V of tile t-1, then S = K Q^T of
  // tile t] (matrix cores) followed by S_t = softmax of tile t (vector unit).  Every wavefront
  // passes one workgroup barrier per iteration, but not at the same place: the first wavefront
  // of a SIMD after its softmax, the second one after its matrix-core block.  Between two
  // barriers the first therefore runs [M_t, S_t] and the second [S_t-1, M_t]: while one is in
  // its matrix-core block the other does its softmax, with nothing holding them in lock-step
  // inside the interval.  (A barrier after each of the two phases makes the two take the plain
  // sum of their times on this hardware; so does running both in phase.)  K runs one tile ahead
  // of V in the LDS buffers: load L_j = (K of tile j, V of tile j-1) is issued at the top of
  // iteration j-1, each wavefront waits for its own loads before its barrier, and the buffer it
  // overwrites was last read in iteration j-2 by either kind of wavefront.  With 64 rows per
  // wavefront (one per SIMD) there is nothing to alternate with and all barriers coincide.
  auto kbuf = [&](int j) { return smem + (grp * 2 + (j & 1)) * BUF_BYTES; };
  auto vbuf = [&](int j) { return smem + (grp * 2 + (j & 1)) * BUF_BYTES + TILE; };
  auto issue_l = [&](int j) {
    const int sk = j * NG + grp, sv = (j - 1) * NG + grp;
    if (sk < n_tiles) fetch_one(tile_of(sk), kbuf(j), std::false_type{});
    if (j >= 1 && sv < n_tiles) fetch_one(tile_of(sv), vbuf(j - 1), std::true_type{});
  };
  {
    const bool s_first = NW == 8 && (NG == 1 ? (wave >= NW / 2) : (grp == 1));
    issue_l(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
    for (int it = 0; it <= n_iter; ++it) {
      const int s = it * NG + grp;
      const bool live_qk = it < n_iter && s < n_tiles;
      const bool live_pv = it >= 1 && s - NG < n_tiles;
      issue_l(it + 1);
      m_phase(vbuf(it - 1), kbuf(it), live_pv, live_qk);
      __builtin_amdgcn_sched_barrier(0);
      // dual pass: O, m, l now cover exactly the streaming part (its last tile's P V has just been added)
      if (NG == 1 && dual && n_middle > 0 && it == n_lambda) emit_streaming_term();
      // the iteration's one barrier: after the matrix-core block for the wavefronts that run the
      // softmax first, after the softmax for the others
      if (s_first) {
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __builtin_amdgcn_s_barrier();
      }
      if (live_qk) softmax_phase(tile_of(s), dual && s >= n_lambda);
      __builtin_amdgcn_sched_barrier(0);
      if (!s_first) {
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __builtin_amdgcn_s_barrier();
      }
    }
  }

  // Row sums over both lane halves.
#pragma unroll
  for (int sb = 0; sb < NSB; ++sb) {
    const HalfPair hp = both_halves(l_i[sb]);
    l_i[sb] = hp.a + hp.b;
  }

  if constexpr (NG == 2) {
    // Key group 1 hands its partial (O, m, l) to key group 0 through LDS.
    constexpr int REGS = NMB * 16 + 2;
    float* xch = (float*)smem;   // the tile buffers are free after the barrier
    __syncthreads();
    if (grp == 1) {
#pragma unroll
      for (int sb = 0; sb < NSB; ++sb) {
        float* base = xch + ((wig * NSB + sb) * REGS) * 64 + lane;
#pragma unroll
        for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) base[(mb * 16 + r) * 64] = o_acc[sb][mb][r];
        base[(NMB * 16) * 64] = m_i[sb];
        base[(NMB * 16 + 1) * 64] = l_i[sb];
      }
    }
    __syncthreads();
    if (grp == 1) return;
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      const float* base = xch + ((wig * NSB + sb) * REGS) * 64 + lane;
      const float m1 = base[(NMB * 16) * 64], l1 = base[(NMB * 16 + 1) * 64];
      const float m_new = fmaxf(m_i[sb], m1);
      const float mu = m_new == -INFINITY ? 0.f : m_new;
      const float a0 = fast_exp2(m_i[sb] - mu), a1 = fast_exp2(m1 - mu);
      l_i[sb] = l_i[sb] * a0 + l1 * a1;
      m_i[sb] = m_new;
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[sb][mb][r] = o_acc[sb][mb][r] * a0 + base[(mb * 16 + r) * 64] * a1;
    }
  }

  // Normalise and store.  Lane (col, half) holds O^T rows 32*mb + 8*bq + 4*half + t.
#pragma unroll
  for (int sb = 0; sb < NSB; ++sb) {
    if (ci[sb] >= a.n) continue;
    float inv = 1.0f / l_i[sb];
    const int64_t row_off = (((int64_t)b * a.n + ci[sb]) * lv.n_q_heads + h) * D * 2;
    uint8_t* orow = (uint8_t*)a.out + row_off;
    // dual pass with a middle part: the state is now full attention, which enters with weight alpha
    // beside the streaming term stored earlier (already rounded to bf16 once); the sum is rounded once.
    // Without a middle part the two terms are the same and the result is written as it is.
    const bool mix = NG == 1 && dual && n_middle > 0;
    if (mix) inv *= a.mix_alpha[kvh];
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
      for (int bq = 0; bq < 4; ++bq) {
        float x[4] = {0.f, 0.f, 0.f, 0.f};
        if (mix) {
          const bf16x4 other = *(const bf16x4*)(orow + (32 * mb + 8 * bq + 4 * half) * 2);
#pragma unroll
          for (int t4 = 0; t4 < 4; ++t4) x[t4] = (float)other[t4];
        }
        bf16x4 w;
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) w[t4] = (__bf16)(o_acc[sb][mb][4 * bq + t4] * inv + x[t4]);
        *(bf16x4*)(orow + (32 * mb + 8 * bq + 4 * half) * 2) = w;
      }
    if (a.lse && half == 0)
      a.lse[((int64_t)b * lv.n_q_heads + h) * a.n + ci[sb]] = (m_i[sb] + log2f(l_i[sb])) * kLn2;
  }
}

template <int D, int NG, int NSB, bool DUAL>
hipError_t launch_one(const PrefillArgs& a, hipStream_t stream) {
  constexpr int NW = NSB == 2 ? 4 : kWaves;
  constexpr int BM = 32 * NSB * (NW / NG);
  constexpr int lds = NG * 2 * Geometry<D>::BUF_BYTES;
  static bool configured = false;   // one attribute call per kernel instantiation and process
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)prefill_kernel<D, NG, NSB, DUAL>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int n_rb = (a.n + BM - 1) / BM;
  const int rb_per_bundle = kBundle / a.lv.group;
  const int bundles = a.lv.n_kv_heads * ((n_rb + rb_per_bundle - 1) / rb_per_bundle);
  dim3 grid((unsigned)((bundles + kDies - 1) / kDies * kDies * kBundle), a.lv.batch);
  prefill_kernel<D, NG, NSB, DUAL><<<grid, NW * 64, lds, stream>>>(a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_prefill(const PrefillArgs& a, hipStream_t stream) {
  constexpr int NSB = kSubBlocks;
  // Two key groups per workgroup when 256-row blocks alone would leave compute units idle.
  // (The dual pass hands one running state from its streaming part to its middle part and so keeps one key group.)
  const int n_heavy_heads = a.dual ? a.lv.n_kv_heads : a.lv.n_ret;
  const int64_t heavy_blocks = (int64_t)a.lv.batch * n_heavy_heads * a.lv.group * ((a.n + 255) / 256);
  if (a.dual) return a.lv.head_dim == 128 ? launch_one<128, 1, NSB, true>(a, stream) : launch_one<64, 1, NSB, true>(a, stream);
  const bool split_keys = heavy_blocks < 384;
  if (a.lv.head_dim == 128) return split_keys ? launch_one<128, 2, NSB, false>(a, stream) : launch_one<128, 1, NSB, false>(a, stream);
  return split_keys ? launch_one<64, 2, NSB, false>(a, stream) : launch_one<64, 1, NSB, false>(a, stream);
}

}  // namespace duo
