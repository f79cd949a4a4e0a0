// Internal declarations shared by the host API and the HIP kernels of libduoattn.
// Nothing here is part of the public C ABI (see include/duoattn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "duoattn.h"

namespace duo {

// Bit 31 of a head_info entry marks a retrieval KV head; the low bits hold the
// head's slot inside its class's cache.
constexpr uint32_t kRetrievalBit = 0x80000000u;

// Upper bound on key splits per retrieval head in decode (sizes the scratch).
constexpr int kMaxDecodeSplits = 256;
// Even-split decode: rows per work unit and the largest grid (sizes the scratch).
constexpr int kDecodeUnitRows = 32;
constexpr int kMaxDecodeWorkers = 1024;

// Device view of one layer's two caches.  Layouts (row = one token of one head):
//   retrieval: [batch][n_ret][max_seq][row_bytes]            (+ scales [batch][n_ret][max_seq][sc_per_row])
//   streaming: [batch][n_str][sink + recent][row_bytes]      (+ scales [batch][n_str][sink+recent][sc_per_row])
// A streaming token at position p lives in slot p (p < sink) or
// sink + (p - sink) % recent (ring buffer; the newest token overwrites the oldest).
struct LayerView {
  uint8_t* k_ret;
  uint8_t* v_ret;
  float* ks_ret;
  float* vs_ret;
  uint8_t* k_str;
  uint8_t* v_str;
  float* ks_str;
  float* vs_str;
  const uint32_t* head_info;  // [n_kv_heads]
  const int32_t* ret_heads;   // [n_ret] KV head index of each retrieval slot
  const int32_t* str_heads;   // [n_str]
  int32_t n_ret, n_str;
  int32_t batch, n_q_heads, n_kv_heads, group, head_dim;
  int32_t sink, recent;
  int32_t row_bytes;          // head_dim * 2 (bf16), head_dim (fp8, int8) or head_dim / 2 (int4)
  int32_t kv_mode;            // duo_kv_dtype_t: 0 bf16, 1 fp8 codes + one scale per row, 2 int4 / 3 int8 codes + (scale, minimum) per row
  int32_t sc_per_row;         // floats per row in the scale arrays: 0, 1 or 2
  int64_t max_seq;
  float scale;                // softmax scale
};

struct DecodeArgs {
  LayerView lv;
  const void* q;       // [batch][n_q_heads][head_dim] bf16
  const void* k_new;   // [batch][n_kv_heads][head_dim] bf16 or null
  const void* v_new;
  void* out;           // [batch][n_q_heads][head_dim] bf16
  float* lse;          // [batch][n_q_heads] or null
  float* part_o;       // [batch][n_q_heads][splits][head_dim]
  float* part_ml;      // [batch][n_q_heads][splits][2]
  int32_t* tickets;    // [batch][n_kv_heads], zero between launches
  int64_t cache_len;   // tokens held by the cache
  int32_t splits;      // key splits per retrieval head
  int32_t commit;      // write k_new / v_new into the caches (position cache_len)
  // even-split kernel: units of kDecodeUnitRows rows per retrieval / streaming segment (>= 1 each);
  // partial rows are indexed workgroup + segment, tickets by segment
  int32_t units_ret, units_str;
  int32_t ret_workers;  // workgroups sharing the retrieval units (0 if the layer has no retrieval head)
};

// Most KV heads a gate-mixed forward takes (their gates ride in the kernel arguments).
constexpr int kMaxGateHeads = 64;

struct PrefillArgs {
  LayerView lv;
  const void* q;       // [batch][n][n_q_heads][head_dim]
  const void* k;       // [batch][n][n_kv_heads][head_dim]
  const void* v;
  void* out;
  float* lse;          // [batch][n_q_heads][n] or null
  int64_t pos0;        // tokens in the cache = position of the chunk's first query
  int32_t n;           // chunk length
  int32_t chunk_causal;  // streaming heads: causal attention over [retained cache || chunk] instead of the Lambda mask
  // Gate-mixed forward (whole sequence, no cache, pos0 = 0): every head is attended to twice from one
  // pass over its causal keys.  The keys the streaming mask shows (sinks and window) are a subset of
  // the causal ones, so a workgroup runs them first, writes the streaming term scaled by
  // 1 - mix_alpha[kv head] to out, continues the SAME online-softmax state over the remaining
  // ("middle") keys, which makes it the full-attention state, and finally writes
  // mix_alpha * full + (what it stored before).  Every score is computed once, except in the few
  // tiles that hold both kinds of keys.
  int32_t dual;
  // Streaming mask of the dual pass: block size of the block-aligned approximation of the Lambda
  // mask (0 = the Lambda mask itself), the number of sink positions it makes visible
  // (ceil(sink / block) * block) and the number of key blocks ending at the query's own block.
  int32_t win_block, sink_eff, n_local_blocks;
  float mix_alpha[kMaxGateHeads];
};

hipError_t launch_append(const LayerView& lv, const void* k, const void* v, int64_t pos0,
                         int n_new, hipStream_t stream);
hipError_t launch_export(const LayerView& lv, int batch_idx, int kv_head, int64_t len,
                         void* k_out, void* v_out, float* ks_out, float* vs_out,
                         int64_t* pos_out, int64_t count, hipStream_t stream);
hipError_t launch_decode(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_decode_sk(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_prefill(const PrefillArgs& a, hipStream_t stream);
// Widen rows a quantised layer holds (cache length len) to bf16 rows in the same layouts:
// k_ret_out / v_ret_out [batch][n_ret][max_seq][head_dim] and k_str_out / v_str_out
// [batch][n_str][sink + recent][head_dim], bf16.  Of the retrieval rows only positions
// first_ret_row .. len-1 are widened (the image already holds the earlier ones); the streaming
// rows (at most sink + recent per head) are widened whole.  Rows beyond the ones held are not written.
hipError_t launch_dequant(const LayerView& lv, int64_t first_ret_row, int64_t len, void* k_ret_out, void* v_ret_out,
                          void* k_str_out, void* v_str_out, hipStream_t stream);

// fp32 -> OCP E4M3 (finite-only) code, round to nearest even, saturating at 448: the one encoder
// of the append kernel and of the decode kernels' fused append.
__device__ inline uint32_t e4m3_encode(float x) {
  uint32_t u = __float_as_uint(x);
  const uint32_t sign = (u >> 24) & 0x80u;
  u &= 0x7FFFFFFFu;
  const float a = __uint_as_float(u);
  uint32_t code;
  if (a >= 448.0f) {
    code = 0x7Eu;
  } else if (a < 0.015625f) {             // below the smallest normal 2^-6: grid step 2^-9
    code = (uint32_t)rintf(a * 512.0f);   // 8 carries into the smallest normal
  } else {
    const uint32_t r = u + 0x7FFFFu + ((u >> 20) & 1u);   // RNE to 3 mantissa bits
    code = (r >> 20) - ((127u - 7u) << 3);
  }
  return code | sign;
}

// Number of rows a streaming cache holds after `len` appends.
__host__ __device__ inline int64_t streaming_rows(int64_t len, int sink, int recent) {
  int64_t cap = (int64_t)sink + recent;
  return len < cap ? len : cap;
}

}  // namespace duo
