// Host side of libduoattn: handle management, argument validation, launches.
// The C ABI is documented in include/duoattn.h.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "duo_internal.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int fail_hip(hipError_t e, const char* what) {
  return fail(DUO_EHIP, "%s: %s", what, hipGetErrorString(e));
}

struct Layer {
  duo::LayerView view;
  std::vector<uint8_t> mask;  // host copy, [n_kv_heads]
  int64_t len = 0;
};

}  // namespace

struct duo_cache {
  duo_config_t cfg;
  std::vector<Layer> layers;
  std::vector<void*> allocations;  // every device pointer owned by the handle
  float* part_o = nullptr;
  float* part_ml = nullptr;
  int32_t* tickets = nullptr;
  int max_splits = 0;
  int user_splits = 0;
  bool force_matrix_decode = false;
  int64_t cache_bytes = 0;
  // bf16 image of one quantised layer's rows for pre-filling (allocated at create for quantised
  // handles): K retrieval, V retrieval, K streaming, V streaming.  deq_layer / deq_rows say which
  // layer's retrieval rows the image holds and how many, so that a chunk widens only the rows
  // appended since the previous chunk of the same layer.
  void* deq[4] = {nullptr, nullptr, nullptr, nullptr};
  int deq_layer = -1;
  int64_t deq_rows = 0;
};

// Split-K scratch of duo_attn_decode_static: partial rows (unnormalised output, then (max, sum)
// pairs) and the merge tickets, in device memory that exists from the moment the library is loaded
// until the process ends, one copy per GPU.
constexpr int kStaticRows = 4096;      // partial rows (one per (workgroup, query head) pair that is split)
constexpr int kStaticTickets = 4096;   // (sequence, KV head) pairs
constexpr int kStaticHeadDim = 128;
constexpr size_t kStaticPartO = (size_t)kStaticRows * kStaticHeadDim * sizeof(float);
constexpr size_t kStaticPartMl = (size_t)kStaticRows * 2 * sizeof(float);
constexpr size_t kStaticBytes = kStaticPartO + kStaticPartMl + (size_t)kStaticTickets * sizeof(int32_t);
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

// The array's address on each device, asked of the runtime once per device (the array's name is
// only a host-side stand-in; every use below goes through these pointers).
constexpr int kMaxDevices = 64;
void* g_static_ptr[kMaxDevices] = {};
std::mutex g_static_mu;

int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(DUO_ERANGE, "device index %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail_hip(e, "hipGetSymbolAddress(static split-K scratch)");
    g_static_ptr[dev] = p;
  }
  *out = g_static_ptr[dev];
  return DUO_OK;
}

// Zero n ints (a kernel, not hipMemsetAsync: the call may be recorded into a graph).
__global__ void clear_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

constexpr int kMaxSplits = duo::kMaxDecodeSplits;

hipError_t dev_alloc(duo_cache* c, void** p, size_t bytes) {
  if (bytes == 0) bytes = 256;
  hipError_t e = hipMalloc(p, bytes);
  if (e == hipSuccess) c->allocations.push_back(*p);
  return e;
}

void release(duo_cache* c) {
  for (void* p : c->allocations) (void)hipFree(p);
  delete c;
}

int check_handle_layer(const duo_cache* c, int layer) {
  if (!c) return fail(DUO_EINVAL, "cache handle is NULL");
  if (layer < 0 || layer >= c->cfg.n_layers)
    return fail(DUO_ERANGE, "layer %d outside [0, %d)", layer, c->cfg.n_layers);
  return DUO_OK;
}

int check_params(const duo_cache* c, int layer, const duo_call_params_t* p) {
  if (!p) return DUO_OK;
  if (p->sink != c->cfg.sink || p->recent != c->cfg.recent)
    return fail(DUO_ESTATE, "call asks for sink=%d recent=%d but the cache was created with sink=%d recent=%d",
                p->sink, p->recent, c->cfg.sink, c->cfg.recent);
  if (p->head_mask) {
    const Layer& L = c->layers[layer];
    for (int h = 0; h < c->cfg.n_kv_heads; ++h) {
      if ((p->head_mask[h] != 0) != (L.mask[h] != 0))
        return fail(DUO_ESTATE, "head_mask[%d]=%d disagrees with the mask layer %d was created with",
                    h, (int)p->head_mask[h], layer);
    }
  }
  return DUO_OK;
}

// Splits per retrieval head.  A workgroup with its two register buffers keeps
// enough bytes in flight for its compute unit, so the aim is one resident
// workgroup per compute unit (two when the per-row arithmetic of a query group is
// heavy) with streaming heads counted in, and at least kMinKeysPerSplit keys each.
int choose_splits(const duo_cache* c, const Layer& L, int64_t keys) {
  if (c->user_splits > 0) return c->user_splits < c->max_splits ? c->user_splits : c->max_splits;
  const int64_t kMinKeysPerSplit = 256;
  const int64_t heads = (int64_t)L.view.n_ret * c->cfg.batch;
  if (heads == 0) return 1;
  const int64_t slots = (L.view.group >= 2 || c->cfg.kv_dtype != DUO_KV_BF16) ? 512 : 256;
  int64_t budget = slots - (int64_t)L.view.n_str * c->cfg.batch;
  if (budget < slots / 2) budget = slots / 2;
  int64_t s = budget / heads;
  const int64_t by_len = keys / kMinKeysPerSplit;
  if (s > by_len) s = by_len;
  if (s > c->max_splits) s = c->max_splits;
  if (s < 1) s = 1;
  return (int)s;
}

// Rate (bytes per second) at which W workgroups of the even-split decode kernel, one per compute
// unit, stream bf16 cache rows together: measured on the part at 128K context over 32 distinct
// layers (nothing served from a cache) - about 42 GB/s per workgroup while they are few, 6.5 TB/s
// from about 220 workgroups on.
// Quantised rows are bound by a workgroup's instructions before the memory system saturates:
// about 30 GB/s per workgroup with one code byte per value, 20 GB/s with two codes per byte.
double decode_stream_rate(int64_t W, int kv_dtype) {
  static const double w_pts[] = {0, 64, 96, 128, 160, 192, 224, 256};
  static const double r_pts[] = {0, 2.84e12, 4.0e12, 5.1e12, 5.7e12, 6.35e12, 6.5e12, 6.6e12};
  double r = r_pts[7];
  if (W < 256) {
    int i = 0;
    while (w_pts[i + 1] < (double)W) ++i;
    const double f = ((double)W - w_pts[i]) / (w_pts[i + 1] - w_pts[i]);
    r = r_pts[i] + f * (r_pts[i + 1] - r_pts[i]);
  }
  if (kv_dtype != DUO_KV_BF16) r = std::min(r, (double)W * (kv_dtype == DUO_KV_INT4 ? 20e9 : 30e9));
  return r;
}

// Workgroups that share the retrieval rows in the even-split decode kernel: one resident
// workgroup per compute unit together with the streaming workgroups, a whole number per
// segment while segments are few (no workgroup then crosses a segment border), and at least
// kMinUnits units of 32 rows each.  With few segments the count per segment is the
// one that minimises streaming time plus merge time: the last workgroup of a segment fetches one
// partial row per workgroup and query head, at the 45 GB/s a single compute unit gets for such
// data, so at 128K context 56 workgroups per segment beat 63 and one segment is best served by
// 128 workgroups, not 252.
int choose_ret_workers(const duo_cache* c, const Layer& L, int64_t units_ret) {
  const int64_t segs = (int64_t)L.view.n_ret * c->cfg.batch;
  if (segs == 0) return 0;
  const int64_t total = segs * units_ret;
  const int64_t kMinUnits = 8;
  int64_t w;
  if (c->user_splits > 0) {
    w = segs * c->user_splits;
  } else {
    // bf16 rows: memory-bound, so the compute units that take the short streaming segments are
    // left out of the count; quantised rows: instruction-bound, every compute unit gets a worker
    // and the streaming workgroups run as units free up - unless they are so few that leaving
    // them their units costs less than making them wait for one (measured: 4 of them at batch 1
    // add 2-3 us behind 256 workers, 64 of them at batch 16 would idle a quarter of the part)
    const int64_t str_wgs = (int64_t)L.view.n_str * c->cfg.batch;
    int64_t budget = 256;
    if (c->cfg.kv_dtype == DUO_KV_BF16 || str_wgs <= 8) budget -= str_wgs;
    if (budget < 128) budget = 128;
    w = segs <= budget ? segs * (budget / segs) : budget;
    const int64_t by_len = total / kMinUnits;
    if (w > by_len) w = segs <= by_len ? segs * (by_len / segs) : by_len;
    if (segs <= 8 && w >= 2 * segs) {
      const double bytes = (double)total * duo::kDecodeUnitRows * (L.view.row_bytes + 4.0 * L.view.sc_per_row) * 2.0;
      const double merge_per_part = (double)L.view.group * (L.view.head_dim + 2) * sizeof(float) / 45e9;
      const int64_t per_max = w / segs;
      int64_t best = per_max;
      double best_t = bytes / decode_stream_rate(w, c->cfg.kv_dtype) + (double)per_max * merge_per_part;
      for (int64_t per = per_max - 1; per >= 1; --per) {
        const double t = bytes / decode_stream_rate(segs * per, c->cfg.kv_dtype) + (double)per * merge_per_part;
        if (t < best_t) { best_t = t; best = per; }
      }
      w = segs * best;
    }
  }
  if (w > duo::kMaxDecodeWorkers) w = duo::kMaxDecodeWorkers;
  if (w > total) w = total;
  if (w < 1) w = 1;
  return (int)w;
}

}  // namespace

extern "C" {

const char* duo_last_error(void) { return g_err; }

int duo_cache_create(const duo_config_t* cfg, duo_cache_t** out) {
  if (!cfg || !out) return fail(DUO_EINVAL, "cfg and out must not be NULL");
  *out = nullptr;
  if (cfg->n_layers < 1) return fail(DUO_EINVAL, "n_layers must be >= 1 (got %d)", cfg->n_layers);
  if (cfg->batch < 1) return fail(DUO_EINVAL, "batch must be >= 1 (got %d)", cfg->batch);
  if (cfg->n_kv_heads < 1) return fail(DUO_EINVAL, "n_kv_heads must be >= 1 (got %d)", cfg->n_kv_heads);
  if (cfg->n_q_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads != 0)
    return fail(DUO_EINVAL, "n_q_heads (%d) must be a positive multiple of n_kv_heads (%d)",
                cfg->n_q_heads, cfg->n_kv_heads);
  int group = cfg->n_q_heads / cfg->n_kv_heads;
  if (group != 1 && group != 2 && group != 4 && group != 8)
    return fail(DUO_EINVAL, "query group size %d not supported (1, 2, 4 or 8)", group);
  if (cfg->head_dim != 64 && cfg->head_dim != 128)
    return fail(DUO_EINVAL, "head_dim %d not supported (64 or 128)", cfg->head_dim);
  if (cfg->sink < 0) return fail(DUO_EINVAL, "sink must be >= 0 (got %d)", cfg->sink);
  if (cfg->recent < 1) return fail(DUO_EINVAL, "recent must be >= 1 (got %d)", cfg->recent);
  if ((int64_t)cfg->sink + cfg->recent > (1 << 20))
    return fail(DUO_EINVAL, "sink + recent = %lld exceeds the supported streaming cache length 1048576",
                (long long)cfg->sink + cfg->recent);
  if (cfg->max_seq < 1) return fail(DUO_EINVAL, "max_seq must be >= 1 (got %lld)", (long long)cfg->max_seq);
  if (cfg->max_seq > ((int64_t)1 << 31) - 1024)
    return fail(DUO_EINVAL, "max_seq %lld exceeds the supported 2^31 - 1024", (long long)cfg->max_seq);
  if (cfg->kv_dtype != DUO_KV_BF16 && cfg->kv_dtype != DUO_KV_FP8_E4M3 && cfg->kv_dtype != DUO_KV_INT4 &&
      cfg->kv_dtype != DUO_KV_INT8)
    return fail(DUO_EINVAL, "kv_dtype %d unknown", cfg->kv_dtype);
  if (!cfg->retrieval_mask) return fail(DUO_EINVAL, "retrieval_mask must not be NULL");
  if (!(cfg->softmax_scale >= 0.0f) || std::isinf(cfg->softmax_scale))
    return fail(DUO_EINVAL, "softmax_scale must be finite and >= 0");

  duo_cache* c = new (std::nothrow) duo_cache();
  if (!c) return fail(DUO_ENOMEM, "host allocation failed");
  c->cfg = *cfg;
  c->cfg.retrieval_mask = nullptr;
  c->layers.resize(cfg->n_layers);

  const int sc_per_row = cfg->kv_dtype == DUO_KV_FP8_E4M3 ? 1
                         : (cfg->kv_dtype == DUO_KV_INT4 || cfg->kv_dtype == DUO_KV_INT8 ? 2 : 0);
  const bool quantised = sc_per_row > 0;   // scale arrays are allocated
  const int row_bytes = cfg->kv_dtype == DUO_KV_FP8_E4M3 || cfg->kv_dtype == DUO_KV_INT8 ? cfg->head_dim
                        : (cfg->kv_dtype == DUO_KV_INT4 ? cfg->head_dim / 2 : cfg->head_dim * 2);
  const int64_t str_rows = (int64_t)cfg->sink + cfg->recent;
  const float scale = cfg->softmax_scale > 0.0f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  const int hkv = cfg->n_kv_heads, hq = cfg->n_q_heads;

  // Per-layer tables (head classes and orders), one device array for all layers.
  // Layout per layer: head_info[hkv] | ret_heads[hkv] | str_heads[hkv]
  const int per_layer = 3 * hkv;
  std::vector<int32_t> tables((size_t)per_layer * cfg->n_layers, 0);
  int32_t* d_tables = nullptr;
  hipError_t e = dev_alloc(c, (void**)&d_tables, tables.size() * sizeof(int32_t));
  if (e != hipSuccess) { release(c); return fail(e == hipErrorOutOfMemory ? DUO_ENOMEM : DUO_EHIP, "hipMalloc(tables): %s", hipGetErrorString(e)); }

  for (int l = 0; l < cfg->n_layers; ++l) {
    Layer& L = c->layers[l];
    L.mask.assign(cfg->retrieval_mask + (size_t)l * hkv, cfg->retrieval_mask + (size_t)(l + 1) * hkv);
    int32_t* t = tables.data() + (size_t)l * per_layer;
    int n_ret = 0, n_str = 0;
    for (int h = 0; h < hkv; ++h) {
      if (L.mask[h]) { t[h] = (int32_t)(duo::kRetrievalBit | (uint32_t)n_ret); t[hkv + n_ret] = h; ++n_ret; }
      else { t[h] = n_str; t[2 * hkv + n_str] = h; ++n_str; }
    }
    duo::LayerView& v = L.view;
    memset(&v, 0, sizeof(v));
    v.head_info = (const uint32_t*)(d_tables + (size_t)l * per_layer);
    v.ret_heads = d_tables + (size_t)l * per_layer + hkv;
    v.str_heads = d_tables + (size_t)l * per_layer + 2 * hkv;
    v.n_ret = n_ret; v.n_str = n_str;
    v.batch = cfg->batch; v.n_q_heads = hq; v.n_kv_heads = hkv; v.group = group;
    v.head_dim = cfg->head_dim; v.sink = cfg->sink; v.recent = cfg->recent;
    v.row_bytes = row_bytes; v.kv_mode = cfg->kv_dtype; v.sc_per_row = sc_per_row; v.max_seq = cfg->max_seq; v.scale = scale;

    const size_t ret_bytes = (size_t)cfg->batch * n_ret * (size_t)cfg->max_seq * row_bytes;
    const size_t str_bytes = (size_t)cfg->batch * n_str * (size_t)str_rows * row_bytes;
    const size_t ret_sc = (size_t)cfg->batch * n_ret * (size_t)cfg->max_seq * sizeof(float) * sc_per_row;
    const size_t str_sc = (size_t)cfg->batch * n_str * (size_t)str_rows * sizeof(float) * sc_per_row;
    struct { void** p; size_t bytes; bool needed; } want[] = {
        {(void**)&v.k_ret, ret_bytes, n_ret > 0}, {(void**)&v.v_ret, ret_bytes, n_ret > 0},
        {(void**)&v.k_str, str_bytes, n_str > 0}, {(void**)&v.v_str, str_bytes, n_str > 0},
        {(void**)&v.ks_ret, ret_sc, quantised && n_ret > 0}, {(void**)&v.vs_ret, ret_sc, quantised && n_ret > 0},
        {(void**)&v.ks_str, str_sc, quantised && n_str > 0}, {(void**)&v.vs_str, str_sc, quantised && n_str > 0}};
    for (auto& w : want) {
      if (!w.needed) continue;
      e = dev_alloc(c, w.p, w.bytes);
      if (e != hipSuccess) {
        release(c);
        return fail(e == hipErrorOutOfMemory ? DUO_ENOMEM : DUO_EHIP,
                    "hipMalloc of %zu bytes for layer %d failed: %s", w.bytes, l, hipGetErrorString(e));
      }
      c->cache_bytes += (int64_t)w.bytes;
    }
  }
  e = hipMemcpy(d_tables, tables.data(), tables.size() * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e != hipSuccess) { release(c); return fail_hip(e, "hipMemcpy(tables)"); }

  if (quantised) {
    // The pre-filling kernel reads bf16 rows: a quantised handle owns a bf16 image of one layer's
    // caches (the largest layer's), refreshed from the codes by the pre-filling calls.
    int max_ret = 0, max_str = 0;
    for (const Layer& x : c->layers) { max_ret = std::max(max_ret, x.view.n_ret); max_str = std::max(max_str, x.view.n_str); }
    const size_t row = (size_t)cfg->head_dim * 2;
    const size_t img_ret = (size_t)cfg->batch * max_ret * (size_t)cfg->max_seq * row;
    const size_t img_str = (size_t)cfg->batch * max_str * (size_t)str_rows * row;
    const size_t want_img[4] = {img_ret, img_ret, img_str, img_str};
    for (int i = 0; i < 4; ++i) {
      e = dev_alloc(c, &c->deq[i], want_img[i]);
      if (e != hipSuccess) {
        release(c);
        return fail(e == hipErrorOutOfMemory ? DUO_ENOMEM : DUO_EHIP,
                    "hipMalloc of %zu bytes for the bf16 pre-filling image of a quantised layer failed: %s", want_img[i],
                    hipGetErrorString(e));
      }
    }
  }

  c->max_splits = kMaxSplits;
  // split-K scratch: the larger of [batch][q head][split] rows and, for the even-split kernel,
  // (workgroups + segments) rows per query head of a group
  size_t part_rows = (size_t)cfg->batch * hq * c->max_splits;
  const size_t sk_rows = ((size_t)duo::kMaxDecodeWorkers + (size_t)cfg->batch * hkv) * group;
  if (sk_rows > part_rows) part_rows = sk_rows;
  e = dev_alloc(c, (void**)&c->part_o, part_rows * cfg->head_dim * sizeof(float));
  if (e == hipSuccess) e = dev_alloc(c, (void**)&c->part_ml, part_rows * 2 * sizeof(float));
  if (e == hipSuccess) e = dev_alloc(c, (void**)&c->tickets, (size_t)cfg->batch * hkv * sizeof(int32_t));
  if (e != hipSuccess) { release(c); return fail(DUO_ENOMEM, "hipMalloc(split-K scratch): %s", hipGetErrorString(e)); }
  e = hipMemset(c->tickets, 0, (size_t)cfg->batch * hkv * sizeof(int32_t));
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) { release(c); return fail_hip(e, "clearing the split-K tickets"); }
  *out = c;
  return DUO_OK;
}

int duo_cache_destroy(duo_cache_t* c) {
  if (!c) return fail(DUO_EINVAL, "cache handle is NULL");
  release(c);
  return DUO_OK;
}

int duo_cache_reset(duo_cache_t* c) {
  if (!c) return fail(DUO_EINVAL, "cache handle is NULL");
  for (auto& L : c->layers) L.len = 0;
  c->deq_layer = -1;
  c->deq_rows = 0;
  return DUO_OK;
}

int64_t duo_cache_len(const duo_cache_t* c, int layer) {
  int rc = check_handle_layer(c, layer);
  if (rc != DUO_OK) return rc;
  return c->layers[layer].len;
}

int64_t duo_cache_bytes(const duo_cache_t* c) {
  if (!c) return fail(DUO_EINVAL, "cache handle is NULL");
  return c->cache_bytes;
}

int duo_set_decode_splits(duo_cache_t* c, int splits) {
  if (!c) return fail(DUO_EINVAL, "cache handle is NULL");
  if (splits < 0 || splits > c->max_splits)
    return fail(DUO_ERANGE, "splits %d outside [0, %d]", splits, c->max_splits);
  c->user_splits = splits;
  return DUO_OK;
}

int duo_set_decode_kernel(duo_cache_t* c, int kernel) {
  if (!c) return fail(DUO_EINVAL, "cache handle is NULL");
  if (kernel != 0 && kernel != 1) return fail(DUO_EINVAL, "kernel must be 0 (automatic) or 1 (matrix-core), got %d", kernel);
  c->force_matrix_decode = kernel == 1;
  return DUO_OK;
}

int duo_kv_append(duo_cache_t* c, int layer, const void* k, const void* v, int n_new,
                  const duo_call_params_t* params, void* stream) {
  int rc = check_handle_layer(c, layer);
  if (rc != DUO_OK) return rc;
  if (!k || !v) return fail(DUO_EINVAL, "k and v must not be NULL");
  if (n_new < 1) return fail(DUO_EINVAL, "n_new must be >= 1 (got %d)", n_new);
  if ((rc = check_params(c, layer, params)) != DUO_OK) return rc;
  Layer& L = c->layers[layer];
  if (L.len + n_new > c->cfg.max_seq)
    return fail(DUO_ERANGE, "append of %d tokens at length %lld exceeds max_seq %lld", n_new,
                (long long)L.len, (long long)c->cfg.max_seq);
  hipError_t e = duo::launch_append(L.view, k, v, L.len, n_new, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(e, "append launch");
  L.len += n_new;
  return DUO_OK;
}

static int prefill_common(duo_cache_t* c, int layer, const void* q, const void* k, const void* v, int n_new,
                          const duo_call_params_t* params, void* out, float* lse, void* stream, bool chunk_causal) {
  int rc = check_handle_layer(c, layer);
  if (rc != DUO_OK) return rc;
  if (!q || !k || !v || !out) return fail(DUO_EINVAL, "q, k, v and out must not be NULL");
  if (n_new < 1) return fail(DUO_EINVAL, "n_new must be >= 1 (got %d)", n_new);
  if ((rc = check_params(c, layer, params)) != DUO_OK) return rc;
  Layer& L = c->layers[layer];
  if (L.len + n_new > c->cfg.max_seq)
    return fail(DUO_ERANGE, "chunk of %d tokens at length %lld exceeds max_seq %lld", n_new,
                (long long)L.len, (long long)c->cfg.max_seq);
  duo::LayerView view = L.view;
  if (c->cfg.kv_dtype != DUO_KV_BF16) {
    // The pre-filling kernel reads bf16 rows: the rows the layer holds are widened into the handle's
    // bf16 image first (a few bytes of traffic per cached row against the chunk's attention over
    // it) - of the retrieval rows only those appended since the image last held this layer - and
    // the kernel runs on that image; the chunk's own rows are attended to as given.
    if (L.len > 0) {
      const bool same = c->deq_layer == layer && c->deq_rows <= L.len;
      const int64_t first = same ? c->deq_rows : 0;
      hipError_t e = duo::launch_dequant(L.view, first, L.len, c->deq[0], c->deq[1], c->deq[2], c->deq[3], (hipStream_t)stream);
      if (e != hipSuccess) { c->deq_layer = -1; return fail_hip(e, "dequantisation launch"); }
      c->deq_layer = layer;
      c->deq_rows = L.len;
    }
    view.k_ret = (uint8_t*)c->deq[0]; view.v_ret = (uint8_t*)c->deq[1];
    view.k_str = (uint8_t*)c->deq[2]; view.v_str = (uint8_t*)c->deq[3];
    view.ks_ret = view.vs_ret = view.ks_str = view.vs_str = nullptr;
    view.row_bytes = c->cfg.head_dim * 2; view.kv_mode = DUO_KV_BF16; view.sc_per_row = 0;
  }
  duo::PrefillArgs a;
  a.lv = view; a.q = q; a.k = k; a.v = v; a.out = out; a.lse = lse; a.pos0 = L.len; a.n = n_new;
  a.chunk_causal = chunk_causal ? 1 : 0;
  a.dual = 0; a.win_block = 0; a.sink_eff = 0; a.n_local_blocks = 0;
  hipError_t e = duo::launch_prefill(a, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(e, "prefill launch");
  return DUO_OK;
}

int duo_attn_prefill(duo_cache_t* c, int layer, const void* q, const void* k, const void* v,
                     int n_new, const duo_call_params_t* params, void* out, float* lse, void* stream) {
  return prefill_common(c, layer, q, k, v, n_new, params, out, lse, stream, false);
}

int duo_attn_prefill_deployed(duo_cache_t* c, int layer, const void* q, const void* k, const void* v,
                              int n_new, const duo_call_params_t* params, void* out, float* lse, void* stream) {
  return prefill_common(c, layer, q, k, v, n_new, params, out, lse, stream, true);
}

int duo_attn_gate_mixed(duo_cache_t* c, int layer, const void* q, const void* k, const void* v, int n_tokens,
                        const float* alpha, int block, void* out, void* workspace, void* stream) {
  int rc = check_handle_layer(c, layer);
  if (rc != DUO_OK) return rc;
  (void)workspace;   // not used: both terms come from one pass and are mixed in registers and in out
  if (!q || !k || !v || !alpha || !out) return fail(DUO_EINVAL, "q, k, v, alpha and out must not be NULL");
  if (n_tokens < 1) return fail(DUO_EINVAL, "n_tokens must be >= 1 (got %d)", n_tokens);
  if (c->cfg.n_kv_heads > duo::kMaxGateHeads)
    return fail(DUO_EINVAL, "gate-mixed attention supports at most %d KV heads (got %d)", duo::kMaxGateHeads,
                c->cfg.n_kv_heads);
  if (block < 0) return fail(DUO_EINVAL, "block must be >= 0 (got %d)", block);
  for (int g = 0; g < c->cfg.n_kv_heads; ++g)
    if (!(alpha[g] >= 0.0f && alpha[g] <= 1.0f))
      return fail(DUO_EINVAL, "alpha[%d] = %g is outside [0, 1]", g, (double)alpha[g]);
  Layer& L = c->layers[layer];
  duo::PrefillArgs a;
  a.lv = L.view; a.q = q; a.k = k; a.v = v; a.lse = nullptr; a.pos0 = 0; a.n = n_tokens; a.chunk_causal = 0;
  a.win_block = 0; a.sink_eff = 0; a.n_local_blocks = 0;
  for (int g = 0; g < duo::kMaxGateHeads; ++g) a.mix_alpha[g] = g < c->cfg.n_kv_heads ? alpha[g] : 0.0f;
  a.out = out; a.dual = 1;
  if (block >= 1) {
    a.win_block = block;
    a.sink_eff = (c->cfg.sink + block - 1) / block * block;
    a.n_local_blocks = (c->cfg.recent - 1 + block - 1) / block + 1;
  }
  hipError_t e = duo::launch_prefill(a, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(e, "gate-mixed attention launch");
  return DUO_OK;
}

static int decode_common(duo_cache_t* c, int layer, const void* q, const void* k, const void* v,
                         const duo_call_params_t* params, void* out, float* lse, void* stream, bool commit,
                         bool static_scratch_call = false) {
  int rc = check_handle_layer(c, layer);
  if (rc != DUO_OK) return rc;
  if (!q || !out) return fail(DUO_EINVAL, "q and out must not be NULL");
  if ((k == nullptr) != (v == nullptr)) return fail(DUO_EINVAL, "k and v must both be given or both be NULL");
  if (commit && !k) return fail(DUO_EINVAL, "k and v must not be NULL");
  if ((rc = check_params(c, layer, params)) != DUO_OK) return rc;
  Layer& L = c->layers[layer];
  if (!k && L.len == 0) return fail(DUO_ESTATE, "decode on an empty cache needs the new token's k and v");
  if (k && L.len + 1 > c->cfg.max_seq)
    return fail(DUO_ERANGE, "decode at length %lld exceeds max_seq %lld", (long long)L.len, (long long)c->cfg.max_seq);
  duo::DecodeArgs a;
  a.lv = L.view; a.q = q; a.k_new = k; a.v_new = v; a.out = out; a.lse = lse;
  a.part_o = c->part_o; a.part_ml = c->part_ml; a.tickets = c->tickets; a.cache_len = L.len;
  a.splits = choose_splits(c, L, L.len);
  a.commit = commit ? 1 : 0;
  hipError_t e;
  // one query head per KV head on a bf16 cache: the vector-unit kernel; query groups and quantised
  // caches: the matrix-core kernel
  const bool use_sk = c->force_matrix_decode || L.view.group >= 2 || c->cfg.kv_dtype != DUO_KV_BF16;
  if (use_sk) {
    const int64_t unit = duo::kDecodeUnitRows;
    const int64_t rows_str = duo::streaming_rows(L.len, c->cfg.sink, c->cfg.recent);
    a.units_ret = (int32_t)std::max<int64_t>(1, (L.len + unit - 1) / unit);
    a.units_str = (int32_t)std::max<int64_t>(1, (rows_str + unit - 1) / unit);
    a.ret_workers = choose_ret_workers(c, L, a.units_ret);
  }
  if (static_scratch_call) {
    // the scratch this launch will index: partial rows [0, rows) and tickets [0, n_tickets)
    const int64_t n_tickets = (int64_t)c->cfg.batch * c->cfg.n_kv_heads;
    const int64_t rows = use_sk ? ((int64_t)a.ret_workers + n_tickets) * L.view.group
                                : (int64_t)c->cfg.batch * c->cfg.n_q_heads * a.splits;
    if (rows > kStaticRows || n_tickets > kStaticTickets || c->cfg.head_dim > kStaticHeadDim)
      return fail(DUO_ERANGE,
                  "duo_attn_decode_static: this step needs %lld partial rows and %lld tickets; the static scratch "
                  "holds %d rows of %d floats and %d tickets (use duo_attn_decode)",
                  (long long)rows, (long long)n_tickets, kStaticRows, kStaticHeadDim, kStaticTickets);
    void* base = nullptr;
    if ((rc = static_scratch(&base)) != DUO_OK) return rc;
    a.part_o = (float*)base;
    a.part_ml = (float*)((unsigned char*)base + kStaticPartO);
    a.tickets = (int32_t*)((unsigned char*)base + kStaticPartO + kStaticPartMl);
    // every call on this GPU shares the array, which keeps what the last call left: the tickets
    // must start at zero (the partial rows are written before they are read)
    clear_i32_kernel<<<dim3((unsigned)((n_tickets + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(a.tickets, (int)n_tickets);
    e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e, "ticket clear launch");
  }
  e = use_sk ? duo::launch_decode_sk(a, (hipStream_t)stream) : duo::launch_decode(a, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(e, "decode launch");
  if (commit) L.len += 1;
  return DUO_OK;
}

int duo_attn_decode(duo_cache_t* c, int layer, const void* q, const void* k, const void* v,
                    const duo_call_params_t* params, void* out, float* lse, void* stream) {
  return decode_common(c, layer, q, k, v, params, out, lse, stream, false);
}

int duo_attn_decode_static(duo_cache_t* c, int layer, const void* q, const void* k, const void* v,
                           const duo_call_params_t* params, void* out, float* lse, void* stream) {
  return decode_common(c, layer, q, k, v, params, out, lse, stream, false, true);
}

int duo_decode_step(duo_cache_t* c, int layer, const void* q, const void* k, const void* v,
                    const duo_call_params_t* params, void* out, float* lse, void* stream) {
  return decode_common(c, layer, q, k, v, params, out, lse, stream, true);
}

int duo_cache_export(duo_cache_t* c, int layer, int batch_idx, int kv_head, void* k_out, void* v_out,
                     float* kscale_out, float* vscale_out, int64_t* positions_out, int64_t capacity,
                     int64_t* count_out, void* stream) {
  int rc = check_handle_layer(c, layer);
  if (rc != DUO_OK) return rc;
  if (batch_idx < 0 || batch_idx >= c->cfg.batch) return fail(DUO_ERANGE, "batch_idx %d outside [0, %d)", batch_idx, c->cfg.batch);
  if (kv_head < 0 || kv_head >= c->cfg.n_kv_heads) return fail(DUO_ERANGE, "kv_head %d outside [0, %d)", kv_head, c->cfg.n_kv_heads);
  if (!k_out || !v_out || !positions_out || !count_out) return fail(DUO_EINVAL, "k_out, v_out, positions_out and count_out must not be NULL");
  const bool quantised = c->cfg.kv_dtype != DUO_KV_BF16;
  if (quantised && (!kscale_out || !vscale_out)) return fail(DUO_EINVAL, "scale outputs are required for a quantised cache");
  Layer& L = c->layers[layer];
  int64_t count = L.mask[kv_head] ? L.len : duo::streaming_rows(L.len, c->cfg.sink, c->cfg.recent);
  if (count > capacity) return fail(DUO_ERANGE, "export needs %lld rows but capacity is %lld", (long long)count, (long long)capacity);
  *count_out = count;
  if (count == 0) return DUO_OK;
  hipError_t e = duo::launch_export(L.view, batch_idx, kv_head, L.len, k_out, v_out, kscale_out, vscale_out,
                                    positions_out, count, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(e, "export launch");
  return DUO_OK;
}

}  // extern "C"
