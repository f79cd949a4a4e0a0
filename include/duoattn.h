/*
 * duoattn.h - C ABI of the MI355X (gfx950) DuoAttention deployment hot path.
 *
 * What the library computes (paper, Section 2.2 and Section 2.3):
 *   - every KV head of a layer is either a RETRIEVAL head (full causal attention
 *     over all cached tokens) or a STREAMING head (attention restricted to the
 *     first `sink` tokens plus a window of `recent` tokens, a Lambda-shaped mask);
 *   - each layer owns two KV caches: a dense full-length cache for its retrieval
 *     heads and a constant-length cache (sink slots + ring buffer) for its
 *     streaming heads, the latter evicting the oldest non-sink token on append;
 *   - decoding attends one new query per sequence against both caches and writes
 *     the heads side by side; chunked pre-filling does the same for a chunk of
 *     queries, after which the chunk is appended (which prunes the streaming cache).
 *
 * Conventions
 *   - All tensors are DEVICE pointers unless a comment says HOST.  Q/K/V/out are
 *     bf16, row-major, contiguous: [batch, n_tokens, n_heads, head_dim].
 *   - Query head h belongs to KV head h / (n_q_heads / n_kv_heads).
 *   - Positions are 0-based token indices inside one sequence.  A streaming query
 *     at position i sees key j iff j <= i and (j < sink or i - j < recent): the
 *     window counts the query's own position.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work; they never synchronise.  One handle must be driven from
 *     one stream at a time.
 *   - The caller owns Q/K/V/out/lse; the library owns the caches, its split-K
 *     scratch and, for a quantised handle, a bf16 image of one layer's caches that
 *     pre-filling reads; all of it is allocated in duo_cache_create - nothing is
 *     allocated by append, prefill or decode (the paper pre-allocates the cache for
 *     the whole run, Section 3.4).
 *   - Every entry point returns a duo_status_t (0 = ok).  Arguments are validated
 *     before anything is launched; on an argument error nothing has been enqueued
 *     and the handle is unchanged.  DUO_EHIP reports a failed launch (an earlier
 *     launch of the same call may then already be enqueued).  duo_last_error()
 *     gives a thread-local message.
 */
#ifndef DUOATTN_H
#define DUOATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct duo_cache duo_cache_t; /* opaque; owns device memory */

typedef enum {
  DUO_OK = 0,
  DUO_EINVAL = -1, /* bad argument (NULL pointer, unsupported shape, bad mask) */
  DUO_ENOMEM = -2, /* device or host allocation failed */
  DUO_ERANGE = -3, /* append would exceed max_seq, index out of range */
  DUO_ESTATE = -4, /* call does not fit the handle's state or geometry */
  DUO_EHIP = -5    /* a HIP runtime call failed; see duo_last_error() */
} duo_status_t;

typedef enum {
  DUO_KV_BF16 = 0,    /* caches hold the bf16 rows unchanged */
  DUO_KV_FP8_E4M3 = 1,/* caches hold OCP E4M3 codes + one fp32 scale per (token, KV head),
                         K and V separately: scale = amax/448 (1 if the row is all zero),
                         code = RNE-saturating(x / scale), x_hat = value(code) * scale.
                         This stands in for the paper's 4-bit KV setting (Section 3.4,
                         combination with quantization). */
  DUO_KV_INT4 = 2,    /* caches hold 4-bit codes, two per byte (element 2i in the low nibble), + two fp32
                         per (token, KV head), K and V separately: (scale, lo) with lo = min x,
                         scale = (max x - lo) / 15 (1 for a constant row), code = clamp(round-to-nearest-
                         even((x - lo) / scale), 0, 15) in fp32, x_hat = code * scale + lo.  The paper's own
                         capacity setting is a 4-bit KV cache (Section 3.4) whose codec it does not give. */
  DUO_KV_INT8 = 3     /* the 8-bit form of the same asymmetric codec: one code 0..255 per byte,
                         scale = (max x - lo) / 255, the same (scale, lo) fp32 pair per row */
} duo_kv_dtype_t;

typedef struct {
  int32_t n_layers;              /* >= 1 */
  int32_t batch;                 /* >= 1; sequences advance in lock-step */
  int32_t n_q_heads;             /* multiple of n_kv_heads, group size 1, 2, 4 or 8 */
  int32_t n_kv_heads;            /* >= 1 */
  int32_t head_dim;              /* 64 or 128 */
  int32_t sink;                  /* >= 0 attention-sink tokens kept by streaming heads */
  int32_t recent;                /* >= 1 recent tokens kept by streaming heads */
  int64_t max_seq;               /* capacity of the full cache per sequence, >= 1 */
  int32_t kv_dtype;              /* duo_kv_dtype_t */
  const uint8_t* retrieval_mask; /* HOST, [n_layers][n_kv_heads], 1 = retrieval; copied */
  float softmax_scale;           /* 0 -> 1/sqrt(head_dim) */
} duo_config_t;

/* Per-call restatement of the head classes and window geometry.  The ring
 * geometry is fixed when the cache is created, so these must agree with the
 * handle (DUO_ESTATE otherwise).  Passing NULL for the struct, or NULL for
 * head_mask, means "use the handle's". */
typedef struct {
  const uint8_t* head_mask; /* HOST, [n_kv_heads] of this layer, 1 = retrieval */
  int32_t sink;
  int32_t recent;
} duo_call_params_t;

/* Allocate both caches of every layer (Section 2.3, Decoding: two KV caches per
 * layer), the split-K scratch and, when kv_dtype is not DUO_KV_BF16, a bf16 image of
 * the largest layer's caches for pre-filling (batch * heads * max_seq * head_dim * 2
 * bytes for K and for V).  DUO_EINVAL for unsupported shapes, DUO_ENOMEM if the
 * device cannot hold them. */
int duo_cache_create(const duo_config_t* cfg, duo_cache_t** out);
int duo_cache_destroy(duo_cache_t* cache);
/* Forget all tokens of all layers (lengths -> 0).  Cache memory is not cleared. */
int duo_cache_reset(duo_cache_t* cache);
/* Tokens appended so far to `layer`, or a negative duo_status_t. */
int64_t duo_cache_len(const duo_cache_t* cache, int layer);
/* Bytes of device memory held by the caches (not counting scratch and the bf16 image). */
int64_t duo_cache_bytes(const duo_cache_t* cache);

/* Append n_new tokens to `layer` at positions len .. len+n_new-1
 * (Section 2.3: the retrieval cache stores all tokens; the streaming cache keeps
 * only sinks and the most recent tokens, so an append overwrites the oldest
 * non-sink entry).  k, v: [batch, n_new, n_kv_heads, head_dim] bf16.
 * DUO_ERANGE if len + n_new > max_seq. */
int duo_kv_append(duo_cache_t* cache, int layer, const void* k, const void* v,
                  int n_new, const duo_call_params_t* params, void* stream);

/* Chunked pre-filling attention (Section 2.3, Chunked Pre-filling; masks of
 * Section 2.2).  q: [batch, n_new, n_q_heads, head_dim]; k, v: the chunk's own
 * rows [batch, n_new, n_kv_heads, head_dim]; the cache supplies positions < len.
 * Query r of the chunk sits at position len + r.  Retrieval heads see every key
 * up to their own position; streaming heads see the Lambda mask exactly,
 * whatever the chunk size.  The cache is NOT modified: call duo_kv_append with
 * the same k, v afterwards.  out: bf16, shape of q.  lse: fp32
 * [batch, n_q_heads, n_new] natural-log-sum-exp of the scaled scores, or NULL.
 * On a quantised cache the cached positions are attended to as the cache holds them
 * (code * scale [+ minimum], rounded to bf16) and the chunk's own positions as given: every
 * call first brings the handle's bf16 image of this layer up to date from the codes, on
 * `stream` (only the rows appended since the previous chunk of the same layer). */
int duo_attn_prefill(duo_cache_t* cache, int layer, const void* q, const void* k,
                     const void* v, int n_new, const duo_call_params_t* params,
                     void* out, float* lse, void* stream);

/* The same call with the streaming heads' attention as the paper deploys it (Section 2.3,
 * Chunked Pre-filling): plain causal attention over [pruned streaming cache || chunk], i.e. a
 * streaming query sees the sink tokens, the `recent` tokens the cache retained when the chunk
 * started, and every earlier token of its own chunk.  The result depends on where the chunks
 * start (a chunk of the whole sequence is full attention; chunks of one token give a Lambda mask
 * of recent + 1 positions).  Retrieval heads, arguments and errors as duo_attn_prefill. */
int duo_attn_prefill_deployed(duo_cache_t* cache, int layer, const void* q, const void* k,
                              const void* v, int n_new, const duo_call_params_t* params,
                              void* out, float* lse, void* stream);

/* Gate-mixed attention forward of the identification phase (Section 2.2, Optimization-based
 * Identification): for every KV head g with gate alpha[g] in [0, 1] and every query head of its
 * group,  out = alpha[g] * full_attn + (1 - alpha[g]) * streaming_attn  over a whole sequence of
 * n_tokens positions, with full_attn causal and streaming_attn restricted to the cache's sink and
 * recent constants.  No KV cache is read or written: the handle supplies the geometry (batch,
 * heads, head_dim, sink, recent, scale) only, and the layer's head classes play no part.
 * q: [batch, n_tokens, n_q_heads, head_dim]; k, v: [batch, n_tokens, n_kv_heads, head_dim];
 * alpha: HOST fp32 [n_kv_heads] (n_kv_heads <= 64), read before the call returns.
 * block = 0: streaming_attn uses the Lambda mask.  block >= 1: the
 * block-aligned approximation the appendix (Experimental Details) mentions for training: query i
 * sees key j <= i iff block j / block is among the first ceil(sink / block) blocks or fewer than
 * ceil((recent - 1) / block) + 1 blocks before block i / block (the paper shows the pattern in a
 * figure only; this is the smallest block-aligned mask of that shape containing the Lambda mask).
 * out: bf16, shape of q.  One launch and one pass over the causal keys of every head: the keys the
 * streaming mask shows are a subset of them, so each workgroup attends to those first, stores
 * (1 - alpha) * streaming_attn of its rows in out (rounded to bf16), carries the same online-softmax
 * state on over the remaining keys, which turns it into the full-attention state, and writes
 * alpha * full_attn + (the stored term), computed in fp32 and rounded once.  Rows whose causal keys
 * are all inside the streaming mask get the common value of both terms.  workspace: not used, may
 * be NULL (the argument stays for callers built against an earlier form, which needed a buffer of
 * out's size).
 * DUO_EINVAL for NULL q, k, v, alpha or out, n_tokens < 1, n_kv_heads > 64, a gate outside [0, 1]
 * or a negative block. */
int duo_attn_gate_mixed(duo_cache_t* cache, int layer, const void* q, const void* k, const void* v,
                        int n_tokens, const float* alpha, int block, void* out, void* workspace,
                        void* stream);

/* One decoding step (Section 2.3, Decoding).  q: [batch, 1, n_q_heads, head_dim].
 * If k and v are NULL the new token has already been appended and the query sits
 * at position len-1.  If both are given ([batch, 1, n_kv_heads, head_dim]) they
 * are the new token's rows, the query sits at position len, and the result is
 * that of append-then-attend, but the cache is left untouched.
 * out: bf16 [batch, 1, n_q_heads, head_dim]; lse: fp32 [batch, n_q_heads] or NULL.
 * DUO_ESTATE if the cache is empty and no k, v are given. */
int duo_attn_decode(duo_cache_t* cache, int layer, const void* q, const void* k,
                    const void* v, const duo_call_params_t* params, void* out,
                    float* lse, void* stream);

/* duo_attn_decode for callers that must not allocate device memory and want no buffer of the
 * handle's touched behind their back: code recorded into a HIP graph, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, result and errors as duo_attn_decode, but the
 * split-K scratch (partial rows and merge tickets) is a fixed array inside the library, present on
 * every GPU from the moment the library is loaded, instead of the handle's allocation.  The call
 * allocates and frees nothing and synchronises nothing; it enqueues one small kernel that zeroes
 * the tickets, then the decode kernel.
 * Limits: the array holds 4096 partial rows of 128 floats with their (max, sum) pairs (2.1 MB)
 * and 4096 tickets.  A step needs (workgroups sharing retrieval rows + batch * n_kv_heads) *
 * group size rows (at most (1024 + batch * n_kv_heads) * group size), or batch * n_q_heads * key
 * splits rows for one query head per KV head on a bf16 cache, and batch * n_kv_heads tickets;
 * DUO_ERANGE, with the numbers in duo_last_error(), if that does not fit.
 * The array is shared by every call on the same GPU and keeps the previous call's contents:
 * calls that overlap in time on one GPU (two streams, two handles) race - serialise them. */
int duo_attn_decode_static(duo_cache_t* cache, int layer, const void* q, const void* k,
                           const void* v, const duo_call_params_t* params, void* out,
                           float* lse, void* stream);

/* duo_kv_append(n_new = 1) followed by duo_attn_decode(k = v = NULL), as ONE
 * launch: the new token's rows are written into both caches (the length grows
 * by one) while its query attends to the cache plus the new token.  k and v are
 * required.  Same result as the two separate calls. */
int duo_decode_step(duo_cache_t* cache, int layer, const void* q, const void* k,
                    const void* v, const duo_call_params_t* params, void* out,
                    float* lse, void* stream);

/* Test hook: the tokens one (layer, sequence, KV head) cache currently holds, in
 * ascending position order.  k_out/v_out: device buffers of capacity
 * `capacity` rows, each row head_dim bf16 (DUO_KV_BF16) or head_dim bytes
 * (DUO_KV_FP8_E4M3, DUO_KV_INT8) or head_dim / 2 bytes (DUO_KV_INT4); kscale_out/vscale_out: fp32
 * [capacity] (fp8) or fp32 [capacity][2] = (scale, lo) pairs (int4, int8), NULL allowed for bf16; positions_out: device int64 [capacity].  *count_out (HOST)
 * receives the number of rows.  DUO_ERANGE if capacity is too small. */
int duo_cache_export(duo_cache_t* cache, int layer, int batch_idx, int kv_head,
                     void* k_out, void* v_out, float* kscale_out, float* vscale_out,
                     int64_t* positions_out, int64_t capacity, int64_t* count_out,
                     void* stream);

/* Tuning knob: number of workgroups per retrieval (sequence, KV head) that share its keys in
 * decode (0 = automatic).  Results do not depend on it beyond floating-point rounding. */
int duo_set_decode_splits(duo_cache_t* cache, int splits);

/* Tuning knob: which decode kernel serves the handle.  0 = automatic (the vector-unit kernel
 * for one query head per KV head on a bf16 cache, the matrix-core kernel for query groups and
 * fp8 caches), 1 = always the matrix-core kernel.  Same results up to rounding. */
int duo_set_decode_kernel(duo_cache_t* cache, int kernel);

/* Thread-local description of the last error returned on this thread. */
const char* duo_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DUOATTN_H */
