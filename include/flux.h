/*
 * flux.h - C ABI of the Flux Attention inference hot path for AMD MI355X (gfx950).
 *
 * The path: a per-layer Layer Router turns the prompt's boundary tokens into a hard
 * Full-Attention / Sparse-Attention decision (paper Sec. 3.1), the decision is cached
 * (Sec. 3.3), and each layer then runs causal grouped-query Full Attention (Eq. 1) or
 * Sparse Attention (Eq. 2; the streaming variant of Sec. 4.1 / App. C.3: sink tokens plus a
 * causal local window) over ONE contiguous bf16 KV cache, in prefill and in decode.
 *
 * General rules
 *  - Every pointer is a raw address.  "dev" = device memory of the context's GPU, "host" =
 *    ordinary host memory.  The caller owns every tensor and the stream; the library owns only
 *    the workspace inside flux_ctx and never allocates in the hot calls.
 *  - All calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL = the default
 *    stream) and never synchronise, except flux_create, flux_destroy, flux_last_device_status.
 *  - Return value: 0 = FLUX_OK, negative = error.  Everything that can be checked from host
 *    arguments is checked before any launch.  What only the device can see (a cache that would
 *    overflow) is clamped so that no access leaves the buffers, and recorded in a sticky status
 *    word readable with flux_last_device_status.
 *  - mode bytes: 1 = FA, 0 = SA (the paper's r_hard; "r_hard = 0 executes SA", Sec. 3.1).
 *  - bf16 tensors are 16-bit brain floats; their base addresses and all strides must be
 *    multiples of 8 elements (16 bytes).  head_dim must be 64 or 128.
 *  - Results are deterministic: same inputs and same shapes give bit-identical outputs.
 *  - Calls that share one flux_ctx must be ordered on one stream (they share its workspace).
 */
#ifndef FLUX_H_
#define FLUX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  FLUX_OK = 0,
  FLUX_EINVAL = -1,      /* null pointer, bad head ratio, unsupported head_dim, negative size,
                            misaligned pointer or stride */
  FLUX_ECAPACITY = -2,   /* growth known on the host exceeds the cache capacity */
  FLUX_EWORKSPACE = -3,  /* the context's workspace is too small for this call */
  FLUX_EHIP = -4,        /* a HIP runtime call failed; text via flux_strerror */
  FLUX_ENOMEM = -5       /* allocation failed in flux_create */
};

/* Bits of the sticky device status word. */
enum {
  FLUX_DEV_KV_OVERFLOW = 1,   /* flux_kv_append dropped rows that did not fit `capacity` */
  FLUX_DEV_BAD_LENGTH = 2     /* a kv_len / cu_seqlens value was inconsistent and was clamped */
};

typedef struct flux_ctx flux_ctx;   /* opaque; owns ONLY its device workspace */

/* Attention shape and the SA pattern of one call.
 * SA visibility (Eq. 2 with the streaming subset): key j is seen by query position i iff
 * j <= i and (j < n_sink or i - j < window); the query's own position counts inside the window.
 * FA (Eq. 1): every j <= i.  Query head h reads KV head h / (n_q_heads / n_kv_heads). */
typedef struct {
  int32_t n_q_heads, n_kv_heads, head_dim;
  int32_t n_sink, window;
  float softmax_scale;      /* 0 => 1/sqrt(head_dim) (the scale Eq. 1 leaves out "for clarity") */
  int32_t out_dtype;        /* 0 = bf16, 1 = fp32 */
  int32_t sa_block;         /* 0 or 1: the token-exact SA rule above.  A power of two b > 1: the
                               block-granular rule of App. C.3 (a block of b positions is the minimum
                               unit of sparsity; the paper uses 64): with B(x) = x / b, key j is seen
                               by query i iff j <= i and (B(j) < ceil(n_sink / b) or
                               B(i) - B(j) < ceil(window / b)). */
} flux_attn_cfg;

/* One LAYER's KV cache, caller-owned: element (b, h, t, d) of K is
 * k[b*stride_b + h*stride_h + t*stride_t + d], d contiguous, same strides for V.
 * head_dim <= stride_t <= 2^22 elements. */
typedef struct {
  void* k;                  /* dev bf16 */
  void* v;                  /* dev bf16 */
  int64_t stride_b, stride_h, stride_t;   /* in elements */
  int32_t* kv_len;          /* dev int32[batch]: valid positions per sequence */
  int32_t batch, capacity;  /* capacity = positions per sequence the buffers can hold */
} flux_kv_cache;

/* Create a context on `device` with a workspace of `workspace_bytes` (0 = a default that covers
 * batch*heads up to 256 and contexts up to 1M positions).  Synchronous.  The context may only
 * be used with that device current. */
int flux_create(flux_ctx** out, int device, size_t workspace_bytes);
int flux_destroy(flux_ctx* ctx);

/* Static text for an error code; for FLUX_EHIP the text of the last HIP error seen. */
const char* flux_strerror(int code);

/* Bytes of workspace flux_attn_decode needs for this shape (pure host arithmetic;
 * prefill, router and append need less than 64 KiB).  0 on invalid arguments. */
size_t flux_workspace_needed(const flux_attn_cfg* cfg, int batch, int max_kv_len);

/* Returns the sticky device status bits (>= 0) and clears them.  Synchronous: copies the word back and
 * waits for `stream`; when a bit was set it then writes the cleared word and waits for `stream` again. */
int flux_last_device_status(flux_ctx* ctx, void* stream);

/* Layer Router, hard-routing inference form (Sec. 3.1 "Architecture and Feature Extraction"
 * and "Deterministic Inference via Hard Routing"; pooling of the first and last 100 tokens,
 * App. C.1).  For each of the `batch` sequences packed in x (rows cu_seqlens[b] ..
 * cu_seqlens[b+1]-1, each `hidden` wide):
 *   p      = mean of the first `pool` and last `pool` rows (every row once if the sequence has
 *            at most 2*pool rows, or if pool == 0)                         fp32
 *   h      = SiLU(w1 p + b1)                                               fp32
 *   logits = w2 h + b2 = (pi_FA, pi_SA)                                    fp32
 *   mode   = 1 (FA) if pi_FA >= pi_SA else 0 (SA)       (argmax; a tie goes to index 0 = FA)
 * x dev bf16 [T, hidden]; cu_seqlens dev int32 [batch+1]; w1 dev bf16 [inner, hidden];
 * b1 dev bf16 [inner] or NULL; w2 dev bf16 [2, inner]; b2 dev bf16 [2] or NULL;
 * mode_out dev uint8 [batch]; logits_out dev fp32 [batch, 2] or NULL.
 * hidden must be a multiple of 8 and at most 16384, inner a multiple of 8 and at most 4096.
 * Cost does not depend on the sequence length when pool > 0. */
int flux_router(flux_ctx* ctx, const void* x, const int32_t* cu_seqlens, int batch, int hidden,
                int pool, const void* w1, const void* b1, const void* w2, const void* b2, int inner,
                uint8_t* mode_out, float* logits_out, void* stream);

/* Append new K/V rows to the tail of each sequence's cache (the cache every later step of
 * Sec. 3.3 reads).  k_new, v_new: dev bf16 [total_new, n_kv_heads, head_dim], rows of sequence b
 * are cu_new[b] .. cu_new[b+1]-1 (dev int32 [batch+1]).  Row r of sequence b goes to position
 * kv_len[b] + r; afterwards kv_len[b] += rows of b.  `total_new` and `max_new` (the largest
 * per-sequence row count) are host values; max_new > capacity gives FLUX_ECAPACITY.  Rows that
 * would pass `capacity` on the device are dropped and FLUX_DEV_KV_OVERFLOW is raised. */
int flux_kv_append(flux_ctx* ctx, const flux_kv_cache* cache, int n_kv_heads, int head_dim,
                   const void* k_new, const void* v_new, const int32_t* cu_new, int total_new,
                   int max_new, void* stream);

/* Prefill attention of one layer (Eq. 1 / Eq. 2, routed per sequence by `mode`, Sec. 3.3).
 * q dev bf16 [T, n_q_heads, head_dim], rows of sequence b are cu_q[b] .. cu_q[b+1]-1 (dev int32
 * [batch+1]).  The n_q(b) queries of sequence b are the LAST n_q(b) positions of its cache:
 * query row r sits at position kv_len[b] - n_q(b) + r (append first, then attend; a chunk of a
 * longer prompt and a whole prompt are the same call).  mode dev uint8 [batch].
 * out dev [T, n_q_heads, head_dim] in cfg->out_dtype.  max_q_len, max_kv_len: host upper bounds
 * on n_q(b) and kv_len[b] (they size the launch; larger than needed is valid, smaller truncates
 * nothing: rows beyond max_q_len are not computed; a bound far above the real lengths costs empty
 * workgroups, and max_q_len from 32768 on (or from 16384 on with max_kv_len from 32768 on) selects
 * the launch shape tuned for long prompts, with the same results bit for bit).  SA tiles that the mask hides are skipped,
 * not masked: their K/V rows are never read.  A 64-key tile that is partly visible is read whole
 * (up to kv_len[b]), so the cached rows below kv_len[b] must hold finite values.  If the device finds n_q(b) > kv_len[b] (the caller did not append first), only the first
 * kv_len[b] query rows of that sequence are computed and FLUX_DEV_BAD_LENGTH is raised. */
int flux_attn_prefill(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, const int32_t* cu_q,
                      int max_q_len, int max_kv_len, const flux_kv_cache* cache,
                      const uint8_t* mode, void* out, void* stream);

/* Prefill attention of one layer with a BLOCK-SPARSE visible set for the sequences whose mode byte is 0 (Eq. 2
 * over an arbitrary set of key blocks: the substrate of the sparse modes of Sec. 4.1 that choose blocks by content;
 * a block of 64 positions is the minimum unit of sparsity, App. C.3).  Same arguments and conventions as
 * flux_attn_prefill; cfg->n_sink, window and sa_block are not used.  A sequence with mode byte 1 runs FA.
 *   block_mask: dev uint8 [batch, mask_heads, n_qblocks, n_kblocks], mask_heads = 1 (all heads share one matrix)
 *               or n_q_heads.  Positions are grouped in blocks of 64.  For sequence b, row rq of its matrix belongs
 *               to the query block  (kv_len[b] - n_q(b)) / 64 + rq  (row 0 is the block that holds its first query
 *               of this call), column kb to key block kb.  Query position i sees key j iff j <= i and
 *               (flag[block of i, block of j] != 0 or block of i == block of j): the causal order holds inside
 *               blocks, and a query's own block is always kept.  Key blocks that no query block of a 128-row tile
 *               keeps are not loaded.
 *   n_kblocks * 64 >= max_kv_len and n_qblocks * 64 >= max_q_len, else FLUX_EINVAL.  A run of queries that starts
 *   inside a block spans one block more than its length suggests: on the device, a pair that lies outside the
 *   matrix counts as not kept and raises FLUX_DEV_BAD_LENGTH. */
int flux_attn_prefill_blocksparse(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, const int32_t* cu_q,
                                  int max_q_len, int max_kv_len, const flux_kv_cache* cache, const uint8_t* mode,
                                  const uint8_t* block_mask, int mask_heads, int n_qblocks, int n_kblocks, void* out,
                                  void* stream);

/* Block selection of the XA sparse mode (Sec. 4.1; Table 3: stride 16, threshold 0.9, selection mode "Inverse",
 * block 64) for whole prompts: writes, for every sequence and query head, the keep matrix that
 * flux_attn_prefill_blocksparse consumes (mask_heads = n_q_heads).  The paper gives the method's name ("Block
 * Sparse Attention with Antidiagonal Scoring") and these parameters, nothing more; what is computed is this reading:
 *   - the scaled scores of a head are cut into squares of stride x stride positions; of a square only the
 *     antidiagonal is sampled (query offset r against key offset stride-1-r: the "Inverse" order), and only the
 *     causal samples inside the prompt; e[a][b] = the mean of the samples of square (a, b);
 *   - softmax over every row a of e (its squares b <= a);
 *   - mass of a block pair = the sum of those probabilities inside it / the rows of e the query block has;
 *   - query block I keeps every key block whose mass is at least the mass of the block at which the masses, taken
 *     in descending order, first reach `threshold` (equal masses are kept together), and always its own block.
 * q, cu_q, cache as in flux_attn_prefill, with n_q(b) == kv_len[b] for every sequence (a whole prompt, appended
 * first; anything else raises FLUX_DEV_BAD_LENGTH and scores the first min(n_q, kv_len) positions).  stride must be
 * 16; 0 < threshold <= 1; cfg->softmax_scale as in Eq. 1; cfg->n_sink, window, sa_block, out_dtype are not used.
 * block_mask: dev uint8 [batch, n_q_heads, n_qblocks, n_kblocks], every byte written (0 or 1);
 * n_kblocks * 64 >= max_kv_len, n_qblocks * 64 >= max_q_len, n_kblocks <= 4096 (262144 positions), else FLUX_EINVAL.
 * max_q_len bounds the prompt lengths (host); a prompt found longer on the device is scored up to the bound, rounded
 * up to whole blocks, and FLUX_DEV_BAD_LENGTH is raised.  Prompts of up to 65536 positions (by that bound) are
 * scored in one walk over the keys, longer ones in two.
 * The masses are computed in fp32 from exact bf16 products: near a tie between the threshold and a partial sum
 * of masses the selection can differ from one made in higher precision. */
int flux_xa_select(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, const int32_t* cu_q, int max_q_len,
                   int max_kv_len, const flux_kv_cache* cache, int stride, float threshold, uint8_t* block_mask,
                   int n_qblocks, int n_kblocks, void* stream);

/* Decode attention of one layer: one query per sequence at position kv_len[b]-1 (append first).
 * q dev bf16 [batch, n_q_heads, head_dim]; out dev [batch, n_q_heads, head_dim].
 * FA streams all kv_len[b] cached rows; SA reads only rows [0, n_sink) and
 * [kv_len[b]-window, kv_len[b]) and never touches the rest (App. B.3).
 * max_kv_len: host upper bound on the number of keys any sequence of this call ATTENDS TO; the
 * largest kv_len[b] (or the capacity) is always valid.  The split of the work over the chip is taken
 * on the device from the lengths and mode bytes found there, so a loose bound costs only idle
 * workgroups and a ragged batch is spread as evenly as a uniform one; the bound limits the launch
 * and the workspace.  A caller that knows every sequence of this layer is SA may pass
 * min(max kv_len, n_sink + window) (both rounded up to multiples of sa_block when that is set).
 * A sequence that attends to more keys than the bound is cut at the bound (its oldest visible
 * keys are kept) and FLUX_DEV_BAD_LENGTH is raised. */
int flux_attn_decode(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, int max_kv_len,
                     const flux_kv_cache* cache, const uint8_t* mode, void* out, void* stream);

/* One whole decode step of a layer (Sec. 3.3, the decode path; App. B.3): the same result and the same cache
 * contents as flux_kv_append of one row per sequence followed by flux_attn_decode, bit for bit, in two launches
 * instead of three (for a sparse layer, whose kernels run for some tens of microseconds, the append launch is a
 * tenth of the step).
 *   k_new, v_new: dev bf16 [batch, n_kv_heads, head_dim], 16-byte aligned: the row sequence b appends at position
 *                 kv_len[b] (before the call).  A sequence whose cache is full drops its row, raises
 *                 FLUX_DEV_KV_OVERFLOW and attends to what is cached, as the pair of calls would.
 *   max_kv_len:   >= 1; bound on the keys any sequence attends to AFTER the append (see flux_attn_decode).
 *   cache:        a full cache (not a ring); kv_len[b] is read by every workgroup and moved on at the end of the
 *                 call (kv_len[b] += 1, cut at the capacity).
 * Other arguments as flux_attn_decode.  The workgroup that owns the end of a sequence's key list stores the new row;
 * workgroups that attend to it read it from k_new / v_new; the merge kernel moves the lengths on. */
int flux_attn_decode_append(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, const void* k_new, const void* v_new,
                            int max_kv_len, const flux_kv_cache* cache, const uint8_t* mode, void* out, void* stream);

/* flux_attn_decode for callers that cannot allocate device memory at all (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): no context, and no hipMalloc / hipFree / allocating library
 * call inside.  The split-K partial results go to a static device array of FLUX_STATIC_SCRATCH_BYTES that
 * every GPU the library runs on holds until the process ends; the call works on the CURRENT device, whose
 * copy of the array is looked up once (at flux_create on that device, else at the first call).
 * Same arguments, kernels and results (bit for bit) as flux_attn_decode, plus
 *   status: dev uint32 (4-byte aligned), caller-owned, or NULL.  The FLUX_DEV_* bits of this call are OR-ed
 *           into it (sticky; the caller reads and clears it); with NULL they go to a word nobody reads.
 * A shape whose partials exceed the array gives FLUX_EWORKSPACE: the partials take
 * min(1024 + pairs, pairs * ceil(max_kv_len / 256)) * min(group, 16) * (head_dim + 2) * 4 bytes with
 * pairs = batch * n_kv_heads * ceil(group / 16), group = n_q_heads / n_kv_heads (2.3 MB for batch 8, 32/8
 * heads of 128 at any length).  All calls on one GPU share that GPU's array: calls that overlap on one GPU
 * (two streams, two threads) race and must be ordered by the caller.  Nothing needs clearing between calls. */
#define FLUX_STATIC_SCRATCH_BYTES ((size_t)16 * 1024 * 1024 + 256)
int flux_attn_decode_static(const flux_attn_cfg* cfg, const void* q, int max_kv_len, const flux_kv_cache* cache,
                            const uint8_t* mode, void* out, uint32_t* status, void* stream);

/* ---- Sparse-decode residency (Sec. 3.3 "Efficient Deployment": a sparse layer keeps only the minimal
 * KV cache its kernel needs and never stores the rest of the history; retrieval layers keep everything).
 *
 * A RING cache is a flux_kv_cache read with these rules: capacity >= n_sink + window rows per
 * (sequence, head); row p < n_sink holds position p; position p >= n_sink lives in row
 * n_sink + (p - n_sink) % window, overwriting the position that has just left the window; kv_len[b] is the
 * LOGICAL length (positions appended so far) and is not bounded by capacity.  The rows stored for a
 * sequence are then exactly the keys Eq. 2 lets its newest position see.  n_sink and window must be the
 * same in every call on one ring cache.  A ring cache serves decode only: the prompt is prefilled on a
 * full cache (the decision exists only after the router has seen the prompt), then compacted. */

/* flux_kv_append on a ring cache.  Same arguments as flux_kv_append plus the ring geometry.  Of the new
 * rows of a sequence only those that are still resident after the call are written (sinks, and the last
 * `window` positions), so any number of rows may be appended at once.  kv_len[b] += rows of b. */
int flux_kv_append_ring(flux_ctx* ctx, const flux_kv_cache* ring, int n_kv_heads, int head_dim, int n_sink,
                        int window, const void* k_new, const void* v_new, const int32_t* cu_new,
                        int total_new, int max_new, void* stream);

/* Copy what a sparse layer keeps from a full cache `src` (after prefill) into the ring cache `dst`:
 * positions [0, n_sink) and [max(len - window, n_sink), len) of every sequence, len = src kv_len[b]
 * (clamped to src capacity); sets dst kv_len[b] = len.  Same batch in both; src is not modified and may
 * be reused for the next layer's prompt. */
int flux_kv_compact_ring(flux_ctx* ctx, const flux_kv_cache* src, const flux_kv_cache* dst, int n_kv_heads,
                         int head_dim, int n_sink, int window, void* stream);

/* flux_attn_decode of a sparse layer on its ring cache: the query of sequence b sits at position
 * kv_len[b] - 1 (append first) and attends to every stored row (Eq. 2).  No mode argument: a ring cache
 * holds a sparse layer.  cfg->n_sink and cfg->window are the ring geometry; with cfg->sa_block = b > 1 the
 * ring must have been filled with n_sink and window rounded up to multiples of b. */
int flux_attn_decode_ring(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, const flux_kv_cache* ring,
                          void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FLUX_H_ */
