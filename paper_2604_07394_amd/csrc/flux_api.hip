// The C ABI of libflux: context, argument validation, dispatch.  Every check that needs only host
// values runs before anything is launched, so the error paths can be exercised without a GPU.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>

#include "flux_internal.h"

using namespace flux;

// Scratch of flux_attn_decode_static, the entry point for callers that cannot allocate: a sticky status word
// (first 256 bytes) and the split-K partial results.  Every GPU the library runs on holds its own copy of the
// array, at its own address, until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress: kernels and copies are given the address that call returns, never the name.
static __device__ __align__(256) unsigned char scratch[FLUX_STATIC_SCRATCH_BYTES];

struct flux_ctx {
  Ctx c;
};

namespace {

thread_local char g_hip_error[256] = "no HIP error recorded";

int hip_fail(hipError_t e) {
  snprintf(g_hip_error, sizeof(g_hip_error), "HIP error %d: %s", (int)e, hipGetErrorString(e));
  return FLUX_EHIP;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

constexpr size_t kStaticHeader = 256;      // status word of the static scratch; the partials follow
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
char* g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, resolved once per device

// Address of the CURRENT device's copy of `scratch` (resolved at the first use on that device; no allocation
// and no stream work).  The array is zero when the module is loaded, which is all the status word needs.
hipError_t static_scratch(char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = (char*)p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

int check_cfg(const flux_attn_cfg* cfg) {
  if (!cfg) return FLUX_EINVAL;
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return FLUX_EINVAL;
  if (cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0) return FLUX_EINVAL;
  if (cfg->n_q_heads % cfg->n_kv_heads != 0) return FLUX_EINVAL;
  if (cfg->n_sink < 0 || cfg->window < 1) return FLUX_EINVAL;   // the query's own key must stay visible
  if (!(cfg->softmax_scale >= 0.f) || isinf(cfg->softmax_scale)) return FLUX_EINVAL;
  if (cfg->out_dtype != 0 && cfg->out_dtype != 1) return FLUX_EINVAL;
  if (cfg->sa_block < 0 || cfg->sa_block > 65536 || (cfg->sa_block & (cfg->sa_block - 1))) return FLUX_EINVAL;
  return FLUX_OK;
}

int check_cache(const flux_kv_cache* kc, int head_dim) {
  if (!kc || !kc->k || !kc->v || !kc->kv_len) return FLUX_EINVAL;
  if (kc->batch <= 0 || kc->capacity <= 0) return FLUX_EINVAL;
  if (!aligned16(kc->k) || !aligned16(kc->v)) return FLUX_EINVAL;
  if (kc->stride_t < head_dim || kc->stride_h < 0 || kc->stride_b < 0) return FLUX_EINVAL;
  if ((kc->stride_t | kc->stride_h | kc->stride_b) & 7) return FLUX_EINVAL;
  if (kc->stride_t > (1 << 22)) return FLUX_EINVAL;        // 32-bit byte offsets inside a 64-row tile
  return FLUX_OK;
}

}  // namespace

extern "C" {

const char* flux_strerror(int code) {
  switch (code) {
    case FLUX_OK: return "ok";
    case FLUX_EINVAL: return "invalid argument";
    case FLUX_ECAPACITY: return "KV cache capacity exceeded";
    case FLUX_EWORKSPACE: return "context workspace too small for this call";
    case FLUX_EHIP: return g_hip_error;
    case FLUX_ENOMEM: return "out of memory";
    default: return "unknown error code";
  }
}

size_t flux_workspace_needed(const flux_attn_cfg* cfg, int batch, int max_kv_len) {
  if (check_cfg(cfg) != FLUX_OK || batch <= 0 || max_kv_len < 0) return 0;
  const DecodePlan p = plan_decode(*cfg, batch, max_kv_len);
  return kHeaderBytes + kSmallBytes + decode_partials_bytes(*cfg, p);
}

int flux_create(flux_ctx** out, int device, size_t workspace_bytes) {
  if (!out) return FLUX_EINVAL;
  *out = nullptr;
  flux_ctx* ctx = new (std::nothrow) flux_ctx();
  if (!ctx) return FLUX_ENOMEM;
  memset(&ctx->c, 0, sizeof(ctx->c));
  ctx->c.device = device;
  if (device < 0) {   // no device: every call validates its arguments, then reports FLUX_EHIP
    *out = ctx;
    return FLUX_OK;
  }
  if (workspace_bytes == 0) workspace_bytes = kHeaderBytes + kSmallBytes + ((size_t)160 << 20);
  if (workspace_bytes < kHeaderBytes + kSmallBytes + 4096) workspace_bytes = kHeaderBytes + kSmallBytes + 4096;
  hipError_t e = hipSetDevice(device);
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->c.ws, workspace_bytes);
  if (e != hipSuccess) {
    delete ctx;
    return e == hipErrorOutOfMemory ? FLUX_ENOMEM : hip_fail(e);
  }
  e = hipMemset(ctx->c.ws, 0, kHeaderBytes);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    (void)hipFree(ctx->c.ws);
    delete ctx;
    return hip_fail(e);
  }
  ctx->c.ws_bytes = workspace_bytes;
  ctx->c.status = (uint32_t*)ctx->c.ws;
  ctx->c.counters = (uint32_t*)(ctx->c.ws + 256);
  ctx->c.small = (float*)(ctx->c.ws + kHeaderBytes);
  ctx->c.partials = (float*)(ctx->c.ws + kHeaderBytes + kSmallBytes);
  ctx->c.partials_bytes = workspace_bytes - kHeaderBytes - kSmallBytes;
  // set-up on this device also resolves the static scratch of flux_attn_decode_static, so that a caller who
  // created a context first never takes that step inside a region where it would be unwelcome
  char* unused = nullptr;
  e = static_scratch(&unused);
  if (e != hipSuccess) {
    (void)hipFree(ctx->c.ws);
    delete ctx;
    return hip_fail(e);
  }
  *out = ctx;
  return FLUX_OK;
}

int flux_destroy(flux_ctx* ctx) {
  if (!ctx) return FLUX_EINVAL;
  int rc = FLUX_OK;
  if (ctx->c.ws) {
    hipError_t e = hipFree(ctx->c.ws);
    if (e != hipSuccess) rc = hip_fail(e);
  }
  delete ctx;
  return rc;
}

int flux_last_device_status(flux_ctx* ctx, void* stream) {
  if (!ctx) return FLUX_EINVAL;
  if (ctx->c.device < 0) return hip_fail(hipErrorNoDevice);
  uint32_t host = 0;
  hipStream_t s = (hipStream_t)stream;
  hipError_t e = hipMemcpyAsync(&host, ctx->c.status, sizeof(host), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e == hipSuccess && host != 0) {
    // cleared by a copy of zeros rather than a memset node, so the call stays graph-safe
    static const uint32_t zero = 0;
    e = hipMemcpyAsync(ctx->c.status, &zero, sizeof(zero), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
  }
  if (e != hipSuccess) return hip_fail(e);
  return (int)host;
}

int flux_router(flux_ctx* ctx, const void* x, const int32_t* cu_seqlens, int batch, int hidden, int pool,
                const void* w1, const void* b1, const void* w2, const void* b2, int inner,
                uint8_t* mode_out, float* logits_out, void* stream) {
  if (!ctx || !x || !cu_seqlens || !w1 || !w2 || !mode_out) return FLUX_EINVAL;
  if (batch <= 0 || pool < 0) return FLUX_EINVAL;
  if (hidden <= 0 || (hidden & 7) || hidden > 16384) return FLUX_EINVAL;
  if (inner <= 0 || (inner & 7) || inner > 4096) return FLUX_EINVAL;
  if (!aligned16(x) || !aligned16(w1)) return FLUX_EINVAL;
  if ((size_t)batch * ((size_t)hidden + inner) * sizeof(float) > kSmallBytes) return FLUX_EWORKSPACE;
  if (ctx->c.device < 0) return hip_fail(hipErrorNoDevice);
  const hipError_t e = launch_router(ctx->c, x, cu_seqlens, batch, hidden, pool, w1, b1, w2, b2, inner, mode_out,
                                     logits_out, (hipStream_t)stream);
  return e == hipSuccess ? FLUX_OK : hip_fail(e);
}

int flux_kv_append(flux_ctx* ctx, const flux_kv_cache* cache, int n_kv_heads, int head_dim, const void* k_new,
                   const void* v_new, const int32_t* cu_new, int total_new, int max_new, void* stream) {
  if (!ctx || !k_new || !v_new || !cu_new) return FLUX_EINVAL;
  if (head_dim != 64 && head_dim != 128) return FLUX_EINVAL;
  if (n_kv_heads <= 0 || total_new < 0 || max_new < 0 || max_new > total_new) return FLUX_EINVAL;
  const int rc = check_cache(cache, head_dim);
  if (rc != FLUX_OK) return rc;
  if (!aligned16(k_new) || !aligned16(v_new)) return FLUX_EINVAL;
  if (max_new > cache->capacity) return FLUX_ECAPACITY;
  if (ctx->c.device < 0) return hip_fail(hipErrorNoDevice);
  if (total_new == 0) return FLUX_OK;
  const hipError_t e =
      launch_kv_append(ctx->c, *cache, n_kv_heads, head_dim, k_new, v_new, cu_new, total_new, 0, 0, 0, (hipStream_t)stream);
  return e == hipSuccess ? FLUX_OK : hip_fail(e);
}

int flux_attn_prefill(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, const int32_t* cu_q, int max_q_len,
                      int max_kv_len, const flux_kv_cache* cache, const uint8_t* mode, void* out, void* stream) {
  if (!ctx || !q || !cu_q || !mode || !out) return FLUX_EINVAL;
  int rc = check_cfg(cfg);
  if (rc != FLUX_OK) return rc;
  rc = check_cache(cache, cfg->head_dim);
  if (rc != FLUX_OK) return rc;
  if (max_q_len < 0 || max_kv_len < 0 || max_q_len > max_kv_len) return FLUX_EINVAL;
  if (max_kv_len > cache->capacity) return FLUX_ECAPACITY;
  if (!aligned16(q) || !aligned16(out)) return FLUX_EINVAL;
  if (ctx->c.device < 0) return hip_fail(hipErrorNoDevice);
  const hipError_t e =
      launch_prefill(ctx->c, *cfg, q, cu_q, max_q_len, max_kv_len, *cache, mode, nullptr, out, (hipStream_t)stream);
  return e == hipSuccess ? FLUX_OK : hip_fail(e);
}

int flux_attn_prefill_blocksparse(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, const int32_t* cu_q,
                                  int max_q_len, int max_kv_len, const flux_kv_cache* cache, const uint8_t* mode,
                                  const uint8_t* block_mask, int mask_heads, int n_qblocks, int n_kblocks, void* out,
                                  void* stream) {
  if (!ctx || !q || !cu_q || !mode || !out || !block_mask) return FLUX_EINVAL;
  int rc = check_cfg(cfg);
  if (rc != FLUX_OK) return rc;
  rc = check_cache(cache, cfg->head_dim);
  if (rc != FLUX_OK) return rc;
  if (max_q_len < 0 || max_kv_len < 0 || max_q_len > max_kv_len) return FLUX_EINVAL;
  if (max_kv_len > cache->capacity) return FLUX_ECAPACITY;
  if (!aligned16(q) || !aligned16(out)) return FLUX_EINVAL;
  if (mask_heads != 1 && mask_heads != cfg->n_q_heads) return FLUX_EINVAL;
  if (n_qblocks < 1 || n_kblocks < 1) return FLUX_EINVAL;
  // the matrix must at least cover the bounds the caller states; whether it covers a run of queries that starts
  // inside a block is seen on the device (FLUX_DEV_BAD_LENGTH)
  if ((long long)n_kblocks * 64 < max_kv_len || (long long)n_qblocks * 64 < max_q_len) return FLUX_EINVAL;
  if (ctx->c.device < 0) return hip_fail(hipErrorNoDevice);
  const BlockMask bm = {block_mask, mask_heads, n_qblocks, n_kblocks};
  const hipError_t e =
      launch_prefill(ctx->c, *cfg, q, cu_q, max_q_len, max_kv_len, *cache, mode, &bm, out, (hipStream_t)stream);
  return e == hipSuccess ? FLUX_OK : hip_fail(e);
}

int flux_xa_select(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, const int32_t* cu_q, int max_q_len,
                   int max_kv_len, const flux_kv_cache* cache, int stride, float threshold, uint8_t* block_mask,
                   int n_qblocks, int n_kblocks, void* stream) {
  if (!ctx || !q || !cu_q || !block_mask) return FLUX_EINVAL;
  int rc = check_cfg(cfg);
  if (rc != FLUX_OK) return rc;
  rc = check_cache(cache, cfg->head_dim);
  if (rc != FLUX_OK) return rc;
  if (stride != 16) return FLUX_EINVAL;                             // the stride of Table 3 is the one built
  if (!(threshold > 0.f) || !(threshold <= 1.f)) return FLUX_EINVAL;
  if (max_q_len < 0 || max_kv_len < 0 || max_q_len > max_kv_len) return FLUX_EINVAL;
  if (max_kv_len > cache->capacity) return FLUX_ECAPACITY;
  if (!aligned16(q)) return FLUX_EINVAL;
  if (n_qblocks < 1 || n_kblocks < 1 || n_kblocks > kXaMaxKBlocks) return FLUX_EINVAL;
  if ((long long)n_kblocks * 64 < max_kv_len || (long long)n_qblocks * 64 < max_q_len) return FLUX_EINVAL;
  // one workgroup per (sequence, head, 8 query blocks), on a one-dimensional grid
  if ((long long)((n_qblocks + 7) / 8) * cfg->n_q_heads * cache->batch > 0x7FFFFFFFll) return FLUX_EINVAL;
  if (ctx->c.device < 0) return hip_fail(hipErrorNoDevice);
  const hipError_t e = launch_xa_select(ctx->c, *cfg, q, cu_q, max_q_len, *cache, threshold, block_mask, n_qblocks,
                                        n_kblocks, (hipStream_t)stream);
  return e == hipSuccess ? FLUX_OK : hip_fail(e);
}

int flux_attn_decode(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, int max_kv_len,
                     const flux_kv_cache* cache, const uint8_t* mode, void* out, void* stream) {
  if (!ctx || !q || !mode || !out) return FLUX_EINVAL;
  int rc = check_cfg(cfg);
  if (rc != FLUX_OK) return rc;
  rc = check_cache(cache, cfg->head_dim);
  if (rc != FLUX_OK) return rc;
  if (max_kv_len < 0) return FLUX_EINVAL;
  if (max_kv_len > cache->capacity) return FLUX_ECAPACITY;
  if (!aligned16(q) || !aligned16(out)) return FLUX_EINVAL;
  const DecodePlan p = plan_decode(*cfg, cache->batch, max_kv_len);
  if (ctx->c.device >= 0 && decode_partials_bytes(*cfg, p) > ctx->c.partials_bytes) return FLUX_EWORKSPACE;
  if (ctx->c.device < 0) return hip_fail(hipErrorNoDevice);
  const hipError_t e = launch_decode(ctx->c, *cfg, q, max_kv_len, *cache, mode, 0, nullptr, nullptr, out, (hipStream_t)stream);
  return e == hipSuccess ? FLUX_OK : hip_fail(e);
}

int flux_attn_decode_append(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, const void* k_new, const void* v_new,
                            int max_kv_len, const flux_kv_cache* cache, const uint8_t* mode, void* out, void* stream) {
  if (!ctx || !q || !k_new || !v_new || !mode || !out) return FLUX_EINVAL;
  int rc = check_cfg(cfg);
  if (rc != FLUX_OK) return rc;
  rc = check_cache(cache, cfg->head_dim);
  if (rc != FLUX_OK) return rc;
  if (max_kv_len < 1) return FLUX_EINVAL;                    // every list holds at least the appended row
  if (max_kv_len > cache->capacity) return FLUX_ECAPACITY;
  if (!aligned16(q) || !aligned16(out) || !aligned16(k_new) || !aligned16(v_new)) return FLUX_EINVAL;
  const DecodePlan p = plan_decode(*cfg, cache->batch, max_kv_len);
  if (ctx->c.device >= 0 && decode_partials_bytes(*cfg, p) > ctx->c.partials_bytes) return FLUX_EWORKSPACE;
  if (ctx->c.device < 0) return hip_fail(hipErrorNoDevice);
  const hipError_t e = launch_decode(ctx->c, *cfg, q, max_kv_len, *cache, mode, 0, k_new, v_new, out, (hipStream_t)stream);
  return e == hipSuccess ? FLUX_OK : hip_fail(e);
}

int flux_attn_decode_static(const flux_attn_cfg* cfg, const void* q, int max_kv_len, const flux_kv_cache* cache,
                            const uint8_t* mode, void* out, uint32_t* status, void* stream) {
  if (!q || !mode || !out) return FLUX_EINVAL;
  int rc = check_cfg(cfg);
  if (rc != FLUX_OK) return rc;
  rc = check_cache(cache, cfg->head_dim);
  if (rc != FLUX_OK) return rc;
  if (max_kv_len < 0) return FLUX_EINVAL;
  if (max_kv_len > cache->capacity) return FLUX_ECAPACITY;
  if (!aligned16(q) || !aligned16(out) || ((uintptr_t)status & 3u)) return FLUX_EINVAL;
  const DecodePlan p = plan_decode(*cfg, cache->batch, max_kv_len);
  if (decode_partials_bytes(*cfg, p) > FLUX_STATIC_SCRATCH_BYTES - kStaticHeader) return FLUX_EWORKSPACE;
  char* base = nullptr;
  const hipError_t es = static_scratch(&base);
  if (es != hipSuccess) return hip_fail(es);
  // A context on the stack that owns nothing: the kernels take the scratch address as they take the
  // workspace of a flux_create context.  Nothing has to be cleared between calls: the merge kernel reads
  // only partial rows that the split-K kernel of the same call has written, and the status word is sticky.
  Ctx c;
  memset(&c, 0, sizeof(c));
  c.device = 0;
  c.status = status ? status : (uint32_t*)base;
  c.partials = (float*)(base + kStaticHeader);
  c.partials_bytes = FLUX_STATIC_SCRATCH_BYTES - kStaticHeader;
  const hipError_t e = launch_decode(c, *cfg, q, max_kv_len, *cache, mode, 0, nullptr, nullptr, out, (hipStream_t)stream);
  return e == hipSuccess ? FLUX_OK : hip_fail(e);
}

// ---- sparse-decode residency (ring caches)

int flux_kv_append_ring(flux_ctx* ctx, const flux_kv_cache* ring, int n_kv_heads, int head_dim, int n_sink,
                        int window, const void* k_new, const void* v_new, const int32_t* cu_new, int total_new,
                        int max_new, void* stream) {
  if (!ctx || !k_new || !v_new || !cu_new) return FLUX_EINVAL;
  if (head_dim != 64 && head_dim != 128) return FLUX_EINVAL;
  if (n_kv_heads <= 0 || total_new < 0 || max_new < 0 || max_new > total_new) return FLUX_EINVAL;
  if (n_sink < 0 || window < 1) return FLUX_EINVAL;
  const int rc = check_cache(ring, head_dim);
  if (rc != FLUX_OK) return rc;
  if (!aligned16(k_new) || !aligned16(v_new)) return FLUX_EINVAL;
  if ((long long)n_sink + window > ring->capacity) return FLUX_ECAPACITY;
  if (ctx->c.device < 0) return hip_fail(hipErrorNoDevice);
  if (total_new == 0) return FLUX_OK;
  const hipError_t e = launch_kv_append(ctx->c, *ring, n_kv_heads, head_dim, k_new, v_new, cu_new, total_new, 1,
                                        n_sink, window, (hipStream_t)stream);
  return e == hipSuccess ? FLUX_OK : hip_fail(e);
}

int flux_kv_compact_ring(flux_ctx* ctx, const flux_kv_cache* src, const flux_kv_cache* dst, int n_kv_heads,
                         int head_dim, int n_sink, int window, void* stream) {
  if (!ctx) return FLUX_EINVAL;
  if (head_dim != 64 && head_dim != 128) return FLUX_EINVAL;
  if (n_kv_heads <= 0 || n_sink < 0 || window < 1) return FLUX_EINVAL;
  int rc = check_cache(src, head_dim);
  if (rc != FLUX_OK) return rc;
  rc = check_cache(dst, head_dim);
  if (rc != FLUX_OK) return rc;
  if (src->batch != dst->batch) return FLUX_EINVAL;
  if ((long long)n_sink + window > dst->capacity) return FLUX_ECAPACITY;
  if (ctx->c.device < 0) return hip_fail(hipErrorNoDevice);
  const hipError_t e = launch_kv_compact_ring(*src, *dst, n_kv_heads, head_dim, n_sink, window, (hipStream_t)stream);
  return e == hipSuccess ? FLUX_OK : hip_fail(e);
}

int flux_attn_decode_ring(flux_ctx* ctx, const flux_attn_cfg* cfg, const void* q, const flux_kv_cache* ring,
                          void* out, void* stream) {
  if (!ctx || !q || !out) return FLUX_EINVAL;
  int rc = check_cfg(cfg);
  if (rc != FLUX_OK) return rc;
  rc = check_cache(ring, cfg->head_dim);
  if (rc != FLUX_OK) return rc;
  const SaGeom geom = sa_geom(*cfg);
  const long long ring_rows = (long long)geom.sink_lim + ((long long)geom.win_blocks << geom.shift);
  if (ring_rows > ring->capacity) return FLUX_ECAPACITY;
  if (!aligned16(q) || !aligned16(out)) return FLUX_EINVAL;
  const int n_keys = (int)ring_rows;                         // the most any sequence attends to
  const DecodePlan p = plan_decode(*cfg, ring->batch, n_keys);
  if (ctx->c.device >= 0 && decode_partials_bytes(*cfg, p) > ctx->c.partials_bytes) return FLUX_EWORKSPACE;
  if (ctx->c.device < 0) return hip_fail(hipErrorNoDevice);
  const hipError_t e = launch_decode(ctx->c, *cfg, q, n_keys, *ring, nullptr, 1, nullptr, nullptr, out, (hipStream_t)stream);
  return e == hipSuccess ? FLUX_OK : hip_fail(e);
}

}  // extern "C"
