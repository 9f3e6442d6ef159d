// Host-side check of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer.  Links the host-only,
// sanitizer-instrumented build of the library (no device code, no GPU needed) and drives every entry point's
// argument validation and the pure host arithmetic (workspace sizing, the sink / window rounding) on a
// device-less context, with the extreme values a caller can pass.  Any sanitizer report aborts the program.
#include <limits.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/flux.h"

static int failures = 0;
#define EXPECT(expr, want)                                                                   \
  do {                                                                                       \
    const long long got_ = (long long)(expr);                                                \
    if (got_ != (long long)(want)) {                                                         \
      printf("FAIL line %d: %s = %lld, expected %lld\n", __LINE__, #expr, got_, (long long)(want)); \
      ++failures;                                                                            \
    }                                                                                        \
  } while (0)

int main() {
  flux_ctx* ctx = nullptr;
  EXPECT(flux_create(nullptr, -1, 0), FLUX_EINVAL);
  EXPECT(flux_create(&ctx, -1, 0), FLUX_OK);               // a context without a device: validation only
  alignas(16) static char buf[4096];
  void* p = buf;                                            // stands in for device pointers; never dereferenced
  int32_t* pi = (int32_t*)buf;
  uint8_t* pb = (uint8_t*)buf;

  flux_kv_cache kc;
  memset(&kc, 0, sizeof(kc));
  kc.k = p; kc.v = p; kc.kv_len = pi;
  kc.stride_b = 128 * 64 * 2; kc.stride_h = 128 * 64; kc.stride_t = 128;
  kc.batch = 1; kc.capacity = 64;

  flux_attn_cfg cfg = {8, 2, 128, 4, 16, 0.f, 0, 0};
  // ---- strerror for every code, and codes it does not know
  for (int c = 1; c >= -8; --c) EXPECT(flux_strerror(c) != nullptr, 1);
  // ---- attention calls: valid arguments reach the missing device, bad ones are named
  EXPECT(flux_attn_prefill(ctx, &cfg, p, pi, 8, 32, &kc, pb, p, nullptr), FLUX_EHIP);
  EXPECT(flux_attn_decode(ctx, &cfg, p, 32, &kc, pb, p, nullptr), FLUX_EHIP);
  EXPECT(flux_attn_prefill(ctx, nullptr, p, pi, 8, 32, &kc, pb, p, nullptr), FLUX_EINVAL);
  EXPECT(flux_attn_prefill(ctx, &cfg, p, pi, 8, 65, &kc, pb, p, nullptr), FLUX_ECAPACITY);
  EXPECT(flux_attn_prefill(ctx, &cfg, buf + 4, pi, 8, 32, &kc, pb, p, nullptr), FLUX_EINVAL);
  EXPECT(flux_attn_decode(ctx, &cfg, p, -1, &kc, pb, p, nullptr), FLUX_EINVAL);
  EXPECT(flux_attn_decode(ctx, &cfg, p, INT_MAX, &kc, pb, p, nullptr), FLUX_ECAPACITY);
  EXPECT(flux_attn_decode_append(ctx, &cfg, p, p, p, 32, &kc, pb, p, nullptr), FLUX_EHIP);
  EXPECT(flux_attn_decode_append(ctx, &cfg, p, p, p, 0, &kc, pb, p, nullptr), FLUX_EINVAL);
  EXPECT(flux_attn_decode_append(ctx, &cfg, p, nullptr, p, 32, &kc, pb, p, nullptr), FLUX_EINVAL);
  EXPECT(flux_attn_decode_append(ctx, &cfg, p, p, buf + 4, 32, &kc, pb, p, nullptr), FLUX_EINVAL);
  EXPECT(flux_attn_decode_append(ctx, &cfg, p, p, p, INT_MAX, &kc, pb, p, nullptr), FLUX_ECAPACITY);
  // extreme sink / window / block sizes: the rounding must not overflow (UBSan watches the arithmetic)
  const int big[] = {1, 63, 64, 65, 1 << 30, INT_MAX - 65536, INT_MAX - 1, INT_MAX};
  const int blocks[] = {0, 1, 2, 64, 4096, 65536};
  for (int w : big)
    for (int s : big)
      for (int b : blocks) {
        flux_attn_cfg c2 = {8, 2, 128, s, w, 0.f, 1, b};
        EXPECT(flux_attn_decode(ctx, &c2, p, 32, &kc, pb, p, nullptr), FLUX_EHIP);
        EXPECT(flux_attn_decode_append(ctx, &c2, p, p, p, 32, &kc, pb, p, nullptr), FLUX_EHIP);
        EXPECT(flux_attn_prefill(ctx, &c2, p, pi, 8, 32, &kc, pb, p, nullptr), FLUX_EHIP);
        EXPECT(flux_workspace_needed(&c2, 3, 1 << 20) > 0, 1);
        const int rc = flux_attn_decode_ring(ctx, &c2, p, &kc, p, nullptr);
        EXPECT(rc == FLUX_ECAPACITY || rc == FLUX_EHIP, 1);
        EXPECT(flux_attn_decode_static(&c2, p, 32, &kc, pb, p, nullptr, nullptr) != FLUX_EINVAL, 1);
      }
  // ---- workspace arithmetic at the extremes (64-bit sizes, no wrap)
  flux_attn_cfg wide = {256, 1, 128, 4, 16, 0.f, 0, 0};
  EXPECT(flux_workspace_needed(&wide, INT_MAX / 16, INT_MAX) > (size_t)1 << 30, 1);
  EXPECT(flux_workspace_needed(&cfg, 0, 10), 0);
  EXPECT(flux_workspace_needed(&cfg, 1, -1), 0);
  flux_attn_cfg bad_ratio = {8, 3, 128, 4, 16, 0.f, 0, 0};
  EXPECT(flux_workspace_needed(&bad_ratio, 1, 10), 0);
  // a shape whose partial results exceed the static array
  flux_attn_cfg g16 = {256, 16, 128, 4, 64, 0.f, 1, 0};
  flux_kv_cache bigc = kc;
  bigc.batch = 256; bigc.capacity = 1 << 20; bigc.stride_h = (int64_t)1 << 27; bigc.stride_b = (int64_t)1 << 31;
  EXPECT(flux_attn_decode_static(&g16, p, 1 << 20, &bigc, pb, p, nullptr, nullptr), FLUX_EWORKSPACE);
  EXPECT(flux_attn_decode_static(&cfg, p, 32, &kc, pb, p, (uint32_t*)(buf + 2), nullptr), FLUX_EINVAL);
  // ---- append, ring, router
  EXPECT(flux_kv_append(ctx, &kc, 2, 128, p, p, pi, 10, 10, nullptr), FLUX_EHIP);
  EXPECT(flux_kv_append(ctx, &kc, 2, 128, p, p, pi, INT_MAX, INT_MAX, nullptr), FLUX_ECAPACITY);
  EXPECT(flux_kv_append(ctx, &kc, 2, 128, p, p, pi, 5, 6, nullptr), FLUX_EINVAL);
  EXPECT(flux_kv_append_ring(ctx, &kc, 2, 128, INT_MAX, INT_MAX, p, p, pi, 5, 5, nullptr), FLUX_ECAPACITY);
  EXPECT(flux_kv_append_ring(ctx, &kc, 2, 128, 4, 16, p, p, pi, 100, 100, nullptr), FLUX_EHIP);
  EXPECT(flux_kv_compact_ring(ctx, &kc, &kc, 2, 128, INT_MAX, INT_MAX, nullptr), FLUX_ECAPACITY);
  EXPECT(flux_kv_compact_ring(ctx, &kc, &kc, 2, 128, 4, 16, nullptr), FLUX_EHIP);
  EXPECT(flux_router(ctx, p, pi, 2, 4096, 100, p, nullptr, p, nullptr, 256, pb, nullptr, nullptr), FLUX_EHIP);
  EXPECT(flux_router(ctx, p, pi, INT_MAX, 16384, 100, p, nullptr, p, nullptr, 4096, pb, nullptr, nullptr), FLUX_EWORKSPACE);
  EXPECT(flux_router(ctx, p, pi, 2, 4100, 100, p, nullptr, p, nullptr, 256, pb, nullptr, nullptr), FLUX_EINVAL);
  // ---- block-sparse prefill and the XA selection
  EXPECT(flux_attn_prefill_blocksparse(ctx, &cfg, p, pi, 64, 64, &kc, pb, pb, 1, 1, 1, p, nullptr), FLUX_EHIP);
  EXPECT(flux_attn_prefill_blocksparse(ctx, &cfg, p, pi, 64, 64, &kc, pb, pb, 3, 1, 1, p, nullptr), FLUX_EINVAL);
  EXPECT(flux_attn_prefill_blocksparse(ctx, &cfg, p, pi, 64, 64, &kc, pb, pb, 8, INT_MAX, INT_MAX, p, nullptr), FLUX_EHIP);
  EXPECT(flux_xa_select(ctx, &cfg, p, pi, 64, 64, &kc, 16, 0.9f, pb, 1, 1, nullptr), FLUX_EHIP);
  EXPECT(flux_xa_select(ctx, &cfg, p, pi, 64, 64, &kc, 16, 0.9f, pb, INT_MAX, 4097, nullptr), FLUX_EINVAL);
  EXPECT(flux_xa_select(ctx, &cfg, p, pi, 64, 64, &kc, 8, 0.9f, pb, 1, 1, nullptr), FLUX_EINVAL);
  // ---- status and teardown
  EXPECT(flux_last_device_status(ctx, nullptr), FLUX_EHIP);
  EXPECT(flux_last_device_status(nullptr, nullptr), FLUX_EINVAL);
  EXPECT(flux_destroy(ctx), FLUX_OK);
  EXPECT(flux_destroy(nullptr), FLUX_EINVAL);
  if (failures == 0) printf("hostcheck ok\n");
  return failures == 0 ? 0 : 1;
}
