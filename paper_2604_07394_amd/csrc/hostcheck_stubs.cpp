// Launchers of the host-only build that checks the C ABI under sanitizers: nothing can be launched there, so each
// reports that there is no device.  (The real ones live next to their kernels.)
#include "flux_internal.h"

namespace flux {

hipError_t launch_kv_append(const Ctx&, const flux_kv_cache&, int, int, const void*, const void*, const int32_t*, int, int, int,
                            int, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_kv_compact_ring(const flux_kv_cache&, const flux_kv_cache&, int, int, int, int, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_decode(const Ctx&, const flux_attn_cfg&, const void*, int, const flux_kv_cache&, const uint8_t*, int, const void*,
                         const void*, void*, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_prefill(const Ctx&, const flux_attn_cfg&, const void*, const int32_t*, int, int, const flux_kv_cache&,
                          const uint8_t*, const BlockMask*, void*, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_router(const Ctx&, const void*, const int32_t*, int, int, int, const void*, const void*, const void*,
                         const void*, int, uint8_t*, float*, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_xa_select(const Ctx&, const flux_attn_cfg&, const void*, const int32_t*, int, const flux_kv_cache&, float,
                            uint8_t*, int, int, hipStream_t) { return hipErrorNoDevice; }

}  // namespace flux
