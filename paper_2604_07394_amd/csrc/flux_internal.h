// Internal declarations shared by the translation units of libflux (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/flux.h"

// The host-only build that checks the C ABI under sanitizers compiles flux_api.hip as plain C++ (no device pass):
// there the few device-side spellings it meets are given host meanings.
#ifndef __HIP__
#ifndef __device__
#define __device__
#endif
#ifndef __align__
#define __align__(n) __attribute__((aligned(n)))
#endif
#ifndef HIP_SYMBOL
#define HIP_SYMBOL(x) x
#endif
#endif

namespace flux {

// ---- vector types for MFMA operands and packed memory access --------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

#define FLUX_LDS __attribute__((address_space(3)))

constexpr float kLog2e = 1.4426950408889634f;

// The context: a device workspace carved into fixed regions.
struct Ctx {
  int device;              // < 0: no device (argument checking only)
  char* ws;                // device workspace base (256-byte aligned)
  size_t ws_bytes;
  // carved regions (device pointers)
  uint32_t* status;        // sticky status word
  uint32_t* counters;      // kCounters zero-initialised arrival counters; users reset them to zero
  float* small;            // router scratch: pooled vectors and hidden activations
  float* partials;         // split-K partial results
  size_t partials_bytes;
};

// The SA visible set in block units (App. C.3): positions are grouped into blocks of 2^shift; the sinks
// are the positions below sink_lim (whole blocks), the window of query position i starts at
// window_start(i).  shift = 0 is the token-exact rule: sink_lim = n_sink, window_start(i) = i - window + 1.
struct SaGeom {
  int shift, sink_lim, win_blocks;
};
inline SaGeom sa_geom(const flux_attn_cfg& cfg) {
  int b = cfg.sa_block > 1 ? cfg.sa_block : 1, sh = 0;
  while ((1 << sh) < b) ++sh;
  SaGeom g;
  g.shift = sh;
  // rounded up in 64 bits and cut at the largest int: n_sink or window near INT32_MAX ("SA sees everything",
  // Eq. 2 degenerating to Eq. 1) must not wrap.  Positions are below INT32_MAX, so the cut changes nothing.
  const long long sink_lim = (((long long)cfg.n_sink + b - 1) >> sh) << sh;
  const long long win_blocks = ((long long)cfg.window + b - 1) >> sh;
  g.sink_lim = sink_lim > 0x7FFFFFFFll ? 0x7FFFFFFF : (int)sink_lim;
  g.win_blocks = win_blocks > (0x7FFFFFFFll >> sh) ? (0x7FFFFFFF >> sh) : (int)win_blocks;
  return g;
}
#ifdef __HIP__   // device helpers: absent from the host-only build that checks the C ABI under sanitizers
__device__ __forceinline__ int window_start(int i, int shift, int win_blocks) {
  const int lo = ((i >> shift) - win_blocks + 1) << shift;
  return lo > 0 ? lo : 0;
}
#endif

constexpr int kCounters = 64;
constexpr size_t kSmallBytes = 8u << 20;      // router: batch * (splits * hidden + inner) floats
constexpr size_t kHeaderBytes = 4096;         // status + counters
constexpr int kPrefillWideMinRows = 32768;    // prefill launches whose longest prompt has at least this many rows use 256-row workgroups

// ---- launchers (each validates nothing: flux_api.hip has done it) ---------------------------
hipError_t launch_kv_append(const Ctx& c, const flux_kv_cache& cache, int hkv, int d, const void* k_new,
                            const void* v_new, const int32_t* cu_new, int total_new, int ring, int n_sink,
                            int window, hipStream_t s);
hipError_t launch_kv_compact_ring(const flux_kv_cache& src, const flux_kv_cache& dst, int hkv, int d, int n_sink,
                                  int window, hipStream_t s);

struct DecodePlan {
  int units;        // workgroups launched: an upper bound on the units of the split the device takes
  int pps;          // (KV head, query block) pairs per sequence
  int rpu;          // partial rows each unit writes
  int table_floats; // 4-byte words in front of the partial rows that hold the split table (2 per sequence, rounded to 256 B)
};
// The split-K decode cuts the visible keys of a call into about kTargetUnits workgroups of at least kMinChunk keys
// (the split itself is taken on the device; the host only bounds it).
constexpr int kTargetUnits = 1024;              // about that many workgroups: 4 per CU (three fit a CU at once)
constexpr int kMinChunk = 256;                  // 64 keys per wave: keeps the per-chunk merge a small part of the streaming
inline DecodePlan plan_decode(const flux_attn_cfg& cfg, int batch, int max_kv_len) {
  // Upper bound on the units the device-side split can produce: kTargetUnits + one per pair from the chunk
  // size it picks, and no more than the pairs times the chunks of the longest list at the smallest chunk.
  DecodePlan p;
  const int group = cfg.n_q_heads / cfg.n_kv_heads;
  p.pps = cfg.n_kv_heads * ((group + 15) / 16);
  p.rpu = group < 16 ? group : 16;
  const long long pairs = (long long)batch * p.pps;
  const long long by_len = pairs * (((long long)(max_kv_len > 0 ? max_kv_len : 1) + kMinChunk - 1) / kMinChunk);
  const long long by_target = kTargetUnits + pairs;
  p.units = (int)(by_len < by_target ? by_len : by_target);
  if (p.units < 1) p.units = 1;                  // one workgroup always runs: it writes the split table
  p.table_floats = (2 * batch + 63) / 64 * 64;
  return p;
}
inline size_t decode_partials_bytes(const flux_attn_cfg& cfg, const DecodePlan& p) {
  return ((size_t)p.table_floats + (size_t)p.units * p.rpu * (cfg.head_dim + 2)) * sizeof(float);
}
// k_new / v_new != nullptr: the fused decode step (append one row per sequence, then attend: two launches instead of
// three); needs c.counters and a cache that is not a ring.
hipError_t launch_decode(const Ctx& c, const flux_attn_cfg& cfg, const void* q, int max_kv_len,
                         const flux_kv_cache& cache, const uint8_t* mode, int ring, const void* k_new,
                         const void* v_new, void* out, hipStream_t s);

// Keep flags of the block-sparse prefill: [batch, heads, n_qblocks, n_kblocks] bytes, heads = 1 or n_q_heads.
struct BlockMask {
  const uint8_t* flags;
  int heads, n_qblocks, n_kblocks;
};
hipError_t launch_prefill(const Ctx& c, const flux_attn_cfg& cfg, const void* q, const int32_t* cu_q,
                          int max_q_len, int max_kv_len, const flux_kv_cache& cache, const uint8_t* mode,
                          const BlockMask* bm /*nullptr: the sink + window form*/, void* out, hipStream_t s);

// XA block selection: LDS of one workgroup (partial tiles + the masses of 8 query blocks), and the launcher
constexpr int kXaMaxKBlocks = 4096;           // key blocks a prompt may have (262144 positions): the masses live in LDS
constexpr int kXaSingleWalkMaxKBlocks = 1024; // up to here the (square row, key block) table of one workgroup fits LDS (144 KB)
inline size_t xa_select_lds_bytes(int n_kblocks) {
  const size_t table = n_kblocks <= kXaSingleWalkMaxKBlocks ? (size_t)32 * n_kblocks : (size_t)8 * n_kblocks;
  return (size_t)2 * 4 * 512 * 4 + table * 4;
}
hipError_t launch_xa_select(const Ctx& c, const flux_attn_cfg& cfg, const void* q, const int32_t* cu_q, int max_q_len,
                            const flux_kv_cache& cache, float threshold, uint8_t* mask, int n_qblocks, int n_kblocks,
                            hipStream_t s);

hipError_t launch_router(const Ctx& c, const void* x, const int32_t* cu_seqlens, int batch, int hidden, int pool,
                         const void* w1, const void* b1, const void* w2, const void* b2, int inner,
                         uint8_t* mode_out, float* logits_out, hipStream_t s);

// ---- small device helpers -------------------------------------------------------------------
#ifdef __HIP__
__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __builtin_bit_cast(float, bits16 << 16);
}
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __builtin_bit_cast(float, packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __builtin_bit_cast(float, packed & 0xFFFF0000u); }

// two fp32 -> packed bf16 pair (round to nearest even), low half = a
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 r;
  r[0] = (__bf16)a;
  r[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max over the two half-waves: lane l and lane l^32 end up with the same value
__device__ __forceinline__ float max_across_halves(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}
__device__ __forceinline__ float sum_across_halves(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (uint32_t)r[0]) + __builtin_bit_cast(float, (uint32_t)r[1]);
}
#endif  // __HIP__

}  // namespace flux
