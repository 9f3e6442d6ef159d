// flux_kv_append: copy new K/V rows to the tail of each sequence's cache, then bump the lengths.
//
// One launch.  Every workgroup reads the old lengths, copies its share of 16-byte chunks, and the
// workgroup that finishes last (arrival counter) writes the new lengths, so no copy can observe a
// bumped length.  Pure HBM copy: 16 bytes per lane per access, rows are contiguous on both sides.
#include "flux_internal.h"

namespace flux {

struct AppendArgs {
  const u32x4* k_new;
  const u32x4* v_new;
  const int32_t* cu_new;
  u32x4* kc;
  u32x4* vc;
  int64_t stride_b, stride_h, stride_t;   // in 16-byte chunks
  int32_t* kv_len;
  int batch, capacity, hkv, chunks_per_row;
  int total_new;
  uint32_t* counter;
  uint32_t* status;
};

__global__ __launch_bounds__(256) void kv_append_kernel(AppendArgs a) {
  __shared__ int is_last;
  const int cpt = a.hkv * a.chunks_per_row;                  // 16-byte chunks per token
  const int lanes = cpt < 256 ? cpt : 256;                   // threads that share one token
  const int tpi = 256 / lanes;                               // tokens per workgroup iteration
  const int tid = threadIdx.x;
  const int c0 = tid % lanes, trow = tid / lanes;
  bool overflow = false;
  if (trow < tpi) {
    for (int t = blockIdx.x * tpi + trow; t < a.total_new; t += gridDim.x * tpi) {
      // sequence of token row t: largest b with cu_new[b] <= t
      int lo = 0, hi = a.batch;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.cu_new[mid] <= t) lo = mid; else hi = mid;
      }
      const int pos = a.kv_len[lo] + (t - a.cu_new[lo]);
      if (pos >= 0 && pos < a.capacity) {
        const int64_t dst0 = (int64_t)lo * a.stride_b + (int64_t)pos * a.stride_t;
        const int64_t src0 = (int64_t)t * cpt;
        for (int c = c0; c < cpt; c += lanes) {
          const int h = c / a.chunks_per_row, cc = c - h * a.chunks_per_row;
          const int64_t off = dst0 + (int64_t)h * a.stride_h + cc;
          a.kc[off] = a.k_new[src0 + c];
          a.vc[off] = a.v_new[src0 + c];
        }
      } else {
        overflow = true;
      }
    }
  }
  if (overflow) atomicOr(a.status, (uint32_t)FLUX_DEV_KV_OVERFLOW);

  // The last workgroup to arrive bumps the lengths.  The others only READ kv_len, and a thread's loads
  // have returned (its stores depend on them) before the barrier lets thread 0 count the arrival, so no
  // fence is needed for this read-before-write order.
  __syncthreads();
  if (tid == 0) is_last = (atomicAdd(a.counter, 1u) == gridDim.x - 1);
  __syncthreads();
  if (is_last) {
    for (int b = tid; b < a.batch; b += blockDim.x) {
      const int n = a.cu_new[b + 1] - a.cu_new[b];
      int len = a.kv_len[b] + (n > 0 ? n : 0);
      if (len > a.capacity) len = a.capacity;
      a.kv_len[b] = len;
    }
    if (tid == 0) *a.counter = 0;   // ready for the next launch on this stream
  }
}

hipError_t launch_kv_append(const Ctx& c, const flux_kv_cache& cache, int hkv, int d, const void* k_new,
                            const void* v_new, const int32_t* cu_new, int total_new, hipStream_t s) {
  AppendArgs a;
  a.k_new = (const u32x4*)k_new;
  a.v_new = (const u32x4*)v_new;
  a.cu_new = cu_new;
  a.kc = (u32x4*)cache.k;
  a.vc = (u32x4*)cache.v;
  a.stride_b = cache.stride_b / 8;
  a.stride_h = cache.stride_h / 8;
  a.stride_t = cache.stride_t / 8;
  a.kv_len = cache.kv_len;
  a.batch = cache.batch;
  a.capacity = cache.capacity;
  a.hkv = hkv;
  a.chunks_per_row = d / 8;
  a.total_new = total_new;
  a.counter = c.counters + 0;
  a.status = c.status;
  const int cpt = hkv * (d / 8);
  const int tpi = 256 / (cpt < 256 ? cpt : 256);
  long long blocks = ((long long)total_new + tpi - 1) / tpi;
  if (blocks < 1) blocks = 1;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace flux
