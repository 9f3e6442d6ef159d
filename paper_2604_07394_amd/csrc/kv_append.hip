// flux_kv_append: copy new K/V rows to the tail of each sequence's cache, then bump the lengths.
// flux_kv_append_ring / flux_kv_compact_ring: the same copy into the sink + ring layout a sparse layer
// keeps for decode (Sec. 3.3): position p sits in row p for p < n_sink, else in row
// n_sink + (p - n_sink) % window.
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
  int ring, n_sink, window;                // ring != 0: sink + ring rows, lengths are logical
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
      const int len0 = a.kv_len[lo];
      const int pos = len0 + (t - a.cu_new[lo]);
      int row = pos;
      bool keep = pos >= 0 && pos < a.capacity;
      if (a.ring) {
        // only rows that are still resident after the whole call are written: the sinks and the last
        // `window` positions (an earlier row of this call may share a ring row with a later one)
        const int len1 = len0 + (a.cu_new[lo + 1] - a.cu_new[lo]);
        keep = pos >= 0 && (pos < a.n_sink || pos >= len1 - a.window);
        row = pos < a.n_sink ? pos : a.n_sink + (pos - a.n_sink) % a.window;
      }
      if (keep) {
        const int64_t dst0 = (int64_t)lo * a.stride_b + (int64_t)row * a.stride_t;
        const int64_t src0 = (int64_t)t * cpt;
        for (int c = c0; c < cpt; c += lanes) {
          const int h = c / a.chunks_per_row, cc = c - h * a.chunks_per_row;
          const int64_t off = dst0 + (int64_t)h * a.stride_h + cc;
          // ordinary loads and stores: the appended rows are read again at once by the attention call
          // that follows (nontemporal accesses measured 10 % slower here)
          a.kc[off] = a.k_new[src0 + c];
          a.vc[off] = a.v_new[src0 + c];
        }
      } else if (!a.ring) {
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
      if (!a.ring && len > a.capacity) len = a.capacity;
      a.kv_len[b] = len;
    }
    if (tid == 0) *a.counter = 0;   // ready for the next launch on this stream
  }
}

hipError_t launch_kv_append(const Ctx& c, const flux_kv_cache& cache, int hkv, int d, const void* k_new,
                            const void* v_new, const int32_t* cu_new, int total_new, int ring, int n_sink,
                            int window, hipStream_t s) {
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
  a.ring = ring;
  a.n_sink = n_sink;
  a.window = window;
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

// ---- compaction of a full cache into a ring cache: list entry p of sequence b (p < n_sink: sink p;
// else the (p - n_sink)-th position of the window tail) is copied to its ring row.
struct CompactArgs {
  const u32x4* ks;
  const u32x4* vs;
  int64_t s_stride_b, s_stride_h, s_stride_t;   // in 16-byte chunks
  const int32_t* s_len;
  int s_capacity;
  u32x4* kd;
  u32x4* vd;
  int64_t d_stride_b, d_stride_h, d_stride_t;
  int32_t* d_len;
  int batch, hkv, chunks_per_row, n_sink, window;
};

__global__ __launch_bounds__(256) void kv_compact_ring_kernel(CompactArgs a) {
  const int cpt = a.hkv * a.chunks_per_row;                  // 16-byte chunks per position
  const int lanes = cpt < 256 ? cpt : 256;
  const int tpi = 256 / lanes;
  const int tid = threadIdx.x;
  const int c0 = tid % lanes, trow = tid / lanes;
  const int b = blockIdx.y;
  int len = a.s_len[b];
  len = len < 0 ? 0 : (len > a.s_capacity ? a.s_capacity : len);
  const int n_keep = len < a.n_sink + a.window ? len : a.n_sink + a.window;
  const int tail0 = len - a.window - a.n_sink;               // list entry p >= n_sink is position p + tail0 (if len is longer than the ring)
  if (trow < tpi) {
    for (int p = blockIdx.x * tpi + trow; p < n_keep; p += gridDim.x * tpi) {
      const int pos = (p < a.n_sink || tail0 <= 0) ? p : p + tail0;
      const int row = pos < a.n_sink ? pos : a.n_sink + (pos - a.n_sink) % a.window;
      const int64_t src0 = (int64_t)b * a.s_stride_b + (int64_t)pos * a.s_stride_t;
      const int64_t dst0 = (int64_t)b * a.d_stride_b + (int64_t)row * a.d_stride_t;
      for (int c = c0; c < cpt; c += lanes) {
        const int h = c / a.chunks_per_row, cc = c - h * a.chunks_per_row;
        a.kd[dst0 + (int64_t)h * a.d_stride_h + cc] = a.ks[src0 + (int64_t)h * a.s_stride_h + cc];
        a.vd[dst0 + (int64_t)h * a.d_stride_h + cc] = a.vs[src0 + (int64_t)h * a.s_stride_h + cc];
      }
    }
  }
  if (blockIdx.x == 0 && tid == 0) a.d_len[b] = len;
}

hipError_t launch_kv_compact_ring(const flux_kv_cache& src, const flux_kv_cache& dst, int hkv, int d, int n_sink,
                                  int window, hipStream_t s) {
  CompactArgs a;
  a.ks = (const u32x4*)src.k;
  a.vs = (const u32x4*)src.v;
  a.s_stride_b = src.stride_b / 8;
  a.s_stride_h = src.stride_h / 8;
  a.s_stride_t = src.stride_t / 8;
  a.s_len = src.kv_len;
  a.s_capacity = src.capacity;
  a.kd = (u32x4*)dst.k;
  a.vd = (u32x4*)dst.v;
  a.d_stride_b = dst.stride_b / 8;
  a.d_stride_h = dst.stride_h / 8;
  a.d_stride_t = dst.stride_t / 8;
  a.d_len = dst.kv_len;
  a.batch = src.batch;
  a.hkv = hkv;
  a.chunks_per_row = d / 8;
  a.n_sink = n_sink;
  a.window = window;
  const int cpt = hkv * (d / 8);
  const int tpi = 256 / (cpt < 256 ? cpt : 256);
  long long blocks = ((long long)n_sink + window + tpi - 1) / tpi;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(kv_compact_ring_kernel, dim3((unsigned)blocks, src.batch), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace flux
