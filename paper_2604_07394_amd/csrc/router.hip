// flux_router: Layer Router in its inference form (Sec. 3.1): prefix/suffix pooling of the first
// and last `pool` token rows (App. C.1) -> Context Encoder Linear+SiLU -> Router Head Linear ->
// argmax (tie to FA).  Everything after the bf16 loads is fp32; nothing is rounded in between.
//
// Three launches, all tiny and latency-bound:
//  1. router_pool: partial column sums of the pooled rows.  grid (column blocks, row splits, batch);
//     a lane owns 8 adjacent columns (one 16-byte load per row), the 4 waves of a workgroup take
//     different rows and are merged in LDS.  Row splits keep whole-sequence pooling (pool = 0) spread
//     over the chip; with pool > 0 the cost is independent of the sequence length.
//  2. router_mlp: grid (inner/8, batch); each wave produces two hidden units (dot of a bf16 W1 row
//     with the pooled fp32 vector held in LDS) and applies SiLU.
//  3. router_head: one wave per sequence turns the hidden vector into the two logits and the decision.
#include "flux_internal.h"

namespace flux {

struct PoolArgs {
  const __bf16* x;
  const int32_t* cu;
  int hidden, pool, splits;
  float* psum;            // [batch, splits, hidden]
};

// pooled row number t (0-based among the pooled rows) -> row of the sequence
__device__ __forceinline__ int pooled_row(int t, int n_rows, int pool, bool all) {
  return (all || t < pool) ? t : n_rows - 2 * pool + t;
}

__global__ __launch_bounds__(256) void router_pool_kernel(PoolArgs a) {
  __shared__ float red[4][512];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  const int col = blockIdx.x * 512 + l * 8;
  const int split = blockIdx.y, b = blockIdx.z;
  const int r0 = a.cu[b];
  const int n_rows = a.cu[b + 1] - r0;
  const bool all = a.pool <= 0 || n_rows <= 2 * a.pool;
  const int n_pooled = all ? n_rows : 2 * a.pool;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (col < a.hidden) {
    const __bf16* xc = a.x + (int64_t)r0 * a.hidden + col;
    const int step = 4 * a.splits;
    int t = split * 4 + w;
    // four rows per round, so that four independent 16-byte loads are in flight per lane; every row is
    // read once, hence nontemporal
    for (; t + 3 * step < n_pooled; t += 4 * step) {
      u32x4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        v[u] = __builtin_nontemporal_load((const u32x4*)(xc + (int64_t)pooled_row(t + u * step, n_rows, a.pool, all) * a.hidden));
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[2 * i] += bf16_lo(v[u][i]);
          acc[2 * i + 1] += bf16_hi(v[u][i]);
        }
    }
    for (; t < n_pooled; t += step) {
      const u32x4 v = *(const u32x4*)(xc + (int64_t)pooled_row(t, n_rows, a.pool, all) * a.hidden);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] += bf16_lo(v[i]);
        acc[2 * i + 1] += bf16_hi(v[i]);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) red[w][l * 8 + i] = acc[i];
  __syncthreads();
  for (int c = tid; c < 512; c += 256) {
    const int cc = blockIdx.x * 512 + c;
    if (cc < a.hidden)
      a.psum[((int64_t)b * a.splits + split) * a.hidden + cc] = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
  }
}

struct MlpArgs {
  const float* psum;      // [batch, splits, hidden]
  const int32_t* cu;
  const __bf16* w1;
  const __bf16* b1;
  const __bf16* w2;
  const __bf16* b2;
  float* hbuf;            // [batch, inner]
  int batch, hidden, inner, pool, splits;
};

__global__ __launch_bounds__(256) void router_mlp_kernel(MlpArgs a) {
  extern __shared__ float pvec[];                           // hidden floats
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  const int b = blockIdx.y;
  const int n_rows = a.cu[b + 1] - a.cu[b];
  const bool all = a.pool <= 0 || n_rows <= 2 * a.pool;
  const int n_pooled = all ? n_rows : 2 * a.pool;
  const float inv = n_pooled > 0 ? 1.0f / (float)n_pooled : 0.f;
  // pooled mean: the row-split partial sums are added in split order (fixed, so the result is
  // reproducible); 4 columns per thread and all splits' loads of a round in flight together
  for (int c = tid * 4; c < a.hidden; c += 1024) {
    const float* p = a.psum + (int64_t)b * a.splits * a.hidden + c;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    int sp = 0;
    for (; sp + 8 <= a.splits; sp += 8) {
      f32x4 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = *(const f32x4*)(p + (int64_t)(sp + i) * a.hidden);
#pragma unroll
      for (int i = 0; i < 8; ++i) s += v[i];
    }
    for (; sp < a.splits; ++sp) s += *(const f32x4*)(p + (int64_t)sp * a.hidden);
    *(f32x4*)(pvec + c) = s * inv;
  }
  __syncthreads();
  // two hidden units per wave, their weight rows streamed together
  const int j0 = blockIdx.x * 8 + w * 2;
  if (j0 < a.inner) {
    const bool two = j0 + 1 < a.inner;
    const __bf16* wrow0 = a.w1 + (int64_t)j0 * a.hidden;
    const __bf16* wrow1 = wrow0 + (two ? a.hidden : 0);
    float acc0 = 0.f, acc1 = 0.f;
    for (int c = l * 8; c < a.hidden; c += 512) {
      const u32x4 v0 = *(const u32x4*)(wrow0 + c);
      const u32x4 v1 = *(const u32x4*)(wrow1 + c);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc0 = __builtin_fmaf(bf16_lo(v0[i]), pvec[c + 2 * i], acc0);
        acc0 = __builtin_fmaf(bf16_hi(v0[i]), pvec[c + 2 * i + 1], acc0);
        acc1 = __builtin_fmaf(bf16_lo(v1[i]), pvec[c + 2 * i], acc1);
        acc1 = __builtin_fmaf(bf16_hi(v1[i]), pvec[c + 2 * i + 1], acc1);
      }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      acc0 += __shfl_xor(acc0, off);
      acc1 += __shfl_xor(acc1, off);
    }
    if (l < 2 && (l == 0 || two)) {
      float acc = l == 0 ? acc0 : acc1;
      const int j = j0 + l;
      if (a.b1) acc += (float)a.b1[j];
      a.hbuf[(int64_t)b * a.inner + j] = acc / (1.0f + expf(-acc));   // SiLU
    }
  }
}

struct HeadArgs {
  const float* hbuf;      // [batch, inner]
  const __bf16* w2;
  const __bf16* b2;
  int inner;
  uint8_t* mode_out;
  float* logits_out;
};

// Router Head: two dot products of length `inner` per sequence, then the hard decision.
__global__ __launch_bounds__(64) void router_head_kernel(HeadArgs a) {
  const int l = threadIdx.x, bb = blockIdx.x;
  float s0 = 0.f, s1 = 0.f;
  for (int j = l; j < a.inner; j += 64) {
    const float hv = a.hbuf[(int64_t)bb * a.inner + j];
    s0 = __builtin_fmaf((float)a.w2[j], hv, s0);
    s1 = __builtin_fmaf((float)a.w2[a.inner + j], hv, s1);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    s0 += __shfl_xor(s0, off);
    s1 += __shfl_xor(s1, off);
  }
  if (l == 0) {
    if (a.b2) {
      s0 += (float)a.b2[0];
      s1 += (float)a.b2[1];
    }
    a.mode_out[bb] = s0 >= s1 ? 1 : 0;                       // argmax, tie -> index 0 = FA
    if (a.logits_out) {
      a.logits_out[2 * bb] = s0;
      a.logits_out[2 * bb + 1] = s1;
    }
  }
}

hipError_t launch_router(const Ctx& c, const void* x, const int32_t* cu_seqlens, int batch, int hidden, int pool,
                         const void* w1, const void* b1, const void* w2, const void* b2, int inner,
                         uint8_t* mode_out, float* logits_out, hipStream_t s) {
  // row splits: ~32 pooled rows per workgroup when the count is known, 64 splits for whole-sequence
  // pooling, bounded by the scratch region
  int splits = pool > 0 ? (2 * pool + 31) / 32 : 64;
  const size_t per_split = (size_t)batch * hidden * sizeof(float);
  const size_t hbytes = (size_t)batch * inner * sizeof(float);
  size_t room = kSmallBytes - hbytes;
  if ((size_t)splits * per_split > room) splits = (int)(room / per_split);
  if (splits < 1) return hipErrorInvalidValue;              // flux_router has checked the sizes
  float* psum = c.small;
  float* hbuf = c.small + (size_t)splits * batch * hidden;

  PoolArgs pa{(const __bf16*)x, cu_seqlens, hidden, pool, splits, psum};
  hipLaunchKernelGGL(router_pool_kernel, dim3((hidden + 511) / 512, splits, batch), dim3(256), 0, s, pa);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  MlpArgs ma;
  ma.psum = psum;
  ma.cu = cu_seqlens;
  ma.w1 = (const __bf16*)w1;
  ma.b1 = (const __bf16*)b1;
  ma.w2 = (const __bf16*)w2;
  ma.b2 = (const __bf16*)b2;
  ma.hbuf = hbuf;
  ma.batch = batch;
  ma.hidden = hidden;
  ma.inner = inner;
  ma.pool = pool;
  ma.splits = splits;
  hipLaunchKernelGGL(router_mlp_kernel, dim3((inner + 7) / 8, batch), dim3(256), hidden * sizeof(float), s, ma);
  e = hipGetLastError();
  if (e != hipSuccess) return e;

  HeadArgs ha{hbuf, (const __bf16*)w2, (const __bf16*)b2, inner, mode_out, logits_out};
  hipLaunchKernelGGL(router_head_kernel, dim3(batch), dim3(64), 0, s, ha);
  return hipGetLastError();
}

}  // namespace flux
