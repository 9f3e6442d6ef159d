// flux_attn_prefill: tiled causal GQA attention on bf16 MFMA, Full (Eq. 1) or Sparse (Eq. 2 with the
// sink + window subset of Sec. 4.1 / App. C.3), chosen per sequence by the cached mode byte.
//
// Shape of the computation (one workgroup = 128 query rows of one head, 4 waves x 32 rows):
//   for each VISITED 64-key block (FA: all blocks up to the diagonal; SA: the sink blocks and the
//   blocks that intersect the tile's window, nothing else: hidden blocks are skipped, not masked)
//     S^T[key][q]  = K[key][:] . Q[q][:]     MFMA 32x32x16 bf16, A = K rows from LDS, B = Q in registers
//     online softmax along keys.  S is kept TRANSPOSED so that one lane owns one query column:
//     the running max / sum are per-lane scalars, 16 of the 32 keys of a block sit in the lane's own
//     accumulator registers, and the only cross-lane step is one half-wave swap.
//     O^T[d][q]   += V^T[d][key] . P^T[key][q]   the accumulator layout of S^T is already the B-operand
//     layout of this product, so P never moves between lanes; V^T comes from row-major LDS through
//     the transposing LDS read.
// Only blocks that straddle the causal diagonal or a window / sink edge evaluate the element mask.
#include "flux_internal.h"

namespace flux {

struct PrefillArgs {
  const __bf16* q;        // [T, Hq, D]
  const int32_t* cu_q;    // [B + 1]
  const __bf16* k;
  const __bf16* v;
  int64_t stride_b, stride_h, stride_t;
  const int32_t* kv_len;
  const uint8_t* mode;
  int capacity;
  int hq, group;
  int n_sink, window;
  int n_qtiles;
  float scale_log2;
  int out_fp32;
  void* out;
};

constexpr int BM = 128;   // query rows per workgroup
constexpr int BN = 64;    // keys per iteration

template <int D>
__global__ __launch_bounds__(256, 2) void prefill_kernel(PrefillArgs a) {
  constexpr int KC = D / 16;            // MFMA k-steps over the head dimension (QK^T)
  constexpr int DB = D / 32;            // 32-wide output blocks over the head dimension (PV)
  constexpr int CPR = D / 8;            // 16-byte chunks per row
  constexpr int NLD = BN * CPR / 256;   // 16-byte chunks per thread per tile
  constexpr int KROW = D + 8;           // LDS row pitch of the K tile (elements): +16 B
  constexpr int VROW = D + 32;          // LDS row pitch of the V tile (elements): +64 B

  __shared__ __attribute__((aligned(16))) __bf16 ks[BN * KROW];
  __shared__ __attribute__((aligned(16))) __bf16 vs[BN * VROW];

  const int tid = threadIdx.x;
  const int w = tid >> 6, l = tid & 63;
  const int g = l >> 5, n = l & 31;
  const int qt = a.n_qtiles - 1 - (int)blockIdx.x;          // heavy tiles first
  const int h = blockIdx.y, b = blockIdx.z;
  const int kvh = h / a.group;

  const int q_begin = a.cu_q[b];
  const int n_q = a.cu_q[b + 1] - q_begin;
  if (qt * BM >= n_q) return;                                // uniform for the workgroup
  int len = a.kv_len[b];
  len = len > a.capacity ? a.capacity : len;
  if (len < 1) return;                                       // nothing cached: nothing to attend
  const int pos0 = max(len - n_q, 0);                        // position of query row 0
  const bool sa = a.mode[b] == 0;

  // query rows of the tile / of this wave, as absolute positions
  const int r_tile_last = min(qt * BM + BM - 1, n_q - 1);
  const int i_tile_min = pos0 + qt * BM;
  const int i_tile_max = pos0 + r_tile_last;
  const int r_w0 = qt * BM + 32 * w;
  const int i_w_min = pos0 + r_w0;
  const int i_w_max = pos0 + min(r_w0 + 31, n_q - 1);       // < i_w_min if the wave has no valid row
  const bool wave_active = r_w0 < n_q;
  const int r_mine = min(r_w0 + n, n_q - 1);                 // clamped row of this lane's query
  const int i_mine = pos0 + r_w0 + n;                        // its position (unclamped)

  // ---- Q operand: lane (n, g) holds d = 16*kc + 8*g .. +7 of its query row
  bf16x8 qf[KC];
  {
    const __bf16* qrow = a.q + ((int64_t)(q_begin + r_mine) * a.hq + h) * D;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) qf[kc] = *(const bf16x8*)(qrow + 16 * kc + 8 * g);
  }

  // ---- visited key blocks: [0, n_a) and [win0, win0 + n_b)
  const int last_blk = i_tile_max / BN;
  int n_a, win0, n_b;
  if (!sa) {
    n_a = last_blk + 1; win0 = 0; n_b = 0;
  } else {
    const int sink_end = min(a.n_sink, i_tile_max + 1);      // keys [0, sink_end) are sinks in reach
    n_a = (sink_end + BN - 1) / BN;
    const int wfirst = max(i_tile_min - a.window + 1, 0);    // first key any row's window reaches
    win0 = max(wfirst / BN, n_a);
    n_b = last_blk + 1 - win0;
    if (n_b < 0) n_b = 0;
  }
  const int n_iter = n_a + n_b;

  const __bf16* kbase = a.k + (int64_t)b * a.stride_b + (int64_t)kvh * a.stride_h;
  const __bf16* vbase = a.v + (int64_t)b * a.stride_b + (int64_t)kvh * a.stride_h;
  const int row_max = len - 1;                               // never read rows that were not appended

  u32x4 kpre[NLD], vpre[NLD];
  auto load_tile = [&](int it) {
    const int j0 = (it < n_a ? it : win0 + (it - n_a)) * BN;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int e = i * 256 + tid;
      const int64_t row = min(j0 + e / CPR, row_max);
      kpre[i] = *(const u32x4*)(kbase + row * a.stride_t + (e % CPR) * 8);
      vpre[i] = *(const u32x4*)(vbase + row * a.stride_t + (e % CPR) * 8);
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int e = i * 256 + tid;
      *(u32x4*)(ks + (e / CPR) * KROW + (e % CPR) * 8) = kpre[i];
      *(u32x4*)(vs + (e / CPR) * VROW + (e % CPR) * 8) = vpre[i];
    }
  };

  float m_run = -INFINITY, l_run = 0.f;
  f32x16 o[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;

  if (n_iter > 0) load_tile(0);
  for (int it = 0; it < n_iter; ++it) {
    __syncthreads();                                         // previous tile fully consumed
    store_tile();
    __syncthreads();
    if (it + 1 < n_iter) load_tile(it + 1);                  // in flight during the math below

    const int j0 = (it < n_a ? it : win0 + (it - n_a)) * BN;
    // does this wave see anything in the block, and does it need the element mask?
    bool skip = !wave_active || j0 > i_w_max;
    bool need_mask = j0 + BN - 1 > i_w_min;
    if (sa) {
      const bool all_sink = j0 + BN <= a.n_sink;
      if (!all_sink) {
        if (j0 >= a.n_sink && j0 + BN - 1 < i_w_min - a.window + 1) skip = true;   // before every window
        if (i_w_max - j0 >= a.window) need_mask = true;                           // some row's window starts inside or after
      }
    }
    if (skip) continue;

    // ---- S^T = K Q^T
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
      const __bf16* krow = ks + (32 * kb + n) * KROW + 8 * g;
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        const bf16x8 kf = *(const bf16x8*)(krow + 16 * kc);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kc], s[kb], 0, 0, 0);
      }
    }
    if (need_mask) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = j0 + 32 * kb + 8 * (r >> 2) + 4 * g + (r & 3);
          bool vis = j <= i_mine;
          if (sa) vis = vis && (j < a.n_sink || i_mine - j < a.window);
          if (!vis) s[kb][r] = -INFINITY;
        }
    }
    // ---- online softmax for this lane's query column
    float mloc = s[0][0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mloc = fmaxf(mloc, s[0][r]);
#pragma unroll
    for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s[1][r]);
    mloc = max_across_halves(mloc);
    const float m_new = fmaxf(m_run, mloc);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;    // a row that has seen no key yet
    const float alpha = fast_exp2((m_run - m_use) * a.scale_log2);
    const float mneg = -m_use * a.scale_log2;
    m_run = m_new;
    bf16x8 pf[2][2];
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        uint32_t pk[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float p0 = fast_exp2(__builtin_fmaf(s[kb][8 * c + 2 * t], a.scale_log2, mneg));
          const float p1 = fast_exp2(__builtin_fmaf(s[kb][8 * c + 2 * t + 1], a.scale_log2, mneg));
          pk[t] = pack_bf16(p0, p1);
          psum += bf16_lo(pk[t]) + bf16_hi(pk[t]);           // the denominator sums the rounded weights
        }
        pf[kb][c] = __builtin_bit_cast(bf16x8, u32x4{pk[0], pk[1], pk[2], pk[3]});
      }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int db = 0; db < DB; ++db) o[db] *= alpha;
    // ---- O^T += V^T P^T
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const __bf16* vrow = vs + (32 * kb + 16 * c + 4 * g + ((l & 15) >> 2)) * VROW + 16 * ((l >> 4) & 1) + 4 * (l & 3);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((FLUX_LDS bf16x4*)(vrow + 32 * db));
          const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((FLUX_LDS bf16x4*)(vrow + 32 * db + 8 * VROW));
          const bf16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb][c], o[db], 0, 0, 0);
        }
      }
  }

  // ---- normalise and store: lane (n, g) holds d = 32*db + 8*(r/4) + 4*g + (r%4) of its query row
  const float l_tot = sum_across_halves(l_run);
  if (r_w0 + n < n_q) {
    const float inv = 1.0f / l_tot;
    const int64_t off = ((int64_t)(q_begin + r_w0 + n) * a.hq + h) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int d = 32 * db + 8 * rr + 4 * g;
        const float x0 = o[db][4 * rr] * inv, x1 = o[db][4 * rr + 1] * inv;
        const float x2 = o[db][4 * rr + 2] * inv, x3 = o[db][4 * rr + 3] * inv;
        if (a.out_fp32) {
          *(f32x4*)((float*)a.out + off + d) = f32x4{x0, x1, x2, x3};
        } else {
          *(u32x2*)((__bf16*)a.out + off + d) = u32x2{pack_bf16(x0, x1), pack_bf16(x2, x3)};
        }
      }
  }
}

hipError_t launch_prefill(const Ctx& c, const flux_attn_cfg& cfg, const void* q, const int32_t* cu_q,
                          int max_q_len, int max_kv_len, const flux_kv_cache& cache, const uint8_t* mode,
                          void* out, hipStream_t s) {
  (void)c;
  (void)max_kv_len;
  const float scale = cfg.softmax_scale != 0.f ? cfg.softmax_scale : 1.0f / sqrtf((float)cfg.head_dim);
  PrefillArgs a;
  a.q = (const __bf16*)q;
  a.cu_q = cu_q;
  a.k = (const __bf16*)cache.k;
  a.v = (const __bf16*)cache.v;
  a.stride_b = cache.stride_b;
  a.stride_h = cache.stride_h;
  a.stride_t = cache.stride_t;
  a.kv_len = cache.kv_len;
  a.mode = mode;
  a.capacity = cache.capacity;
  a.hq = cfg.n_q_heads;
  a.group = cfg.n_q_heads / cfg.n_kv_heads;
  a.n_sink = cfg.n_sink;
  a.window = cfg.window;
  a.n_qtiles = (max_q_len + BM - 1) / BM;
  a.scale_log2 = scale * kLog2e;
  a.out_fp32 = cfg.out_dtype;
  a.out = out;
  if (a.n_qtiles == 0) return hipSuccess;
  const dim3 grid(a.n_qtiles, cfg.n_q_heads, cache.batch);
  if (cfg.head_dim == 128) hipLaunchKernelGGL(prefill_kernel<128>, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(prefill_kernel<64>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace flux
