// flux_xa_select: the key blocks each query block of a prompt keeps under the XA sparse mode (Sec. 4.1; Table 3:
// stride 16, threshold 0.9, selection mode "Inverse", block 64), written as the keep matrix that
// flux_attn_prefill_blocksparse consumes.  The paper names the method ("Block Sparse Attention with
// Antidiagonal Scoring") and its parameters only; what is computed is this reading of them:
//
//   1. The scaled score matrix of one head is cut into squares of 16 x 16 positions.  Of square (a, b) only the
//      antidiagonal is looked at (query row offset r against key column offset 15 - r: the rows taken in inverse
//      order against the columns), and of it only the causal samples inside the prompt; e[a][b] is their mean.
//   2. Every row a of e becomes probabilities over its squares b <= a by a softmax.
//   3. The mass of block pair (I, J) is the sum of those probabilities over its 4 x 4 squares divided by the rows
//      of e the query block has; the masses of a query block sum to one.
//   4. Query block I keeps every key block whose mass is at least that of the block at which the masses, taken
//      in descending order, first reach the threshold; and always its own block.
//
// Step 1 is a matrix product over 16 * D numbers per square: the 16 query rows of square row a laid end to end
// against the 16 key rows of square column b laid end to end in inverse order.  One workgroup owns 32 square
// rows (512 queries, 8 query blocks) of one head and walks the square columns 16 at a time (256 keys):
//   - the contraction is split over the four waves by the row offset r (wave w takes r = 4w .. 4w+3), so each
//     wave keeps its share of the query operand in registers for the whole kernel and loads only its share of
//     every key tile, straight from global memory in MFMA operand layout (16x16x32 bf16, S^T = K Q^T); a key
//     fragment is used for both halves of the 32 square rows (the kernel is bound by the rate at which key rows
//     reach the CUs, so every use of a fragment counts), and the next tile is asked for once the MFMAs have
//     taken this tile's registers;
//   - the four partial 32 x 16 tiles meet in LDS, where thread (a, b) adds them in wave order.  On the diagonal
//     the samples r < 8 are not causal: exactly the partial tiles of waves 0 and 1, which are left out there;
//     positions past the prompt are zeroed in the operands, and the number of samples of a square is a closed form;
//   - the softmax over a row of squares needs the row's maximum and sum, which are known only at the end of the
//     row.  Prompts of up to 65536 positions are walked once: of every (square row, key block) the logarithm of
//     the summed exponentials of its 4 squares is kept in LDS (it needs no reference), and when the row's
//     log-sum-exp is known the masses are the exponentials of the differences, summed over the 4 rows of a query
//     block.  Longer prompts (the table would not fit) are walked twice: once for (max, sum), once for the
//     probabilities, which are summed 4 x 4 into the masses (a wave of the reduction phase holds the 4 square rows
//     of one query block);
//   - the threshold is found without sorting: the largest mass value t with sum(mass >= t) >= threshold * total,
//     by bisection over the bit patterns of the positive floats (32 steps, one row reduction each).
#include <type_traits>

#include "flux_internal.h"

namespace flux {

struct XaArgs {
  const __bf16* q;        // [T, Hq, D]
  const int32_t* cu_q;    // [B + 1]
  const __bf16* k;
  int64_t stride_b, stride_h, stride_t;   // elements
  const int32_t* kv_len;
  int capacity;
  int hq, group, batch;
  int n_groups;           // workgroups per (sequence, head): groups of 8 query blocks
  float scale;            // softmax scale (not in log2 units)
  float threshold;
  uint8_t* mask;          // [B, Hq, n_qblocks, n_kblocks]
  int n_qblocks, n_kblocks;
  int tab_cols;           // key blocks the host's bound on the prompt length allows (<= n_kblocks): the width of the LDS tables
  int single_walk;        // the (square row, key block) table fits LDS: one walk over the keys
  uint32_t* status;
};

constexpr int kXaRows = 32;        // square rows per workgroup (512 queries): two halves of 16, the N of one MFMA
constexpr int kXaStride = 16;      // positions per square side (Table 3: stride 16)

template <int D>
__global__ __launch_bounds__(256, 2) void xa_select_kernel(XaArgs a) {
  constexpr int ST = D / 8;        // k-steps of 32 numbers per wave: 4 row offsets x D / 32
  constexpr int SPR = D / 32;      // k-steps per row offset
  extern __shared__ __attribute__((aligned(16))) char xa_smem[];
  float* part = (float*)xa_smem;                       // [2 buffers][4 waves][32 a][16 b]
  float* mass = part + 2 * 4 * 512;                    // [8 query blocks][tab_cols]; one walk: [32 square rows][tab_cols]
  float* lse = part;                                   // one walk: log-sum-exp of every square row, kept where the partial
                                                       // tiles were once the walk is over (two workgroups of a 32768-token
                                                       // prompt then fit the LDS of a CU exactly)
  const bool single = a.single_walk != 0;

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;
  const int g = l >> 4, nn = l & 15;
  // ---- which (sequence, head, group of 8 query blocks) this workgroup owns.  Workgroups go to the 8 XCDs round-robin
  // by linear id and every XCD has its own L2: all heads and groups that read one (sequence, KV head) pair get ids of
  // one residue mod 8, longest walks first and the heads of a GQA group next to each other, so that the workgroups
  // resident on an XCD walk the same key rows at about the same time and the rows reach that L2 once.
  int grp, h, b;
  {
    const int i = blockIdx.x;
    const int hkv = a.hq / a.group, n_pairs = a.batch * hkv;
    if ((n_pairs & 7) == 0) {
      const int x = i & 7, j = i >> 3;
      // (the XCD's pairs one after the other, not interleaved group by group: the groups past a short sequence's end
      // are empty workgroups, and at fixed places of a short period they would keep falling to the same CUs)
      const int r = j / (a.group * a.n_groups), gd = (j / a.group) % a.n_groups, gh = j % a.group;
      const int pair = x + 8 * r;
      b = pair / hkv;
      h = (pair % hkv) * a.group + gh;
      grp = a.n_groups - 1 - gd;
    } else {
      grp = a.n_groups - 1 - i % a.n_groups;
      h = (i / a.n_groups) % a.hq;
      b = i / (a.n_groups * a.hq);
    }
  }
  const int kvh = h / a.group;

  const int q_begin = a.cu_q[b];
  const int n_q = a.cu_q[b + 1] - q_begin;
  int len = a.kv_len[b];
  // the selection is defined for a whole prompt: as many queries as cached positions
  if (grp == 0 && h == 0 && tid == 0 && (len < 0 || len > a.capacity || n_q != len)) atomicOr(a.status, (uint32_t)FLUX_DEV_BAD_LENGTH);
  len = len < 0 ? 0 : (len > a.capacity ? a.capacity : len);
  int n = n_q < len ? (n_q < 0 ? 0 : n_q) : len;         // positions 0 .. n-1 are scored
  if (n > 64 * a.tab_cols) {                             // a prompt longer than the host's bound: cut there, and say so
    if (grp == 0 && h == 0 && tid == 0) atomicOr(a.status, (uint32_t)FLUX_DEV_BAD_LENGTH);
    n = 64 * a.tab_cols;
  }
  const int a0 = grp * kXaRows;                          // first square row of the workgroup
  uint8_t* mrow0 = a.mask + (((int64_t)b * a.hq + h) * a.n_qblocks + 8 * grp) * (int64_t)a.n_kblocks;
  const int n_sq = (n + kXaStride - 1) / kXaStride;      // square rows / columns of the prompt
  if (a0 >= n_sq) {                                      // nothing to score: the rows of the matrix are cleared
    for (int qb = 0; qb < 8; ++qb)
      if (8 * grp + qb < a.n_qblocks)
        for (int j = tid; j < a.n_kblocks; j += 256) mrow0[(int64_t)qb * a.n_kblocks + j] = 0;
    return;
  }
  const int a_last = min(a0 + kXaRows, n_sq) - 1;        // last existing square row of the workgroup
  const int n_ct = a_last / 16 + 1;                      // column tiles (16 square columns each) to walk

  // ---- query operand of this wave: lane (nn, g) holds, for half ah and k-step st, 8 numbers of query row
  // 16*(a0 + 16*ah + nn) + r, r = 4w + st / SPR, d = 32 * (st % SPR) + 8g; rows past the prompt are zero
  bf16x8 qf[2][ST];
  {
    const u32x4 zero = {0, 0, 0, 0};
#pragma unroll
    for (int ah = 0; ah < 2; ++ah)
#pragma unroll
      for (int st = 0; st < ST; ++st) {
        const int r = 4 * w + st / SPR, d = 32 * (st % SPR) + 8 * g;
        const int pos = kXaStride * (a0 + 16 * ah + nn) + r;
        const int pc = pos < n ? pos : (n > 0 ? n - 1 : 0);
        const u32x4 t = *(const u32x4*)(a.q + ((int64_t)(q_begin + pc) * a.hq + h) * D + d);
        qf[ah][st] = __builtin_bit_cast(bf16x8, pos < n ? t : zero);
      }
  }
  const __bf16* kbase = a.k + (int64_t)b * a.stride_b + (int64_t)kvh * a.stride_h;

  // One column tile: the key operand of this wave is fetched one tile ahead (the fetch of tile ct + 1 is issued
  // right behind the products of tile ct, into the registers they have just read, so the rest of a tile's work
  // covers its latency); partial sums go to part[buf][w].
  // Keys past the prompt (only the last tile can hold any) are fetched from a clamped address and zeroed when
  // they are used, not when they are fetched: a select behind the load would wait for it at once.
  u32x4 kreg[ST];
  auto key_of = [&](int ct, int st) __attribute__((always_inline)) { return kXaStride * (16 * ct + nn) + (kXaStride - 1) - (4 * w + st / SPR); };
  auto fetch_tile = [&](int ct) __attribute__((always_inline)) {
#pragma unroll
    for (int st = 0; st < ST; ++st) {
      const int key = key_of(ct, st);                        // key row of square column 16*ct + nn, inverse order
      const int kc = key < n ? key : (n > 0 ? n - 1 : 0);
      kreg[st] = *(const u32x4*)(kbase + (int64_t)kc * a.stride_t + 32 * (st % SPR) + 8 * g);
    }
  };
  auto partial_tile = [&](int ct, int buf) __attribute__((always_inline)) {
    if (256 * (ct + 1) > n) {                                // uniform: this tile reaches past the prompt
      const u32x4 zero = {0, 0, 0, 0};
#pragma unroll
      for (int st = 0; st < ST; ++st) kreg[st] = key_of(ct, st) < n ? kreg[st] : zero;
    }
    f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int st = 0; st < ST; ++st)
#pragma unroll
      for (int ah = 0; ah < 2; ++ah)
        acc[ah] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kreg[st]), qf[ah][st], acc[ah], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (ct + 1 < n_ct) fetch_tile(ct + 1);
    __builtin_amdgcn_sched_barrier(0);
    // acc[ah][i] = square (a0 + 16*ah + nn, 16*ct + 4g + i): stored as part[a][b]
#pragma unroll
    for (int ah = 0; ah < 2; ++ah) *(f32x4*)(part + ((buf * 4 + w) * 32 + 16 * ah + nn) * 16 + 4 * g) = acc[ah];
  };
  // the reduction phase: thread (ra, rb) of the workgroup owns the squares (a0 + 16*ah + ra, 16*ct + rb), ah = 0, 1
  const int ra = tid >> 4, rb = tid & 15;
  auto square_value = [&](int ct, int buf, int ah) __attribute__((always_inline)) -> float {
    const int a_abs = a0 + 16 * ah + ra;
    const int b_abs = 16 * ct + rb;
    if (a_abs > a_last || b_abs > a_abs) return -INFINITY;               // no such square
    const int r_min = max(max(b_abs == a_abs ? 8 : 0, kXaStride * b_abs + kXaStride - n), 0);
    const int r_max = min(kXaStride - 1, n - 1 - kXaStride * a_abs);
    const int cnt = r_max - r_min + 1;
    if (cnt <= 0) return -INFINITY;
    const float* p = part + (buf * 4 * 32 + 16 * ah + ra) * 16 + rb;
    // on the diagonal the samples r < 8 (waves 0 and 1) are not causal
    const float lo = b_abs == a_abs ? 0.f : p[0] + p[512];
    const float sum = lo + (p[1024] + p[1536]);
    return a.scale * sum / (float)cnt;
  };

  // ---- first walk: maximum and sum of every row of squares (the 16 lanes rb = 0..15 of a row agree on both)
  float m_row[2] = {-INFINITY, -INFINITY}, l_row[2] = {0.f, 0.f};
  auto first_walk = [&](int ct) __attribute__((always_inline)) {
    const int buf = ct & 1;
    partial_tile(ct, buf);
    __syncthreads();
#pragma unroll
    for (int ah = 0; ah < 2; ++ah) {
      const float e = square_value(ct, buf, ah);
      float mt = e;
      mt = fmaxf(mt, __shfl_xor(mt, 1));
      mt = fmaxf(mt, __shfl_xor(mt, 2));
      mt = fmaxf(mt, __shfl_xor(mt, 4));
      mt = fmaxf(mt, __shfl_xor(mt, 8));
      const float m_new = fmaxf(m_row[ah], mt);
      float pe = e == -INFINITY ? 0.f : __expf(e - m_new);
      pe += __shfl_xor(pe, 1);
      pe += __shfl_xor(pe, 2);
      if (single && (rb & 3) == 0) {                                    // the 4 squares of one key block, reference-free
        const int kbk = 4 * ct + (rb >> 2);
        if (kbk < a.tab_cols) mass[(16 * ah + ra) * a.tab_cols + kbk] = pe > 0.f ? m_new + __logf(pe) : -INFINITY;
      }
      pe += __shfl_xor(pe, 4);
      pe += __shfl_xor(pe, 8);
      l_row[ah] = (m_row[ah] == -INFINITY ? 0.f : l_row[ah] * __expf(m_row[ah] - m_new)) + pe;
      m_row[ah] = m_new;
    }
  };
  fetch_tile(0);
  for (int ct = 0; ct < n_ct; ++ct) first_walk(ct);
  // ---- second walk: probabilities, summed 4 x 4 into block masses.  Wave wv of this phase holds the square rows
  // 16*ah + 4wv .. + 3 (query block 8*grp + 4*ah + wv); a key block is 4 adjacent square columns.
  int rows_in_block[2];                                               // rows of e this wave's query blocks have
#pragma unroll
  for (int ah = 0; ah < 2; ++ah) rows_in_block[ah] = min(4, n_sq - (a0 + 16 * ah + 4 * w));
  auto second_walk = [&](int ct) __attribute__((always_inline)) {
    const int buf = ct & 1;
    partial_tile(ct, buf);
    __syncthreads();
#pragma unroll
    for (int ah = 0; ah < 2; ++ah) {
      const float e = square_value(ct, buf, ah);
      float p = (e == -INFINITY || l_row[ah] == 0.f) ? 0.f : __expf(e - m_row[ah]) / l_row[ah];
      p += __shfl_xor(p, 1);                                          // over the 4 square columns of a key block
      p += __shfl_xor(p, 2);
      p += __shfl_xor(p, 16);                                         // over the 4 square rows of the query block
      p += __shfl_xor(p, 32);
      if ((l & 0x33) == 0 && rows_in_block[ah] > 0) {
        const int kbk = 4 * ct + (rb >> 2);
        if (kbk < a.tab_cols) mass[(4 * ah + w) * a.tab_cols + kbk] = p / (float)rows_in_block[ah];
      }
    }
  };
  __syncthreads();                                                    // the first walk's last readers are done
  if (!single) {
    fetch_tile(0);
    for (int ct = 0; ct < n_ct; ++ct) second_walk(ct);
  } else if (rb == 0) {
#pragma unroll
    for (int ah = 0; ah < 2; ++ah) lse[16 * ah + ra] = m_row[ah] + __logf(l_row[ah]);
  }
  __syncthreads();

  // ---- selection: wave w owns the query blocks 8*grp + w and 8*grp + 4 + w and their masses of key blocks 0 .. own
  const int n_blk = (n + 63) / 64;
  auto wave_sum = [&](float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
  };
  for (int ah = 0; ah < 2; ++ah) {
    const int qi = 4 * ah + w;
    const int qb_abs = 8 * grp + qi;
    if (qb_abs >= a.n_qblocks) continue;
    uint8_t* mrow = mrow0 + (int64_t)qi * a.n_kblocks;
    if (qb_abs >= n_blk) {                                            // a row of the matrix beyond the prompt
      for (int j = l; j < a.n_kblocks; j += 64) mrow[j] = 0;
      continue;
    }
    const int nj = min(qb_abs + 1, a.tab_cols);
    float* mq = mass + (single ? 4 * qi : qi) * a.tab_cols;
    if (single) {
      // masses of this query block from the table, written over its first row (this wave alone touches these rows)
      const int rows = min(4, n_sq - (a0 + 4 * qi));
      for (int j = l; j < nj; j += 64) {
        float acc = 0.f;
        for (int r = 0; r < rows; ++r) acc += __expf(mq[r * a.tab_cols + j] - lse[4 * qi + r]);
        mq[j] = acc / (float)rows;
      }
    }
    float tot = 0.f, mx = 0.f;
    for (int j = l; j < nj; j += 64) {
      tot += mq[j];
      mx = fmaxf(mx, mq[j]);
    }
    tot = wave_sum(tot);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    const float need = a.threshold * tot;
    // largest t (as a bit pattern; positive floats order like their bits) with sum(mass >= t) >= need
    uint32_t lo = 0, hi = __builtin_bit_cast(uint32_t, mx) + 1;       // feasible at lo, not at hi (or hi is past the maximum)
    while (hi - lo > 1) {
      const uint32_t mid = lo + (hi - lo) / 2;
      const float t = __builtin_bit_cast(float, mid);
      float sm = 0.f;
      for (int j = l; j < nj; j += 64) sm += mq[j] >= t ? mq[j] : 0.f;
      sm = wave_sum(sm);
      if (sm >= need) lo = mid; else hi = mid;
    }
    const float cut = __builtin_bit_cast(float, lo);
    for (int j = l; j < a.n_kblocks; j += 64) mrow[j] = (j < nj && (mq[j] >= cut || j == qb_abs)) ? 1 : 0;
  }
}

hipError_t launch_xa_select(const Ctx& c, const flux_attn_cfg& cfg, const void* q, const int32_t* cu_q, int max_q_len,
                            const flux_kv_cache& cache, float threshold, uint8_t* mask, int n_qblocks, int n_kblocks,
                            hipStream_t s) {
  XaArgs a;
  a.q = (const __bf16*)q;
  a.cu_q = cu_q;
  a.k = (const __bf16*)cache.k;
  a.stride_b = cache.stride_b;
  a.stride_h = cache.stride_h;
  a.stride_t = cache.stride_t;
  a.kv_len = cache.kv_len;
  a.capacity = cache.capacity;
  a.hq = cfg.n_q_heads;
  a.group = cfg.n_q_heads / cfg.n_kv_heads;
  a.batch = cache.batch;
  a.scale = cfg.softmax_scale != 0.f ? cfg.softmax_scale : 1.0f / sqrtf((float)cfg.head_dim);
  a.threshold = threshold;
  a.mask = mask;
  a.n_qblocks = n_qblocks;
  a.n_kblocks = n_kblocks;
  const int need = (max_q_len + 63) / 64;                 // the prompt is the whole cache: its length is bounded by max_q_len
  a.tab_cols = need < n_kblocks ? (need > 0 ? need : 1) : n_kblocks;
  a.single_walk = a.tab_cols <= kXaSingleWalkMaxKBlocks;
  a.status = c.status;
  const int groups = (n_qblocks + 7) / 8;                 // every row of the matrix is written
  a.n_groups = groups;
  const dim3 grid((unsigned)((long long)groups * cfg.n_q_heads * cache.batch));
  const size_t lds = xa_select_lds_bytes(a.tab_cols);
  if (cfg.head_dim == 128) {
    if (lds > 48 * 1024) {
      const hipError_t e = hipFuncSetAttribute((const void*)xa_select_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(xa_select_kernel<128>, grid, dim3(256), lds, s, a);
  } else {
    if (lds > 48 * 1024) {
      const hipError_t e = hipFuncSetAttribute((const void*)xa_select_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(xa_select_kernel<64>, grid, dim3(256), lds, s, a);
  }
  return hipGetLastError();
}

}  // namespace flux
