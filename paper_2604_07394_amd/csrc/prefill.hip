// flux_attn_prefill: tiled causal GQA attention on bf16 MFMA, Full (Eq. 1) or Sparse (Eq. 2 with the
// sink + window subset of Sec. 4.1 / App. C.3), chosen per sequence by the cached mode byte.
//
// Shape of the computation (one workgroup = 128 query rows of one head, 4 waves x 32 rows = 2 column blocks
// of 16 queries; launches for long prompts use 8 waves per workgroup: the same 128 rows of two heads of a GQA
// group, or 256 rows of one head, see launch_prefill):
//   for each VISITED 64-key block (FA: all blocks up to the diagonal; SA: the sink blocks and the
//   blocks that intersect the tile's window, nothing else: hidden blocks are skipped, not masked)
//     S^T[key][q]  = K[key][:] . Q[q][:]     MFMA 16x16x32 bf16, A = K rows from LDS, B = Q in registers
//     online softmax along keys.  S is kept TRANSPOSED: a query column belongs to the 4 lanes
//     (n, g = 0..3), each holding 4 of a 16-key block's scores in its accumulator registers, so the
//     running reference is a per-lane scalar and the row sum a per-lane partial that is only combined
//     across the 4 lanes at the end.
//     O^T[d][q]   += V^T[d][key] . P^T[key][q]   the accumulator layout of two 16-key blocks of S^T is the
//     B-operand layout of this product for 32 keys (keys taken in the order 4g..4g+3, 16+4g..16+4g+3), so
//     P never moves between lanes; V^T comes from row-major LDS through the transposing LDS read, its
//     keys in the same order.
// The 16x16x32 form is used because it is the one this chip sustains: a loop of nothing but MFMAs on
// random bf16 data reaches 2030-2280 TFLOP/s with it and 1170-1450 with 32x32x16, whatever the number of
// independent accumulators.
// Only blocks that straddle the causal diagonal or a window / sink edge evaluate the element mask.
//
// flux_attn_prefill_blocksparse is the same kernel (template flag BS) with another list of visited blocks: a
// sequence whose mode byte is 0 visits the key blocks that a caller-given keep matrix marks for the query
// blocks of the workgroup's tile (Eq. 2 over an arbitrary set of 64-position blocks, App. C.3: the block is
// the minimum unit of sparsity), found by scanning the matrix 64 key blocks at a time; blocks that no row of
// the tile keeps are never loaded.
#include <type_traits>

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
  int hq, hkv, group, batch;
  int xcd_map;            // 0 plain, 1 pairs-per-XCD, 2 XCDs-per-pair (see the kernel)
  int sink_lim, win_blocks, blk_shift;   // SA geometry (see sa_geom)
  int n_qtiles;
  float scale_log2;
  int out_fp32;
  void* out;
  uint32_t* status;       // sticky device status word
  // block-sparse form only: keep flags [batch, bm_heads, bm_qblocks, bm_kblocks], one byte per (query block, key
  // block) pair of 64 x 64 positions; row 0 is the block that holds the call's first query of that sequence
  const uint8_t* bmask;
  int bm_heads, bm_qblocks, bm_kblocks;
};

constexpr float kWeightGuard = 1073741824.0f;   // 2^30: a block whose weights sum past this moves the softmax reference

// One wave-wide direct global -> LDS transfer: every lane fetches its own 16 bytes, the 64 pieces land
// at lds_base + 16 * lane.  Issued as inline assembly so that the compiler does not serialise later LDS
// reads of the OTHER stage behind it; completion is awaited explicitly with vmcnt(0) before the barrier.
// M0 (the LDS base of the transfer) is written here and declared as clobbered.
__device__ __forceinline__ void dma16(const char* base /*uniform*/, int lane_off, uint32_t lds_base /*uniform*/) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_off), "s"(base), "s"(lds_base) : "memory", "m0");
}

// All transfers of one wave for one whole tile in a single statement (four for K and four for V, or two and two):
// the LDS destination of transfer t is the uniform base plus a compile-time offset, so M0 is produced by one
// scalar add, and nothing is scheduled between the transfers.  A transfer keeps the issuing wave for about 64
// cycles whatever surrounds it (measured: the vector memory port of a SIMD takes one lane's 16 bytes per cycle),
// so their place in the iteration does not matter; they sit right behind the barrier, where the stage is free.
#define FLUX_DMA_ONE(v, p, o) "s_add_u32 m0, %[lds], %[" o "]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[" v "], %[" p "]\n\t"
template <int OFF, int KT>   // OFF: LDS offset of the stage; KT: bytes from the K tile to the V tile of a stage
__device__ __forceinline__ void dma_tile4(const char* kt, const char* vt, const int (&ko)[4], const int (&vo)[4],
                                          uint32_t lds_base) {
  asm volatile(FLUX_DMA_ONE("k0", "kt", "o0") FLUX_DMA_ONE("k1", "kt", "o1") FLUX_DMA_ONE("k2", "kt", "o2")
               FLUX_DMA_ONE("k3", "kt", "o3") FLUX_DMA_ONE("v0", "vt", "o4") FLUX_DMA_ONE("v1", "vt", "o5")
               FLUX_DMA_ONE("v2", "vt", "o6") FLUX_DMA_ONE("v3", "vt", "o7")
               : : [k0] "v"(ko[0]), [k1] "v"(ko[1]), [k2] "v"(ko[2]), [k3] "v"(ko[3]), [v0] "v"(vo[0]), [v1] "v"(vo[1]),
                   [v2] "v"(vo[2]), [v3] "v"(vo[3]), [kt] "s"(kt), [vt] "s"(vt), [lds] "s"(lds_base), [o0] "i"(OFF),
                   [o1] "i"(OFF + 4096), [o2] "i"(OFF + 8192), [o3] "i"(OFF + 12288), [o4] "i"(OFF + KT),
                   [o5] "i"(OFF + KT + 4096), [o6] "i"(OFF + KT + 8192), [o7] "i"(OFF + KT + 12288)
               : "memory", "m0", "scc");
}
template <int OFF, int KT, int STEP = 4096>   // STEP: bytes between the two transfers of a wave (1 KB per wave of the workgroup)
__device__ __forceinline__ void dma_tile2(const char* kt, const char* vt, const int (&ko)[2], const int (&vo)[2],
                                          uint32_t lds_base) {
  asm volatile(FLUX_DMA_ONE("k0", "kt", "o0") FLUX_DMA_ONE("k1", "kt", "o1") FLUX_DMA_ONE("v0", "vt", "o4")
               FLUX_DMA_ONE("v1", "vt", "o5")
               : : [k0] "v"(ko[0]), [k1] "v"(ko[1]), [v0] "v"(vo[0]), [v1] "v"(vo[1]), [kt] "s"(kt), [vt] "s"(vt),
                   [lds] "s"(lds_base), [o0] "i"(OFF), [o1] "i"(OFF + STEP), [o4] "i"(OFF + KT), [o5] "i"(OFF + KT + STEP)
               : "memory", "m0", "scc");
}

template <int D, bool BS, int NW, int HP = 1>   // NW: waves per workgroup, 4 (two workgroups per CU) or 8 (one); HP: heads per workgroup
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void prefill_kernel(PrefillArgs a) {
  constexpr int RW = NW / HP;             // waves per head
  constexpr int BM = 32 * RW;             // query rows per workgroup (of each of its heads)
  constexpr int BN = 64;                  // keys per iteration: two halves of 32, the K dimension of one PV MFMA
  constexpr int KC = D / 32;              // MFMA k-steps over the head dimension (QK^T)
  constexpr int DB = D / 16;              // 16-wide output blocks over the head dimension (PV)
  constexpr int KB = BN / 16;             // 16-key blocks of S^T per iteration
  constexpr int KS = BN / 32;             // 32-key steps of the PV product per iteration
  constexpr int CPR = D / 8;              // 16-byte chunks per row
  constexpr int ROWB = D * 2;             // bytes per K/V row
  // K tile: unpadded rows, the 16-byte chunk index XOR-swizzled by the row (D = 128: row & 15; D = 64, two
  // rows per 64 banks: (row >> 1) & 7).  A wave-wide 16-byte LDS read is served in four passes of 16 lanes,
  // and within lanes 0..31 the passes are {0-3, 12-15, 20-27} and {4-11, 16-19, 28-31} (measured with the
  // bank conflict counter).  With lane (n, g) reading row n, chunk 4*kc + g, a pass holds rows {0-3, 12-15}
  // at one chunk and rows {4-11} at the chunk next to it; both row sets are closed under XOR with 1, 2 and
  // 3, so the swizzled chunks of a pass are a permutation of all 16 and every pass covers 64 distinct banks.
  // (Rows padded by one chunk give two-way conflicts with this mapping, by two chunks none.)
  constexpr int KPITCH = ROWB;
  constexpr int NKI = BN * CPR / 64;         // wave-wide 1 KB transfers per K tile
  constexpr int NVI = BN * CPR / 64;         // wave-wide 1 KB transfers per V tile
  constexpr int KTILE = BN * ROWB;
  constexpr int VTILE = BN * ROWB;        // V tile: unpadded rows, 32-byte units XOR-swizzled by the row
  constexpr int STAGE = KTILE + VTILE;
  constexpr int KPW = NKI / NW;               // K transfers per wave
  constexpr int VPW = NVI / NW;               // V transfers per wave
  constexpr int RPI = 64 / CPR;              // V rows per transfer
  static_assert(BN * CPR % 64 == 0, "V tile must split into whole wave transfers");
  static_assert(NKI % NW == 0 && NVI % NW == 0 && (KPW == 4 || KPW == 2) && VPW == KPW, "every wave issues the same transfers");

  __shared__ __attribute__((aligned(1024))) char smem[2 * STAGE];

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave of the workgroup: its share of the tile transfers
  const int wr = w % RW, hsel = w / RW;                      // its rows within the tile, and which of the workgroup's heads
  const int l = tid & 63;
  const int g = l >> 4, n = l & 15;
  // ---- which (sequence, head, query tile) this workgroup owns.  Workgroups go to the 8 XCDs round-robin
  // by linear id, and each XCD has its own L2.  The workgroups that an XCD holds at one time are therefore
  // given neighbouring query tiles of one (sequence, KV head) pair, heaviest tiles first and the heads of a
  // group next to each other, so that they walk the same K/V rows at the same time and the rows come from
  // HBM once per XCD and round instead of once per workgroup.
  int qt, h, b;
  {
    const int i = blockIdx.x;
    const int n_pairs = a.batch * a.hkv;
    if (a.xcd_map == 1) {                                    // n_pairs a multiple of 8: eight pairs at a time, one per XCD
      const int x = i & 7, j = i >> 3;
      const int gw = a.group / HP;                           // workgroups per (pair, query tile)
      // An XCD takes its pairs one after the other (all tiles of a pair, heaviest first, the heads of a tile next to
      // each other).  Interleaving the pairs tile by tile looks more even, but in a ragged batch the tiles past a
      // short sequence's end are empty workgroups, and at fixed places of a short period they keep falling to the
      // same CUs (consecutive workgroups go round the CUs of an XCD), leaving the others idle: measured 1.5 - 2 x.
      // Two rotations even out work that differs between heads (block-sparse launches whose heads keep different
      // shares), at no cost where it does not: the heads of a tile change places from tile to tile, so that a CU
      // (which sees every 32nd workgroup of its XCD) meets all heads of the group; and the eight pairs of a round
      // change XCD every 16 tiles (one round of resident workgroups), so that every XCD works through two rounds of
      // every pair instead of all rounds of one.  A round streams its K/V rows from behind the L2 anyway.
      const int r = j / (gw * a.n_qtiles), qtd = (j / gw) % a.n_qtiles, g = (j + qtd) % gw;
      const int pair = ((x + qtd / 16) & 7) + 8 * r;
      b = pair / a.hkv;
      h = (pair % a.hkv) * a.group + HP * g + hsel;
      qt = a.n_qtiles - 1 - qtd;
    } else if (a.xcd_map == 2) {                             // n_pairs divides 8: 8 / n_pairs XCDs share a pair
      const int x = i & 7, j = i >> 3, share = 8 / n_pairs;
      const int pair = x % n_pairs, sl = x / n_pairs;
      const int gw = a.group / HP;
      const int g = j % gw, qtd = (j / gw) * share + sl;
      b = pair / a.hkv;
      h = (pair % a.hkv) * a.group + HP * g + hsel;
      qt = a.n_qtiles - 1 - qtd;
      if (qt < 0) return;                                    // padding of the last round (uniform)
    } else {                                                 // any other shape: plain order, heavy tiles first
      qt = a.n_qtiles - 1 - i % a.n_qtiles;
      h = HP * ((i / a.n_qtiles) % (a.hq / HP)) + hsel;
      b = i / (a.n_qtiles * (a.hq / HP));
    }
  }
  const int kvh = h / a.group;

  const int q_begin = a.cu_q[b];
  const int n_q_given = a.cu_q[b + 1] - q_begin;
  int len = a.kv_len[b];
  // lengths the host could not see: negative, past the capacity, or more queries than cached positions;
  // they are clamped below, and reported once per sequence
  if (qt == a.n_qtiles - 1 && h == 0 && tid == 0 && (n_q_given < 0 || len < 0 || len > a.capacity || n_q_given > len))
    atomicOr(a.status, (uint32_t)FLUX_DEV_BAD_LENGTH);
  len = len > a.capacity ? a.capacity : len;
  if (len < 1) return;                                       // nothing cached: nothing to attend
  // the queries are the last n_q cached positions, so there cannot be more of them than positions: the
  // surplus rows of an inconsistent call are not computed (every key tile then starts inside the cache)
  const int n_q = n_q_given < len ? n_q_given : len;
  if (qt * BM >= n_q) return;                                // uniform for the workgroup
  const int pos0 = max(len - n_q, 0);                        // position of query row 0
  const bool sa = a.mode[b] == 0;

  // query rows of the tile / of this wave, as absolute positions
  const int r_tile_last = min(qt * BM + BM - 1, n_q - 1);
  const int i_tile_min = pos0 + qt * BM;
  const int i_tile_max = pos0 + r_tile_last;
  const int r_w0 = qt * BM + 32 * wr;
  const int i_w_min = pos0 + r_w0;
  const int i_w_max = pos0 + min(r_w0 + 31, n_q - 1);       // < i_w_min if the wave has no valid row
  const bool wave_active = r_w0 < n_q;
  // this lane's two query rows (column n of column block qb): clamped row, unclamped position, and the
  // first key of the row's SA window
  int r_mine[2], i_mine[2], w_lo_mine[2];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    r_mine[qb] = min(r_w0 + 16 * qb + n, n_q - 1);
    i_mine[qb] = pos0 + r_w0 + 16 * qb + n;
    w_lo_mine[qb] = window_start(i_mine[qb], a.blk_shift, a.win_blocks);
  }
  // first key of the SA window of the wave's first row and of its last row
  const int w_lo_first = window_start(i_w_min, a.blk_shift, a.win_blocks);
  const int w_lo_last = window_start(max(i_w_max, i_w_min), a.blk_shift, a.win_blocks);

  // ---- Q operand: lane (n, g) holds d = 32*kc + 8*g .. +7 of its two query rows
  bf16x8 qf[2][KC];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const __bf16* qrow = a.q + ((int64_t)(q_begin + r_mine[qb]) * a.hq + h) * D;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) qf[qb][kc] = *(const bf16x8*)(qrow + 32 * kc + 8 * g);
  }

  // ---- visited key blocks: [0, n_a) and [win0, win0 + n_b)
  const int last_blk = i_tile_max / BN;
  int n_a, win0, n_b;
  if (!sa) {
    n_a = last_blk + 1; win0 = 0; n_b = 0;
  } else {
    const int sink_end = min(a.sink_lim, i_tile_max + 1);    // keys [0, sink_end) are sinks in reach
    n_a = (sink_end + BN - 1) / BN;
    const int wfirst = window_start(i_tile_min, a.blk_shift, a.win_blocks);   // first key any row's window reaches
    win0 = max(wfirst / BN, n_a);
    n_b = last_blk + 1 - win0;
    if (n_b < 0) n_b = 0;
  }
  const int n_iter = n_a + n_b;

  const char* kbase = (const char*)(a.k + (int64_t)b * a.stride_b + (int64_t)kvh * a.stride_h);
  const char* vbase = (const char*)(a.v + (int64_t)b * a.stride_b + (int64_t)kvh * a.stride_h);
  const int pitch_g = (int)a.stride_t * 2;                   // bytes between rows in the cache

  // ---- direct global -> LDS transfers.  One transfer moves 64 x 16 bytes to 1 KB of consecutive LDS;
  // which (row, chunk) a lane fetches decides where that chunk lands.  Per lane, the row and chunk of
  // each of this wave's transfers are fixed for the whole kernel.
  // Transfer I covers rows I*RPI .. +RPI-1 of a tile; lane l sits at (row l/CPR, physical chunk l%CPR) and
  // fetches the logical chunk that the swizzle maps there.  Wave w issues the transfers w, w + NW, ...  For K the
  // swizzle of row (w + NW*t)*RPI + l/CPR is (4w + l/16) & (CPR-1) for both head sizes, a per-lane constant.
  const int v_lrow = l / CPR;
  const int k_chunk = (l % CPR) ^ ((4 * w + (l >> 4)) & (CPR - 1));
  auto k_slot = [&](int t, int rmax) { return min((w + NW * t) * RPI + v_lrow, rmax) * pitch_g + k_chunk * 16; };
  // the 32-byte units of a V row are XOR-swizzled by the row (D = 128: row & 7; D = 64, two rows per 64
  // banks: (row >> 1) & 3), which makes the transposing reads below conflict-free; the row of transfer
  // w + NW*t, lane l is (w + NW*t) * RPI + l / CPR, so the swizzle is a per-lane constant
  const int v_swz = D == 128 ? ((4 * (w & 1) + v_lrow) << 1) : (((v_lrow >> 1) & 3) << 1);
  const int v_chunk = (l % CPR) ^ v_swz;
  auto v_slot = [&](int t, int rmax) { return min((w + NW * t) * RPI + v_lrow, rmax) * pitch_g + v_chunk * 16; };
  int k_off[KPW], v_off[VPW];                                // byte offsets inside a tile that is fully cached
#pragma unroll
  for (int t = 0; t < KPW; ++t) k_off[t] = k_slot(t, BN);
#pragma unroll
  for (int t = 0; t < VPW; ++t) v_off[t] = v_slot(t, BN);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(FLUX_LDS char*)smem;

  const uint32_t lds_w = lds0 + 1024 * w;                    // this wave's 1 KB slot inside every NW KB of a stage

  // tile index (in units of BN keys) of iteration `it`: the blocks [0, n_a) first, then [win0, win0 + n_b)
  auto tile_of = [&](int it) { return it < n_a ? it : win0 + (it - n_a); };

  // All transfers of one tile with rows clamped to the cached length: the first tile, and a last tile that
  // is only partly inside the cache.
  auto issue_tile_clamped = [&](int tile, int stage) {
    const int j0 = tile * BN;
    const int rmax = len - 1 - j0;                           // rows past the cached length are clamped
    const char* kt = kbase + (int64_t)j0 * pitch_g;
    const char* vt = vbase + (int64_t)j0 * pitch_g;
    const uint32_t lk = lds_w + stage * STAGE;
#pragma unroll
    for (int t = 0; t < KPW; ++t)
      dma16(kt, k_slot(t, rmax), lk + 1024 * NW * t);
#pragma unroll
    for (int t = 0; t < VPW; ++t)
      dma16(vt, v_slot(t, rmax), lk + KTILE + 1024 * NW * t);
  };

  // ---- per-lane LDS read offsets (bytes, relative to stage 0; the stage is added as an immediate)
  // K fragment (kb, kc): row 16*kb + n, logical chunk 4*kc + g (d = 32*kc + 8*g ..), swizzled by the row
  const int k_xr = D == 128 ? n : (n >> 1);
  int k_rd[KC];
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) k_rd[kc] = n * KPITCH + (((4 * kc + g) ^ k_xr) * 16);
  // V^T fragment for output block db: the transposing read of lane (n, g) addresses row 4*g + n/4, columns
  // 16*db + 4*(n%4) .. +3, and returns V^T[16*db + n][keys 4g .. 4g+3] of the 16-row group
  const int v_row = 4 * g + (n >> 2);
  const int v_xr = D == 128 ? (v_row & 7) : ((v_row >> 1) & 3);
  int v_rd[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) v_rd[db] = KTILE + v_row * ROWB + ((db ^ v_xr) * 32) + (n & 3) * 8;

  float m_ref[2] = {-INFINITY, -INFINITY};                   // the score the exponents of a row refer to
  float mneg[2] = {0.f, 0.f};                                // -m_ref * scale_log2 (0 while a row has no reference yet)
  float l_run[2] = {0.f, 0.f};                               // this lane's part of the row sums
  bool all_ref = false;                                      // wave-uniform: every row of the wave has a reference
  f32x4 o[DB][2];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) o[i][qb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ---- which iterations are PLAIN for this wave: the wave is active, every key of the block is visible to
  // every row of the wave (no element mask, nothing to skip).  In tile indices: the block ends at or before the
  // wave's first row (tile < c_end), and for SA it lies wholly inside the sinks (tile < s_full) or starts at
  // or after the window start of the wave's LAST row (tile >= w_first_full).  As iteration ranges:
  // [0, pa_end) and [pb_begin, pb_end).  A wave issues its instructions in order and two waves share a SIMD, so
  // every instruction of the loop shows in its time: the plain iterations (all but a few per workgroup) skip the
  // mask flags and the block's first key altogether.
  int pa_end = 0, pb_begin = 0, pb_end = 0;
  if (wave_active) {
    const int c_end = (i_w_min + 1) / BN;
    if (!sa) {
      pa_end = min(n_a, c_end);
    } else {
      pa_end = min(min(n_a, c_end), a.sink_lim / BN);
      const int w_first_full = (w_lo_last + BN - 1) / BN;
      pb_begin = n_a + max(w_first_full - win0, 0);
      pb_end = min(n_a + max(c_end - win0, 0), n_iter);
    }
  }
  // the last tile may be only partly inside the cache; every other tile is whole
  const bool last_whole = n_iter > 0 && len - 1 - tile_of(n_iter - 1) * BN >= BN - 1;
  const int lim_whole = last_whole ? n_iter : n_iter - 1;    // iterations it + 1 < lim_whole transfer a whole tile
  const unsigned pb_len = pb_end > pb_begin ? pb_end - pb_begin : 0;
  const int64_t step_b = (int64_t)BN * pitch_g;              // bytes from one key block to the next
  const int64_t jump_b = (int64_t)(win0 - n_a + 1) * step_b; // from the last sink block to the first window block
  const char* kt_n = kbase + (int64_t)(n_iter > 1 ? tile_of(1) : 0) * step_b;   // the tile the next transfer brings in
  const char* vt_n = vbase + (int64_t)(n_iter > 1 ? tile_of(1) : 0) * step_b;

  // ---- block-sparse form: the visited key blocks come from the keep matrix.  The tile's 128 rows lie in up
  // to three 64-position query blocks (two when the first query sits on a block boundary); a key block is
  // visited when any of them keeps it.  The matrix is scanned 64 key blocks at a time: lane l of every wave reads
  // the flag of key block win + l for each of the tile's query blocks, a ballot turns them into one 64-bit word
  // per query block, and the blocks are taken from the lowest set bit up.  Every wave runs the same scan (all of
  // it in scalar registers), so no exchange is needed.  A query block always keeps its own (diagonal) block, and
  // never a later one; an FA sequence (mode byte 1) keeps everything.
  const int rb0 = i_tile_min >> 6;                           // absolute index of the tile's first query block
  const int n_rb = (i_tile_max >> 6) - rb0 + 1;              // 1 .. 3
  int scan_win = -64;                                        // first key block of the 64 being scanned
  unsigned long long scan_bits[3] = {0, 0, 0};               // what is left of them, per query block of the tile
  int cur_kb = -1, cur_rows = 0;                             // the block of this iteration, and which query blocks keep it
  const uint8_t* bm_seq = nullptr;
  if constexpr (BS) {
    if (sa) bm_seq = a.bmask + ((int64_t)b * a.bm_heads + (a.bm_heads > 1 ? h : 0)) * a.bm_qblocks * (int64_t)a.bm_kblocks;
  }
  auto next_kept_block = [&](int& rows) -> int {
    for (;;) {
      const unsigned long long any = scan_bits[0] | scan_bits[1] | scan_bits[2];
      if (any != 0) {
        const int bit = __builtin_ctzll(any);
        rows = (int)((scan_bits[0] >> bit) & 1) | (int)(((scan_bits[1] >> bit) & 1) << 1) | (int)(((scan_bits[2] >> bit) & 1) << 2);
        const unsigned long long clr = ~(1ull << bit);
        scan_bits[0] &= clr;
        scan_bits[1] &= clr;
        scan_bits[2] &= clr;
        return scan_win + bit;
      }
      scan_win += 64;
      if (scan_win > last_blk) return -1;
      const int kbk = scan_win + l;
#pragma unroll
      for (int r = 0; r < 3; ++r) {
        const int rb = rb0 + r;                              // absolute query block
        bool keep = r < n_rb && kbk <= rb;                   // never a later block (causal), nothing for absent rows
        if (keep && kbk < rb && bm_seq != nullptr) {         // the diagonal block is kept whatever the flag says
          const int rq = rb - (pos0 >> 6);
          // a matrix too small for the lengths found on the device hides what it does not cover, and says so
          const bool inside = rq < a.bm_qblocks && kbk < a.bm_kblocks;
          if (!inside && w == 0 && h == 0) atomicOr(a.status, (uint32_t)FLUX_DEV_BAD_LENGTH);
          keep = inside && bm_seq[(int64_t)rq * a.bm_kblocks + kbk] != 0;
        }
        scan_bits[r] = __builtin_amdgcn_ballot_w64(keep);
      }
    }
  };
  int nxt_kb = -1, nxt_rows = 0;

  // One iteration.  STG (the LDS stage of this tile) is a compile-time constant: the loop is unrolled by two so
  // that every LDS address is a loop-invariant register plus an immediate.
  auto iteration = [&](int it, auto stg_c) {
    constexpr int STG = decltype(stg_c)::value;
    __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0): this wave's transfers have landed
    __syncthreads();                                         // ... and everyone's; the other stage is free
    if constexpr (BS) {
      nxt_kb = next_kept_block(nxt_rows);
      if (nxt_kb >= 0) {                                     // the next kept block, in flight during the math below
        if ((nxt_kb + 1) * BN <= len) {
          const int64_t off = (int64_t)nxt_kb * step_b;
          if constexpr (KPW == 4) dma_tile4<(STG ^ 1) * STAGE, KTILE>(kbase + off, vbase + off, k_off, v_off, lds_w);
          else dma_tile2<(STG ^ 1) * STAGE, KTILE, 1024 * NW>(kbase + off, vbase + off, k_off, v_off, lds_w);
        } else {
          issue_tile_clamped(nxt_kb, STG ^ 1);
        }
      }
    } else if (it + 1 < lim_whole) {                         // the next tile, in flight during the math below
      if constexpr (KPW == 4) dma_tile4<(STG ^ 1) * STAGE, KTILE>(kt_n, vt_n, k_off, v_off, lds_w);
      else dma_tile2<(STG ^ 1) * STAGE, KTILE, 1024 * NW>(kt_n, vt_n, k_off, v_off, lds_w);
      const int64_t adv = it + 2 == n_a ? jump_b : step_b;   // on to the tile after it (the window part starts at win0)
      kt_n += adv;
      vt_n += adv;
    } else if (it + 1 < n_iter) {
      issue_tile_clamped(tile_of(it + 1), STG ^ 1);          // a last tile that is only partly inside the cache
    }
    bool plain = it < pa_end || (unsigned)(it - pb_begin) < pb_len;
    // block-sparse form: this block (cur_kb) as the wave's rows see it.  The wave's 32 rows lie in one or two of
    // the tile's query blocks; the block is plain when both keep it and it ends at or before the wave's first row.
    const int bs_j0 = cur_kb * BN, bs_rows = cur_rows;
    if constexpr (BS) {
      const int r_lo = (i_w_min >> 6) - rb0, r_hi = (max(i_w_max, i_w_min) >> 6) - rb0;
      const bool k_lo = (bs_rows >> r_lo) & 1, k_hi = (bs_rows >> r_hi) & 1;
      plain = wave_active && k_lo && k_hi && bs_j0 + BN - 1 <= i_w_min;
      cur_kb = nxt_kb;                                       // the state moves on; this iteration keeps bs_j0 / bs_rows
      cur_rows = nxt_rows;
      if (!plain && (!wave_active || bs_j0 > i_w_max || !(k_lo || k_hi))) return;   // nothing for this wave here
    }

    FLUX_LDS char* st = (FLUX_LDS char*)smem + STG * STAGE;
    // Order of the block, written out so that every LDS read is issued well before its use (the fences keep
    // the compiler from moving the reads):
    //   K fragments of half 0 | S^T half 0, the K fragments of half 1 read between its MFMAs |
    //   S^T half 1, the V fragments of half 0 read between its MFMAs | weights |
    //   O^T += half 0, the V fragments of half 1 read between its MFMAs | O^T += half 1
    f32x4 s[KB][2];              // s[kb][qb][i]: key j0 + 16*kb + 4*g + i against query row (qb, n)
    bf16x8 pf[2][KS];            // pf[qb][ks]: weights of keys 32*ks + {4g..4g+3, 16+4g..16+4g+3}, as a B operand
    bf16x8 kf[KB][KC];
    bf16x8 vf[KS][DB];
    auto read_k = [&](int kb, int kc) { kf[kb][kc] = *(FLUX_LDS bf16x8*)(st + k_rd[kc] + 16 * kb * KPITCH); };
    auto read_v = [&](int ks, int db) {
      FLUX_LDS char* vp = st + v_rd[db] + 32 * ks * ROWB;
      const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((FLUX_LDS bf16x4*)vp);
      const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((FLUX_LDS bf16x4*)(vp + 16 * ROWB));
      vf[ks][db] = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    // Softmax weights against the reference m_ref the accumulators already refer to, WITHOUT looking for the
    // block's maximum first: any reference gives the same quotient, and fp32 / bf16 keep their relative
    // precision over the whole exponent range.  A row without a reference yet uses 0.
    float l_blk[2];
    auto weights = [&]() {
      const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        l_blk[qb] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          uint32_t pk[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const f32x4& sv = s[2 * ks + (t >> 1)][qb];
            const float p0 = fast_exp2(__builtin_fmaf(sv[2 * (t & 1)], a.scale_log2, mneg[qb]));
            const float p1 = fast_exp2(__builtin_fmaf(sv[2 * (t & 1) + 1], a.scale_log2, mneg[qb]));
            pk[t] = pack_bf16(p0, p1);
            // the denominator sums the same rounded weights the numerator uses
            l_blk[qb] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk[t]), ones, l_blk[qb], false);
          }
          pf[qb][ks] = __builtin_bit_cast(bf16x8, u32x4{pk[0], pk[1], pk[2], pk[3]});
        }
      }
    };
    auto accumulate = [&](int ks) {        // o[db][qb][i] is d = 16*db + 4*g + i of query row (qb, n)
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
          o[db][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[ks][db], pf[qb][ks], o[db][qb], 0, 0, 0);
    };
    // Only when a row has no reference yet, or some weight of the block left the guarded range (or
    // overflowed), does the wave take the block's maximum, move the reference there (rescaling l and O) and
    // redo the weights.  In the steady state the maximum, its cross-lane steps and the rescale are not executed.
    auto weights_guarded = [&]() {
      weights();
      // (one ballot per comparison: each is then the comparison's own lane mask, with no vector instruction between)
      if (!all_ref || (__builtin_amdgcn_ballot_w64(!(l_blk[0] < kWeightGuard)) | __builtin_amdgcn_ballot_w64(!(l_blk[1] < kWeightGuard))) != 0) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          float mloc = s[0][qb][0];
#pragma unroll
          for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int i = 0; i < 4; ++i) mloc = fmaxf(mloc, s[kb][qb][i]);
          mloc = fmaxf(mloc, __shfl_xor(mloc, 16));                              // over the 4 lanes of the row
          mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
          const float m_new = fmaxf(m_ref[qb], mloc);
          if (m_new > m_ref[qb]) {                                               // false while both are -inf
            const float al = fast_exp2((m_ref[qb] - m_new) * a.scale_log2);      // 0 for a row's first reference
            l_run[qb] *= al;
#pragma unroll
            for (int db = 0; db < DB; ++db) o[db][qb] *= al;
            m_ref[qb] = m_new;
            mneg[qb] = -m_new * a.scale_log2;
          }
        }
        weights();
        all_ref = __builtin_amdgcn_ballot_w64((m_ref[0] == -INFINITY) | (m_ref[1] == -INFINITY)) == 0;
      }
      l_run[0] += l_blk[0];
      l_run[1] += l_blk[1];
    };

    // a block that an edge of the visible set crosses, or that this wave does not see at all, needs the
    // block's first key and the mask flags; a plain block needs none of that scalar work
    int j0 = 0;
    bool mask_causal = false, mask_edge = false;
    if constexpr (BS) {
      j0 = bs_j0;
      mask_causal = !plain;
    } else if (!plain) {
      j0 = tile_of(it) * BN;
      bool skip = !wave_active || j0 > i_w_max;
      mask_causal = j0 + BN - 1 > i_w_min;                   // the diagonal crosses the block
      if (sa) {
        const bool all_sink = j0 + BN <= a.sink_lim;
        if (!all_sink) {
          if (j0 >= a.sink_lim && j0 + BN - 1 < w_lo_first) skip = true;          // before every window
          mask_edge = j0 < w_lo_last;                        // a window or sink edge falls inside the block
        }
      }
      if (skip) return;
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) read_k(kb, kc);
    __builtin_amdgcn_sched_barrier(0);
    // S^T of keys 0..31 with the K fragments of keys 32..63 read between the MFMAs, then S^T of keys 32..63 with the V
    // fragments of keys 0..31 read between them: a read between two MFMAs costs the wave a few cycles, in a run of
    // reads sixteen, and every fragment is asked for at least sixteen MFMAs before its use.  The accumulators start
    // from what the caller put into s.
    auto scores = [&]() {
#pragma unroll
      for (int t = 0; t < 2 * KC; ++t) {
        const int kc = t >> 1, kb = t & 1;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) s[kb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kb][kc], qf[qb][kc], s[kb][qb], 0, 0, 0);
        read_k(2 + kb, kc);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int t = 0; t < 2 * KC; ++t) {
        const int kc = t >> 1, kb = 2 + (t & 1);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) s[kb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kb][kc], qf[qb][kc], s[kb][qb], 0, 0, 0);
#pragma unroll
        for (int db = t * DB / (2 * KC); db < (t + 1) * DB / (2 * KC); ++db) read_v(0, db);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // Element masks are put into the accumulators the scores start from: 0 for a visible pair, -inf for a hidden one
    // (the sum of the products then stays -inf), so a plain block starts from the constant 0 and the scores of either
    // kind of block come out of the MFMAs in the same registers.  (With the masks applied to the finished scores the
    // compiler keeps masked and unmasked scores in different registers and copies all 32 of them in every plain
    // block.)  Key j = j0 + 4*g + c with the constant c = 16*kb + i, so each bound is moved into the lane once
    // (bound - j0 - 4*g) and compared with constants.
    if (mask_edge) {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const int hi = i_mine[qb] - j0 - 4 * g, lo = w_lo_mine[qb] - j0 - 4 * g, sl = a.sink_lim - j0 - 4 * g;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int c = 16 * kb + i;
            const bool vis = (c <= hi) & ((c < sl) | (c >= lo));
            s[kb][qb][i] = vis ? 0.f : -INFINITY;
          }
      }
      scores();
    } else if (mask_causal) {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        int hi = i_mine[qb] - j0 - 4 * g;
        // block-sparse form: a row whose query block does not keep this key block sees none of it
        if constexpr (BS) hi = ((bs_rows >> ((i_mine[qb] >> 6) - rb0)) & 1) ? hi : -1;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int i = 0; i < 4; ++i) s[kb][qb][i] = 16 * kb + i <= hi ? 0.f : -INFINITY;
      }
      scores();
    } else {
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) s[kb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
      scores();
    }
    // The softmax part runs at a raised wave priority: while it is short, the other wave of this SIMD is mostly
    // inside a run of MFMAs, which queue on the matrix pipe anyway, so letting the vector work through first
    // shortens this wave's way back to its own MFMAs (measured: +2.7 % on the FA launch).
    __builtin_amdgcn_s_setprio(1);
    weights_guarded();
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    // O^T += keys 0..31 with the V fragments of keys 32..63 read between the MFMAs
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) o[db][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[0][db], pf[qb][0], o[db][qb], 0, 0, 0);
      read_v(1, db);
      __builtin_amdgcn_sched_barrier(0);
    }
    accumulate(1);
  };

  if constexpr (!BS) {
    if (n_iter > 0) issue_tile_clamped(tile_of(0), 0);
    for (int it = 0; it < n_iter; it += 2) {
      iteration(it, std::integral_constant<int, 0>());
      if (it + 1 < n_iter) iteration(it + 1, std::integral_constant<int, 1>());
    }
  } else {
    cur_kb = next_kept_block(cur_rows);
    if (cur_kb >= 0) issue_tile_clamped(cur_kb, 0);
    while (cur_kb >= 0) {
      iteration(0, std::integral_constant<int, 0>());
      if (cur_kb < 0) break;
      iteration(0, std::integral_constant<int, 1>());
    }
  }

  // ---- normalise and store: lane (n, g) holds d = 16*db + 4*g .. +3 of its two query rows
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    float l_tot = l_run[qb];
    l_tot += __shfl_xor(l_tot, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (r_w0 + 16 * qb + n < n_q) {
      const float inv = 1.0f / l_tot;
      const int64_t off = ((int64_t)(q_begin + r_w0 + 16 * qb + n) * a.hq + h) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const int d = 16 * db + 4 * g;
        const float x0 = o[db][qb][0] * inv, x1 = o[db][qb][1] * inv;
        const float x2 = o[db][qb][2] * inv, x3 = o[db][qb][3] * inv;
        if (a.out_fp32) {
          *(f32x4*)((float*)a.out + off + d) = f32x4{x0, x1, x2, x3};
        } else {
          *(u32x2*)((__bf16*)a.out + off + d) = u32x2{pack_bf16(x0, x1), pack_bf16(x2, x3)};
        }
      }
    }
  }
}

hipError_t launch_prefill(const Ctx& c, const flux_attn_cfg& cfg, const void* q, const int32_t* cu_q,
                          int max_q_len, int max_kv_len, const flux_kv_cache& cache, const uint8_t* mode,
                          const BlockMask* bm, void* out, hipStream_t s) {
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
  a.hkv = cfg.n_kv_heads;
  a.group = cfg.n_q_heads / cfg.n_kv_heads;
  a.batch = cache.batch;
  const SaGeom geom = sa_geom(cfg);
  a.sink_lim = geom.sink_lim;
  a.win_blocks = geom.win_blocks;
  a.blk_shift = geom.shift;
  // Long prompts at head dimension 128 run with eight waves per workgroup (one workgroup per CU) that share every K/V
  // tile, so that each wave issues half the tile transfers per block: waves 0-3 and 4-7 take the same 128 query rows of
  // two heads of a GQA group (an even group size), else 256 rows of one head.  Measured against the four-wave shape
  // with 256 rows: FA launches gain 1-3 % from 16384 tokens up; SA launches lose 4 % at 16384 tokens (more of a 256-row
  // tile's blocks are cut by the window's start and by the diagonal), under 1 % at 32768 and nothing at 65536; short
  // prompts lose 4-25 % (fewer, longer workgroups).  Two heads on the same rows have one diagonal and one window
  // start: another 0.2 % on FA and 1 % on SA from 32768 tokens up.  Hence the bound on the longest prompt of the
  // launch, which is all the host knows.  The results are the same bit for bit.  The block-sparse form keeps four
  // waves (its scan handles three query blocks per tile).
  // A chunk of half that length of a prompt that long (chunked prefill: every workgroup walks many blocks) gains too:
  // FA +1-2 %, SA +0-1.5 % for 16384-row chunks behind 16384 to 114688 cached positions.
  const bool wide = !bm && cfg.head_dim == 128 &&
                    (max_q_len >= kPrefillWideMinRows || (max_q_len >= kPrefillWideMinRows / 2 && max_kv_len >= kPrefillWideMinRows));
  const int HP = wide && a.group % 2 == 0 ? 2 : 1;          // two heads of a group share the workgroup's K/V tiles
  const int BM = wide && HP == 1 ? 256 : 128;
  a.n_qtiles = (max_q_len + BM - 1) / BM;
  a.scale_log2 = scale * kLog2e;
  a.out_fp32 = cfg.out_dtype;
  a.out = out;
  a.status = c.status;
  a.bmask = bm ? bm->flags : nullptr;
  a.bm_heads = bm ? bm->heads : 0;
  a.bm_qblocks = bm ? bm->n_qblocks : 0;
  a.bm_kblocks = bm ? bm->n_kblocks : 0;
  if (a.n_qtiles == 0) return hipSuccess;
  const long long n_pairs = (long long)cache.batch * cfg.n_kv_heads;
  long long n_wg;
  if (n_pairs % 8 == 0) {
    a.xcd_map = 1;
    n_wg = (long long)a.n_qtiles * (cfg.n_q_heads / HP) * cache.batch;
  } else if (8 % n_pairs == 0) {
    a.xcd_map = 2;
    const long long share = 8 / n_pairs;
    n_wg = 8 * (a.group / HP) * ((a.n_qtiles + share - 1) / share);
  } else {
    a.xcd_map = 0;
    n_wg = (long long)a.n_qtiles * (cfg.n_q_heads / HP) * cache.batch;
  }
  if (n_wg > 0x7FFFFFFFll) return hipErrorInvalidValue;
  const dim3 grid((unsigned)n_wg);
  if (bm) {
    if (cfg.head_dim == 128) hipLaunchKernelGGL((prefill_kernel<128, true, 4>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((prefill_kernel<64, true, 4>), grid, dim3(256), 0, s, a);
  } else {
    if (wide && HP == 2) hipLaunchKernelGGL((prefill_kernel<128, false, 8, 2>), grid, dim3(512), 0, s, a);
    else if (wide) hipLaunchKernelGGL((prefill_kernel<128, false, 8>), grid, dim3(512), 0, s, a);
    else if (cfg.head_dim == 128) hipLaunchKernelGGL((prefill_kernel<128, false, 4>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((prefill_kernel<64, false, 4>), grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace flux
