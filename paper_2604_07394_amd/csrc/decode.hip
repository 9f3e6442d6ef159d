// flux_attn_decode: split-K streaming attention for one query row per sequence (Eq. 1 / Eq. 2 with
// one query; the decode step of Sec. 3.3 / App. B.3).
//
// Decode is bound by reading the K and V rows of the cache once from HBM.  The work of one
// (sequence, KV head) pair is the VISIBLE key list (FA: all positions; SA: the sinks followed by the
// window tail, so the hidden middle of the cache is never addressed), taken in blocks of 128 keys that
// go round the pair's units.  One 256-thread workgroup is one unit and serves all query heads of the GQA
// group at once, so every K/V row is fetched exactly once per step.
//
// The split is taken ON THE DEVICE from the lengths and mode bytes the call finds there: the chunk
// size (the keys one unit takes) is the one that cuts the visible keys of the whole batch into about
// kTargetUnits workgroups, a pair of nv visible keys gets ceil(nv / chunk) units, and workgroup u finds
// its (sequence, KV head, unit of the pair) by a prefix sum over the batch.  Every
// workgroup with work therefore sits at the front of the grid whatever the mix of lengths and
// modes in the batch, and a ragged batch fills the chip like a uniform one (a grid shaped by the
// longest sequence leaves most workgroups of the short ones empty and the rest badly spread).
//
// Per wave, 32 keys at a time:
//   S^T[key][q]  = K[key][:] . Q[q][:]       4 (D=128) MFMA 16x16x32 bf16 per 16 keys; the A operand
//                                            (8 consecutive d of one key row per lane) is loaded
//                                            straight from global memory, 64 contiguous bytes per row
//                                            and instruction
//   online softmax in the MFMA accumulator layout (one query per lane column, 4 keys per lane)
//   O^T[d][q]   += V^T[d][key] . P^T[key][q] the P operand is the accumulator layout itself; the
//                                            V operand needs keys along the lane's registers, so V
//                                            rows are staged in wave-private LDS and read back with
//                                            the transposing LDS read
// The four waves keep private (m, l, O) and are merged through LDS at the end; the unit's
// unnormalised result goes to the workspace and a second small kernel merges the units of a pair in a fixed
// order (deterministic, no float atomics).
#include "flux_internal.h"

namespace flux {

// What both kernels read to agree on the split.
struct SplitArgs {
  const int32_t* kv_len;
  const uint8_t* mode;
  int batch, capacity;
  int ring;               // != 0: the cache is a sink + ring store of a sparse layer, kv_len is logical, no mode bytes
  int sink_lim, win_blocks, blk_shift;   // SA geometry (see sa_geom)
  int max_keys;           // the host's bound on the keys any sequence attends to
  int pps;                // (KV head, query block) pairs per sequence = hkv * qblocks
  int bump;               // 1: the call also appends one row per sequence, so every list is one key longer than kv_len says
};

struct DecodeArgs {
  const __bf16* q;        // [B, Hq, D]
  const __bf16* k;
  const __bf16* v;
  int64_t stride_b, stride_h, stride_t;   // elements
  SplitArgs sp;
  int hq, hkv, group;     // group = hq / hkv
  int qblocks;            // ceil(group / 16)
  int rpu;                // partial rows per unit = min(group, 16)
  float scale_log2;       // softmax scale * log2(e)
  float* partials;        // per pair [rpu, chunks of the pair, D + 2], pairs in unit order
  int* table;             // [batch][2]: first unit and chunks per pair of every sequence, for the merge kernel
  uint32_t* status;       // sticky device status word
  // the fused decode step only: the row each sequence appends at position kv_len[b], [B, Hkv, D]
  const __bf16* k_new;
  const __bf16* v_new;
};

// Number of keys the query at position n - 1 attends to.  The visible list is the sinks [0, s_end)
// followed by the window tail [tail_start, n); `sparse` says whether anything lies hidden between them.
__device__ __forceinline__ int visible_len(int n, int md, int sink_lim, int win_blocks, int shift, bool& sparse,
                                           int& s_end, int& tail_start) {
  s_end = n < sink_lim ? n : sink_lim;
  const int lo = n > 0 ? window_start(n - 1, shift, win_blocks) : 0;
  tail_start = lo > s_end ? lo : s_end;
  sparse = ((md & 1) == 0) && (tail_start > s_end);          // bit 0 of md: 1 = FA
  return sparse ? s_end + (n - tail_start) : n;
}

constexpr int kResidentUnits = 768;             // workgroups the chip holds at once (three per CU at this register count)

// Length and mode of sequence b under the clamp: a length the host could not see (negative, or past the
// capacity of a full cache) is cut and reported through `bad`.
// With s.bump the length returned counts the row the call appends, and bit 1 of md says that it does (a full cache
// drops the row).
__device__ __forceinline__ void load_seq(const SplitArgs& s, int b, int& len, int& md, bool& bad) {
  len = s.kv_len[b];
  md = s.ring ? 0 : s.mode[b];
  bad = len < 0 || (!s.ring && len > s.capacity);
  len = len < 0 ? 0 : ((!s.ring && len > s.capacity) ? s.capacity : len);
  md = md != 0 ? 1 : 0;
  if (s.bump && len < s.capacity) {
    ++len;
    md |= 2;
  }
}

// Visible keys of a sequence of `len` rows in mode `md`, cut at the host's bound (reported through `bad`).
__device__ __forceinline__ int seq_visible(const SplitArgs& s, int len, int md, bool& bad, bool& sparse, int& s_end,
                                           int& tail_start) {
  int nv = visible_len(len, md, s.sink_lim, s.win_blocks, s.blk_shift, sparse, s_end, tail_start);
  if (nv > s.max_keys) {
    bad = true;
    nv = s.max_keys;
  }
  return nv;
}

// The split of one call, as every wave of both kernels computes it from the lengths and mode bytes.
struct Split {
  int chunk;        // keys per unit: the visible keys of all pairs, counted in 128-key pieces, divided over
                    // kTargetUnits (at least kMinChunk); the units then number at most kTargetUnits + batch * pps
  int b;            // the sequence found (-1: the unit lies past the last one)
  int first_unit;   // first unit of that sequence
  int nc;           // its chunks per (KV head, query block) pair
  int len, md;      // its clamped length and mode
  bool any_bad;     // this lane saw a clamp trip
};

// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves (add within rows of 16 by
// shifts of 1, 2, 4, 8, then carry lane 15 of each row into the next row and lane 31 into the upper half);
// lanes without a source keep the 0 passed as the old value.  Lane 63 ends up with the total.
__device__ __forceinline__ int wave_inclusive_sum(int x) {
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);   // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);   // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);   // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);   // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
  return x;
}

// unit >= 0: find the sequence whose units contain `unit`.  unit < 0: locate sequence `want_b`.
// Lane i of the wave looks after sequences i, i + 64, ...; a batch of up to 64 takes one load per lane.
__device__ __forceinline__ Split find_split(const SplitArgs& s, int lane, int unit, int want_b) {
  Split r;
  r.b = -1;
  r.first_unit = r.nc = r.len = 0;
  r.md = 1;
  r.any_bad = false;
  bool sparse;
  int s_end, tail_start;
  int len0 = 0, md0 = 1, nv0 = 0;                          // block 0 stays in registers for the second pass
  int pieces = 0;
  for (int b0 = 0; b0 < s.batch; b0 += 64) {
    int len = 0, md = 1, nv = 0;
    if (b0 + lane < s.batch) {
      bool bad;
      load_seq(s, b0 + lane, len, md, bad);
      nv = seq_visible(s, len, md, bad, sparse, s_end, tail_start);
      r.any_bad |= bad;
    }
    if (b0 == 0) {
      len0 = len;
      md0 = md;
      nv0 = nv;
    }
    pieces += __builtin_amdgcn_readlane(wave_inclusive_sum((nv + 127) >> 7), 63);
  }
  const long long c128 = ((long long)pieces * s.pps + (kTargetUnits - 1)) / kTargetUnits;
  r.chunk = c128 * 128 < kMinChunk ? kMinChunk : (int)(c128 * 128);
  // If a chunk of about twice that size cuts the batch into one nearly full round of the workgroups the chip
  // holds at once, take it: a single round of equal workgroups pays the start and the merge of a workgroup
  // once instead of twice (3 us of a 30 us call).  Uniform batches do; a ragged one usually spills a few
  // units into a second round, which would double the time, and a short list (a sparse layer) leaves much
  // of the round empty: both keep the smaller chunk.
  if (s.batch <= 64) {
    const long long o128 = ((long long)pieces * s.pps + (kResidentUnits - 1)) / kResidentUnits;
    const int big = o128 * 128 < kMinChunk ? kMinChunk : (int)(o128 * 128);
    const int units = __builtin_amdgcn_readlane(wave_inclusive_sum(s.pps * ((nv0 + big - 1) / big)), 63);
    if (units <= kResidentUnits && units > kResidentUnits - kResidentUnits / 10) r.chunk = big;
  }

  for (int b0 = 0, base = 0; b0 < s.batch; b0 += 64) {
    int len = len0, md = md0, nv = nv0;
    if (b0 > 0) {
      len = 0, md = 1, nv = 0;
      if (b0 + lane < s.batch) {
        bool bad;
        load_seq(s, b0 + lane, len, md, bad);
        nv = seq_visible(s, len, md, bad, sparse, s_end, tail_start);
      }
    }
    const int nc = (nv + r.chunk - 1) / r.chunk;
    const int incl = wave_inclusive_sum(s.pps * nc);        // units up to and including this lane's sequence
    const int total = __builtin_amdgcn_readlane(incl, 63);
    const bool here = unit >= 0 ? unit < base + total : want_b < b0 + 64;
    if (here) {                                             // wave-uniform
      const int idx = unit >= 0 ? __builtin_popcountll(__builtin_amdgcn_ballot_w64(base + incl <= unit)) : want_b - b0;
      const int sidx = __builtin_amdgcn_readfirstlane(idx);
      r.b = b0 + sidx;
      r.first_unit = base + (sidx > 0 ? __builtin_amdgcn_readlane(incl, sidx - 1) : 0);
      r.nc = __builtin_amdgcn_readlane(nc, sidx);
      r.len = __builtin_amdgcn_readlane(len, sidx);
      r.md = __builtin_amdgcn_readlane(md, sidx);
      break;
    }
    base += total;
  }
  return r;
}

// Merge the chunks of one (sequence, query head): out[d] = sum_c w_c O_c[d] / sum_c w_c l_c, w_c = exp(m_c - max m),
// chunks taken in index order.  Called by D consecutive threads (d = 0 .. D-1, whole waves) that share `wgt` (D floats)
// and `red` (4 floats) in LDS.  It holds workgroup barriers: every thread of the workgroup makes the call, each group
// of D threads with its own arrays and the same nc.  base: the head's rows [chunk][D + 2] of the workspace.
// The split as a table, for the merge kernel: entry b = (first unit, chunks per pair) of sequence b.  One wave writes
// it (lane i looks after sequences i, i + 64, ...), with the same arithmetic as find_split.
__device__ __forceinline__ void write_split_table(const SplitArgs& s, int lane, int chunk, int* table) {
  bool sparse, bad;
  int s_end, tail_start;
  for (int b0 = 0, base = 0; b0 < s.batch; b0 += 64) {
    int len = 0, md = 1, nv = 0;
    if (b0 + lane < s.batch) {
      load_seq(s, b0 + lane, len, md, bad);
      nv = seq_visible(s, len, md, bad, sparse, s_end, tail_start);
    }
    const int nc = (nv + chunk - 1) / chunk;
    const int incl = wave_inclusive_sum(s.pps * nc);
    if (b0 + lane < s.batch) {
      table[2 * (b0 + lane)] = base + incl - s.pps * nc;
      table[2 * (b0 + lane) + 1] = nc;
    }
    base += __builtin_amdgcn_readlane(incl, 63);
  }
}

template <int D>
__device__ __forceinline__ float merge_head(const float* base, int nc, float scale_log2, int d, float* wgt, float* red) {
  constexpr int RED = D + 2;
  // ---- maximum over the chunks (threads take chunks round-robin, then a reduction over the group's waves)
  float m = -INFINITY;
  for (int c = d; c < nc; c += D) m = fmaxf(m, base[c * RED + D]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  if ((d & 63) == 0) red[d >> 6] = m;
  __syncthreads();
  m = D == 128 ? fmaxf(red[0], red[1]) : red[0];
  // ---- weights per chunk in LDS, D chunks at a time; every thread then sums its own column
  float num = 0.f, den = 0.f;
  for (int c0 = 0; c0 < nc; c0 += D) {
    __syncthreads();
    const int c = c0 + d;
    float w = 0.f, l = 0.f;
    if (c < nc) {
      w = fast_exp2((base[c * RED + D] - m) * scale_log2);
      l = base[c * RED + D + 1];
    }
    wgt[d] = w;
    den += w * l;                                            // partial; reduced over the group below
    __syncthreads();
    const int cn = min(D, nc - c0);
    for (int cc = 0; cc < cn; ++cc) num += wgt[cc] * base[(c0 + cc) * RED + d];
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) den += __shfl_xor(den, off);
  __syncthreads();
  if ((d & 63) == 0) red[2 + (d >> 6)] = den;
  __syncthreads();
  den = D == 128 ? red[2] + red[3] : red[2];
  return nc > 0 ? num / den : 0.f;                          // an empty cache yields zeros
}

// FUSED: the call is a whole decode step of the layer (Sec. 3.3): it also appends the row k_new / v_new of every
// sequence at position kv_len[b].  The unit that owns the end of a list stores the row in the cache; the units that
// attend to it take it from k_new / v_new, so no read waits for that store.  The lengths are moved on by the merge
// kernel, after every workgroup of both kernels has read them.  Two launches instead of three.
template <int D, bool NT, bool FUSED>
__global__ __launch_bounds__(256) void decode_splitk_kernel(DecodeArgs a) {
  constexpr int KC = D / 32;          // MFMA k-steps over the head dimension
  constexpr int DB = D / 16;          // 16-wide output blocks over the head dimension
  constexpr int VL = D / 16;          // 16-byte V loads per lane per 32-key block
  constexpr int CPR = D / 8;          // 16-byte chunks per row
  constexpr int VROW = D + 8;         // padded LDS row (elements)
  constexpr int RED = D + 2;

  __shared__ __attribute__((aligned(16))) char smem[4 * 32 * VROW * 2];

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;
  const int g = l >> 4, n = l & 15;
  const int unit = blockIdx.x;

  // ---- the split: chunk size from the whole batch, then the sequence whose units contain `unit`
  const Split sp = find_split(a.sp, l, unit, -1);
  if (unit == 0 && w == 0 && sp.any_bad) atomicOr(a.status, (uint32_t)FLUX_DEV_BAD_LENGTH);
  // the last workgroup of the grid (idle unless the host's bound on the units is met exactly) leaves the split
  // behind for the merge kernel, which then needs neither the lengths nor the scan
  if (unit == (int)gridDim.x - 1 && w == 0) write_split_table(a.sp, l, sp.chunk, a.table);
  if (sp.b < 0) return;                                     // past the last unit: uniform for the whole workgroup
  const int b = sp.b;
  const int local = unit - sp.first_unit;                   // < pps * nc, chunk index fastest
  const int ci = local % sp.nc;
  const int pair = local / sp.nc;
  const int kvh = pair / a.qblocks;
  const int qb = pair % a.qblocks;

  bool bad_b = false, sparse;
  int s_end, tail_start;
  const int n_vis = seq_visible(a.sp, sp.len, sp.md, bad_b, sparse, s_end, tail_start);
  // The chunk size fixes how many units a pair has (sp.nc); the pair's 128-key blocks then go round its units: unit ci
  // takes the blocks ci, ci + nc, ci + 2 nc, ...  Every unit of a pair gets the same number of blocks to within one
  // (chunks of consecutive keys leave the last unit of every pair a remainder, which costs a ragged batch a tenth of
  // its time), and the units of a pair, which run side by side, read one moving window of consecutive rows.
  const int c0 = ci * 128;
  const int c1 = n_vis;
  const int pstep = 128 * sp.nc;
  const int tail0 = tail_start - s_end;                     // list index p >= s_end maps to key p + tail0
  // ring store (s_end = sink_lim when sparse): that key sits in row sink_lim + (p + tail0 - sink_lim) % ring_window
  //                                                               = sink_lim + (p - sink_lim + ring0) % ring_window
  const int ring_window = a.sp.win_blocks << a.sp.blk_shift;
  const int ring0 = (a.sp.ring && sparse) ? tail0 % ring_window : 0;

  const __bf16* kbase = a.k + (int64_t)b * a.stride_b + (int64_t)kvh * a.stride_h;
  const __bf16* vbase = a.v + (int64_t)b * a.stride_b + (int64_t)kvh * a.stride_h;

  // FUSED: the appended row is position sp.len - 1, the last key of every list (none when the cache was full).
  int new_key = -1;
  const __bf16* knew = nullptr;
  const __bf16* vnew = nullptr;
  if constexpr (FUSED) {
    if (sp.md & 2) {                                         // the sequence takes its row
      new_key = sp.len - 1;
      knew = a.k_new + ((int64_t)b * a.hkv + kvh) * D;
      vnew = a.v_new + ((int64_t)b * a.hkv + kvh) * D;
      if (ci == ((n_vis - 1) >> 7) % sp.nc && qb == 0 && tid < 2 * CPR) {   // this unit owns the list's last block: it stores the row
        const int c = tid % CPR;
        const __bf16* src = (tid < CPR ? knew : vnew) + 8 * c;
        __bf16* dst = const_cast<__bf16*>(tid < CPR ? kbase : vbase) + (int64_t)new_key * a.stride_t + 8 * c;
        *(u32x4*)dst = *(const u32x4*)src;
      }
    } else if (ci == 0 && pair == 0 && tid == 0) {
      atomicOr(a.status, (uint32_t)FLUX_DEV_KV_OVERFLOW);
    }
  }

  // ---- Q operand: lane (n, g) holds d = 32*kc + 8*g .. +7 of query head kvh*group + 16*qb + n
  const int qh = 16 * qb + n;
  bf16x8 qf[KC];
  {
    const u32x4 zero = {0, 0, 0, 0};
    const __bf16* qrow = a.q + ((int64_t)b * a.hq + (int64_t)kvh * a.group + (qh < a.group ? qh : 0)) * D;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      u32x4 t = *(const u32x4*)(qrow + 32 * kc + 8 * g);
      qf[kc] = __builtin_bit_cast(bf16x8, qh < a.group ? t : zero);
    }
  }

  auto key_of = [&](int p) -> int64_t {
    p = p < c1 ? p : c1 - 1;                                // keep every address inside the list
    if (!sparse || p < s_end) return (int64_t)p;
    if (!a.sp.ring) return (int64_t)p + tail0;
    const int x = p - s_end + ring0;                        // < 2 * ring_window
    return (int64_t)s_end + (x >= ring_window ? x - ring_window : x);
  };

  // A 32-key block whose keys are 32 consecutive cache rows (every block of an FA chunk, and all but the
  // few SA blocks that contain the sink / tail seam, the ring wrap or the end of the list) is addressed as
  // a wave-uniform row pointer plus per-lane offsets fixed for the whole kernel: no per-lane multiplies.
  // The lane's offset is the same for every load of a block (one register for K, one for V); what differs between
  // the loads, 16 rows per K half and 64 / CPR rows per V load, is added to the uniform row pointer.
  constexpr int RPL = 64 / CPR;                             // V rows per wave-wide load
  const int k_lane = n * (int)a.stride_t + 8 * g;           // element offsets inside a block of consecutive rows
  const int v_lane = (l / CPR) * (int)a.stride_t + (l % CPR) * 8;

  // Rows that are read once and evicted before the next step (the launcher decides by the bytes of the call) are
  // fetched with nontemporal loads (NT), which measurably raise the streaming rate of this access shape
  // (6.2 -> 7.1 TB/s in isolation).
  auto ld = [](const u32x4* p) -> u32x4 { return NT ? __builtin_nontemporal_load(p) : *p; };
  u32x4 kreg[2][KC], vreg[VL];
  auto load_block = [&](int p0) {                           // p0 is wave-uniform
    const int64_t r0 = key_of(p0);
    // (FUSED: the block that holds the appended row takes the per-lane path, where that row comes from k_new / v_new)
    const bool linear = p0 + 32 <= c1 && key_of(p0 + 31) - r0 == 31 && !(FUSED && new_key >= 0 && r0 + 31 >= new_key);
    if (linear) {
      const __bf16* kb0 = kbase + r0 * a.stride_t;
      const __bf16* vb0 = vbase + r0 * a.stride_t;
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) kreg[sb][kc] = ld((const u32x4*)(kb0 + 16 * sb * a.stride_t + k_lane + 32 * kc));
#pragma unroll
      for (int i = 0; i < VL; ++i) vreg[i] = ld((const u32x4*)(vb0 + i * RPL * a.stride_t + v_lane));
    } else {
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        const int64_t key = key_of(p0 + 16 * sb + n);
        const __bf16* row = (FUSED && key == new_key) ? knew : kbase + key * a.stride_t;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) kreg[sb][kc] = ld((const u32x4*)(row + 32 * kc + 8 * g));
      }
#pragma unroll
      for (int i = 0; i < VL; ++i) {
        const int e = i * 64 + l;
        const int64_t key = key_of(p0 + e / CPR);
        const __bf16* row = (FUSED && key == new_key) ? vnew : vbase + key * a.stride_t;
        vreg[i] = ld((const u32x4*)(row + (e % CPR) * 8));
      }
    }
  };

  FLUX_LDS __bf16* vs = (FLUX_LDS __bf16*)smem + w * 32 * VROW;

  float m_run = -INFINITY, l_run = 0.f;
  f32x4 o[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) o[i] = f32x4{0.f, 0.f, 0.f, 0.f};

  int p0 = c0 + 32 * w;
  if (p0 < c1) load_block(p0);
  while (p0 < c1) {
    // ---- stage this block's V rows in LDS and take K into MFMA operands
#pragma unroll
    for (int i = 0; i < VL; ++i) {
      const int e = i * 64 + l;
      *(FLUX_LDS u32x4*)(vs + (e / CPR) * VROW + (e % CPR) * 8) = vreg[i];
    }
    bf16x8 kf[2][KC];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) kf[sb][kc] = __builtin_bit_cast(bf16x8, kreg[sb][kc]);
    const int pnext = p0 + pstep;
    // ---- scores: s[sb][i] is key p0 + 16*sb + 4*g + i against query n
    f32x4 s[2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      s[sb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kc = 0; kc < KC; ++kc)
        s[sb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[sb][kc], qf[kc], s[sb], 0, 0, 0);
    }
    // the next block is asked for once the score MFMAs have taken this block's K registers, which the loads then
    // reuse (asked for before them, the block in flight needs registers of its own: 30 more per lane)
    __builtin_amdgcn_sched_barrier(0);
    if (pnext < c1) load_block(pnext);
    __builtin_amdgcn_sched_barrier(0);
    if (p0 + 32 > c1) {
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (p0 + 16 * sb + 4 * g + i >= c1) s[sb][i] = -INFINITY;
    }
    // ---- online softmax (row maximum over the 4 lane groups of this query)
    float mloc = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                       fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    const float m_new = fmaxf(m_run, mloc);                 // finite: the block holds a valid key
    const float alpha = fast_exp2((m_run - m_new) * a.scale_log2);
    const float mneg = -m_new * a.scale_log2;
    m_run = m_new;
    uint32_t pk[4];
    float psum = 0.f;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      const float p0f = fast_exp2(__builtin_fmaf(s[sb][0], a.scale_log2, mneg));
      const float p1f = fast_exp2(__builtin_fmaf(s[sb][1], a.scale_log2, mneg));
      const float p2f = fast_exp2(__builtin_fmaf(s[sb][2], a.scale_log2, mneg));
      const float p3f = fast_exp2(__builtin_fmaf(s[sb][3], a.scale_log2, mneg));
      pk[2 * sb] = pack_bf16(p0f, p1f);
      pk[2 * sb + 1] = pack_bf16(p2f, p3f);
      // the denominator sums the same rounded weights the numerator uses
      psum += (bf16_lo(pk[2 * sb]) + bf16_hi(pk[2 * sb])) + (bf16_lo(pk[2 * sb + 1]) + bf16_hi(pk[2 * sb + 1]));
    }
    l_run = l_run * alpha + psum;
    const bf16x8 pf = __builtin_bit_cast(bf16x8, u32x4{pk[0], pk[1], pk[2], pk[3]});
    // ---- O^T += V^T P^T
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      o[db] *= alpha;
      FLUX_LDS __bf16* src = vs + (4 * g + (n >> 2)) * VROW + 16 * db + 4 * (n & 3);
      const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((FLUX_LDS bf16x4*)src);
      const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((FLUX_LDS bf16x4*)(src + 16 * VROW));
      const bf16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
      o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf, o[db], 0, 0, 0);
    }
    p0 = pnext;
  }

  // ---- merge the four waves through LDS: red[w][n][0..D-1] = O, [D] = m, [D+1] = l
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  __syncthreads();                                          // every wave is done with its V staging
  FLUX_LDS float* red = (FLUX_LDS float*)smem;
  static_assert(4 * 16 * RED * 4 <= 4 * 32 * VROW * 2, "merge buffer must fit the staging buffer");
  {
    FLUX_LDS float* mine = red + (w * 16 + n) * RED;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) mine[16 * db + 4 * g + i] = o[db][i];
    if (g == 0) {
      mine[D] = m_run;
      mine[D + 1] = l_run;
    }
  }
  __syncthreads();
  const int nq = min(16, a.group - 16 * qb);
  for (int idx = tid; idx < nq * RED; idx += 256) {
    const int qi = idx / RED, e = idx % RED;
    float mw[4], m = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) {
      mw[ww] = red[(ww * 16 + qi) * RED + D];
      m = fmaxf(m, mw[ww]);
    }
    float val;
    if (e == D) {
      val = m;
    } else {
      val = 0.f;
#pragma unroll
      for (int ww = 0; ww < 4; ++ww) {
        const float wgt = fast_exp2((mw[ww] - m) * a.scale_log2);   // exp2(-inf) = 0 for idle waves
        val += wgt * red[(ww * 16 + qi) * RED + e];                 // e == D+1 merges l the same way
      }
    }
    // the units of one pair are consecutive: inside their block the rows run [query head][chunk], so the
    // second kernel reads one head's chunks as one contiguous run
    a.partials[(((int64_t)(unit - ci) * a.rpu) + (int64_t)qi * sp.nc + ci) * RED + e] = val;
  }
}

// Merge the chunks of one (sequence, query head): out = sum_c w_c O_c / sum_c w_c l_c,
// w_c = exp(m_c - max m), chunks taken in index order.
struct CombineArgs {
  const float* partials;
  const int* table;       // the split the first kernel took: [batch][2] = first unit, chunks per pair
  int hq, group, qblocks, rpu, out_fp32;
  float scale_log2;
  void* out;
  // the fused decode step only (bump = 1): the lengths, which this kernel moves on.  Nothing reads them any more
  // at that point: the first kernel has ended and this one takes the split from the table.
  int bump, capacity;
  int32_t* kv_len_rw;
};

template <int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(CombineArgs a) {
  constexpr int RED = D + 2;
  __shared__ float wgt[D];
  __shared__ float red[4];
  const int d = threadIdx.x, head = blockIdx.x, b = blockIdx.y;
  const int first_unit = a.table[2 * b], nc = a.table[2 * b + 1];
  const int hh = head % a.group;
  const int64_t unit0 = first_unit + (int64_t)((head / a.group) * a.qblocks + hh / 16) * nc;
  const float* base = a.partials + (unit0 * a.rpu + (int64_t)(hh % 16) * nc) * RED;
  const float r = merge_head<D>(base, nc, a.scale_log2, d, wgt, red);
  const int64_t off = ((int64_t)b * a.hq + head) * D + d;
  if (a.out_fp32) ((float*)a.out)[off] = r;
  else ((__bf16*)a.out)[off] = (__bf16)r;
  if (a.bump && head == 0 && d == 0) {
    int len = a.kv_len_rw[b];
    len = len < 0 ? 0 : (len > a.capacity ? a.capacity : len);
    a.kv_len_rw[b] = len < a.capacity ? len + 1 : len;
  }
}

hipError_t launch_decode(const Ctx& c, const flux_attn_cfg& cfg, const void* q, int max_kv_len,
                         const flux_kv_cache& cache, const uint8_t* mode, int ring, const void* k_new,
                         const void* v_new, void* out, hipStream_t s) {
  const bool fused = k_new != nullptr;                       // append + attend + merge in one launch
  const DecodePlan plan = plan_decode(cfg, cache.batch, max_kv_len);
  const float scale = cfg.softmax_scale != 0.f ? cfg.softmax_scale : 1.0f / sqrtf((float)cfg.head_dim);
  DecodeArgs a;
  a.q = (const __bf16*)q;
  a.k = (const __bf16*)cache.k;
  a.v = (const __bf16*)cache.v;
  a.stride_b = cache.stride_b;
  a.stride_h = cache.stride_h;
  a.stride_t = cache.stride_t;
  const SaGeom geom = sa_geom(cfg);
  a.sp.kv_len = cache.kv_len;
  a.sp.mode = mode;
  a.sp.batch = cache.batch;
  a.sp.capacity = cache.capacity;
  a.sp.ring = ring;
  a.sp.sink_lim = geom.sink_lim;
  a.sp.win_blocks = geom.win_blocks;
  a.sp.blk_shift = geom.shift;
  a.sp.max_keys = max_kv_len;
  a.sp.pps = plan.pps;
  a.sp.bump = fused ? 1 : 0;
  a.k_new = (const __bf16*)k_new;
  a.v_new = (const __bf16*)v_new;
  a.hq = cfg.n_q_heads;
  a.hkv = cfg.n_kv_heads;
  a.group = cfg.n_q_heads / cfg.n_kv_heads;
  a.qblocks = (a.group + 15) / 16;
  a.rpu = plan.rpu;
  a.scale_log2 = scale * kLog2e;
  a.table = (int*)c.partials;                                // the split table sits in front of the partial rows
  a.partials = c.partials + plan.table_floats;
  a.status = c.status;
  const dim3 grid(plan.units);
  // K and V bytes one call may read.  A call of a model whose layers together stream more than the 256 MB last-level
  // cache finds none of its rows there, whatever its own size (an SA layer reads 138 MB of a 4 GB cache): from 64 MB
  // on the rows are fetched with nontemporal loads (SA layer 34.5 -> 33.4 us, FA layers as before); smaller calls are
  // bound by their launches either way.
  const bool nt = 4.0 * cache.batch * cfg.n_kv_heads * cfg.head_dim * (double)max_kv_len > 64.0 * 1024 * 1024;
  if (fused) {
    if (cfg.head_dim == 128) {
      if (nt) hipLaunchKernelGGL((decode_splitk_kernel<128, true, true>), grid, dim3(256), 0, s, a);
      else hipLaunchKernelGGL((decode_splitk_kernel<128, false, true>), grid, dim3(256), 0, s, a);
    } else {
      if (nt) hipLaunchKernelGGL((decode_splitk_kernel<64, true, true>), grid, dim3(256), 0, s, a);
      else hipLaunchKernelGGL((decode_splitk_kernel<64, false, true>), grid, dim3(256), 0, s, a);
    }
  } else if (cfg.head_dim == 128) {
    if (nt) hipLaunchKernelGGL((decode_splitk_kernel<128, true, false>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((decode_splitk_kernel<128, false, false>), grid, dim3(256), 0, s, a);
  } else {
    if (nt) hipLaunchKernelGGL((decode_splitk_kernel<64, true, false>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((decode_splitk_kernel<64, false, false>), grid, dim3(256), 0, s, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  CombineArgs ca;
  ca.partials = a.partials;
  ca.table = a.table;
  ca.hq = cfg.n_q_heads;
  ca.group = a.group;
  ca.qblocks = a.qblocks;
  ca.rpu = plan.rpu;
  ca.out_fp32 = cfg.out_dtype;
  ca.scale_log2 = a.scale_log2;
  ca.out = out;
  ca.bump = a.sp.bump;
  ca.capacity = cache.capacity;
  ca.kv_len_rw = cache.kv_len;
  const dim3 cgrid(cfg.n_q_heads, cache.batch);
  if (cfg.head_dim == 128) hipLaunchKernelGGL(decode_combine_kernel<128>, cgrid, dim3(128), 0, s, ca);
  else hipLaunchKernelGGL(decode_combine_kernel<64>, cgrid, dim3(64), 0, s, ca);
  return hipGetLastError();
}

}  // namespace flux
