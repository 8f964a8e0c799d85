// Verification attention on the matrix cores (bf16 MFMA 32x32x16, fp32 online softmax).
//
// What it computes (paper Section 3.2, Eq. 8 in the chain case of the tree-ancestry mask): draft row r of
// sequence s at absolute position p attends to the cached positions 0..p of s -- the accepted prefix plus
// the rows before it in its own block, which the QKV epilogue appended to the pages just before.
//
// Work split.  A workgroup owns one (sequence, kv head, tile of query rows).  Its waves come in pairs: the two
// waves of a pair hold the same 32 queries of one query head (lane l <-> query l % 32) and share every
// 128-key stage between them, the first taking keys 0-63 of the stage and the second keys 64-127 ("parity").
// The pairs of a workgroup are the query heads that share the kv head (GQA) and/or further 32-row sub-tiles,
// so every K/V stage in LDS is used by all of them: 4 pairs per workgroup for region-level batches (many short
// blocks, Eq. 2), 8 pairs for page-level ones (few long blocks, Eq. 4: twice the reuse of each stage).
//
// One row's arithmetic is the same in every variant and every batch: its keys are visited in 64-key groups at
// absolute positions, even groups by one accumulator set and odd groups by another, in ascending order, and the
// two sets are folded at the end (even first).  Verification of a block and token-by-token decoding therefore give
// the same bits.
//
// Orientation.  Both products are computed transposed so that a lane owns ONE query:
//   S^T = K Q^T   (MFMA i = key, j = query)  -> the lane's 32 registers per step are 32 keys of its query:
//                 row max / row sum are in-register plus one exchange between the two lane halves;
//   O^T = V^T P^T (MFMA i = head dim, j = query) -> rescaling by the softmax correction is a per-lane scalar.
// P^T is fed straight from the S^T registers as the B operand.  Register v of lane half h holds key
// 8*(v/4) + 4h + v%4, so the contraction slots of a 16-key step are keys {4h..4h+3, 8+4h..8+4h+3}; the V
// pages are stored transposed and in exactly that token order ([dim][perm(token)], see kv_v_slot), hence the
// A operand of the second product is one 16-byte LDS read per lane and no transpose is ever done here.
//
// The key loop has two forms.  Stages whose every key is visible to every query of the workgroup (the bulk of a
// cached prefix) run with no mask, no validity checks and no special cases; the last one or two stages of a
// workgroup (the diagonal of the causal mask, the tree-ancestry mask, the partly filled last page) run the
// checked form.
#pragma once

#include "common.h"
#include "gemm_mfma.h"
#include "misc_kernels.h"

namespace hsd {

constexpr int kAttnKeys = 128;            // keys per LDS stage: 8 pages; keys 0-63 for parity 0, 64-127 for parity 1
constexpr int kKsStride = kHd + 8;        // bf16 per K row in LDS (16 B pad: conflict-free 128-bit reads)
constexpr int kVtStride = kAttnKeys + 8;  // bf16 per V^T row (one head dim, the 8 pages' token slots side by side;
                                          // 16 B pad: a row is 68 dwords, so the 128-bit reads of 16 consecutive
                                          // dims, and the stores of 16 consecutive dims, cover all 64 banks once)
constexpr int kAttnStage = kAttnKeys * kKsStride + kHd * kVtStride;   // bf16 elements per stage: K rows, then V^T rows
// Dynamic LDS of k_attn_mfma: two stages, reused after the key loop for handing the odd-parity partial results of
// each of the QS query sets (34 floats per lane) to their even-parity partners.
constexpr size_t attn_smem_bytes(int qs) {
  const size_t stages = 2 * static_cast<size_t>(kAttnStage) * 2, merge = static_cast<size_t>(qs) * 34 * 64 * 4;
  return stages > merge ? stages : merge;
}

// What a workgroup needs to know about its task -- one (query tile, kv head group) -- resolved once per pass instead
// of by every workgroup of every layer (a binary search and four dependent reads before the first K/V request
// could go out).
struct __attribute__((aligned(32))) AttnTile {
  int32_t seq;          // batch index of the sequence, -1: no task (padding of the launch)
  int32_t tile_in_seq;  // index of the tile among the sequence's tiles
  int32_t slot;         // state row (seq_len / block_table row)
  int32_t S, base, Lq;  // cached length, first row and number of rows of the sequence's block
  int32_t y;            // kv head * (head groups per kv head) + head group
  int32_t pad;
};

constexpr int kAttnMaxGroups = 1024;   // task groups placed by the balancing pass (more: plain order)
// Workgroups in the launch for `max_tiles` query tiles (an upper bound known on the host), `n_y` head groups and
// groups of `sub_tiles` tiles: 8 lists of equal length with room for the unevenness the placement can leave.
__host__ __device__ inline int attn_grid_size(int max_tiles, int n_y, int sub_tiles) {
  return 8 * ((max_tiles * n_y + 7) / 8 + sub_tiles);
}

// Task table of an attention launch: tasks[i] is the task of workgroup i, for i < n_wg = attn_grid_size(...).
//
// Placement.  Workgroup i runs on XCD i % 8 (workgroups go to the 8 XCDs round robin), and each XCD has its own L2.
// The tiles of one sequence and kv head read the same K/V, so they should meet in one L2: tasks are grouped by
// (sequence, head group, run of `sub_tiles` consecutive tiles), every group goes to ONE XCD as a whole, and the
// groups are dealt to the XCDs heaviest first, each to the XCD with the least work so far (work = 128-key stages a
// task walks) among those whose list still has room, which keeps the 8 lists level.  Inside a group the tile with
// the most keys comes first, and heavy groups come first in every list, so the long tasks of a ragged batch start
// early instead of forming the tail.  List x's j-th task becomes workgroup 8 j + x; workgroups past the end of a
// list find seq = -1.  Batches with more than kAttnMaxGroups groups are even enough by sheer number: they keep the
// plain order (sequence by sequence, heaviest tile first).
// The placement moves work between compute units and changes no result.  One block of 1024 threads.
__global__ void __launch_bounds__(1024) k_attn_tiles(int n_seq, const int32_t *__restrict__ cu_q,
                                                     const int32_t *__restrict__ seq_slot, int n_slots,
                                                     const int32_t *__restrict__ seq_len, int q_tile, int n_y,
                                                     int sub_tiles, int n_wg, AttnTile *__restrict__ tasks) {
  __shared__ int s_cnt[HSD_MAX_SEQ];      // per sequence: groups (or tiles) before it, after the scan
  __shared__ int s_part[1024];
  __shared__ int g_work[kAttnMaxGroups], g_key[kAttnMaxGroups], g_n[kAttnMaxGroups];
  __shared__ int o_group[kAttnMaxGroups], o_work[kAttnMaxGroups], o_n[kAttnMaxGroups];   // the groups in dealing order
  __shared__ int g_bin[kAttnMaxGroups], g_pos[kAttnMaxGroups];
  const int t = threadIdx.x;
  const AttnTile none{-1, 0, 0, 0, 0, 0, 0, 0};
  for (int i = t; i < n_wg; i += blockDim.x) tasks[i] = none;
  for (int s = t; s < n_seq; s += blockDim.x) {
    const int tiles = (cu_q[s + 1] - cu_q[s] + q_tile - 1) / q_tile;
    s_cnt[s] = n_y * ((tiles + sub_tiles - 1) / sub_tiles);
  }
  __syncthreads();   // also: the padding above is complete before any task is written
  const int n_groups = block_exclusive_scan_4096(s_cnt, n_seq, s_part);
  if (n_groups > kAttnMaxGroups) {
    __syncthreads();
    for (int s = t; s < n_seq; s += blockDim.x) s_cnt[s] = (cu_q[s + 1] - cu_q[s] + q_tile - 1) / q_tile;
    __syncthreads();
    block_exclusive_scan_4096(s_cnt, n_seq, s_part);
    for (int s = t; s < n_seq; s += blockDim.x) {
      const int slot = slot_of(seq_slot, s, n_slots), base = cu_q[s], Lq = cu_q[s + 1] - base;
      const int tiles = (Lq + q_tile - 1) / q_tile, S = seq_len[slot];
      for (int k = 0; k < tiles; ++k)
        for (int y = 0; y < n_y; ++y) {
          const int i = (s_cnt[s] + k) * n_y + y;
          if (i < n_wg) tasks[i] = AttnTile{s, tiles - 1 - k, slot, S, base, Lq, y, 0};
        }
    }
    return;
  }
  // group t of the batch: sequence s, head group y = local % n_y, tiles [t0, t1) with t0 = (local / n_y) * sub_tiles
  int gs = 0, gy = 0, t0 = 0, t1 = 0, slot = 0, S = 0, base = 0, Lq = 0;
  auto stages_of = [&](int tile) { return (S + min((tile + 1) * q_tile, Lq) + kAttnKeys - 1) / kAttnKeys; };
  if (t < n_groups) {
    int lo = 0, hi = n_seq - 1;   // last sequence whose first group is <= t (every sequence has at least one)
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (s_cnt[mid] <= t) lo = mid; else hi = mid - 1;
    }
    gs = lo;
    const int local = t - s_cnt[gs];
    gy = local % n_y;
    slot = slot_of(seq_slot, gs, n_slots);
    S = seq_len[slot];
    base = cu_q[gs];
    Lq = cu_q[gs + 1] - base;
    t0 = (local / n_y) * sub_tiles;
    t1 = min(t0 + sub_tiles, (Lq + q_tile - 1) / q_tile);
    int w = 0;
    for (int tile = t0; tile < t1; ++tile) w += stages_of(tile);
    g_work[t] = w;
    g_n[t] = t1 - t0;
    g_key[t] = stages_of(t1 - 1);   // its heaviest task
  }
  __syncthreads();
  if (t < n_groups) {   // rank: heaviest task first, then more work first, then lower index
    int rank = 0;
    const int k = g_key[t], w = g_work[t];
    for (int o = 0; o < n_groups; ++o) {
      const int ko = g_key[o], wo = g_work[o];
      rank += (ko > k) || (ko == k && (wo > w || (wo == w && o < t)));
    }
    o_group[rank] = t;
    o_work[rank] = w;
    o_n[rank] = g_n[t];
  }
  __syncthreads();
  if (t < kWave) {
    // One wave deals the groups; lane x < 8 keeps list x's work and length in registers.  The lists hold n_wg / 8
    // tasks each and the tasks number at most 8 * (n_wg / 8 - sub_tiles), so some list always has room for one
    // more group of at most sub_tiles tasks.
    const int cap = n_wg / 8;
    int load = 0, count = 0;
    for (int r0 = 0; r0 < n_groups; r0 += kWave) {
      // 64 groups at a time: lane l fetches group r0 + l once, the dealing loop then runs out of registers
      const bool valid = r0 + t < n_groups;
      const int n_v = valid ? o_n[r0 + t] : 0, w_v = valid ? o_work[r0 + t] : 0, g_v = valid ? o_group[r0 + t] : 0;
      int my_bin = 0, my_pos = 0;
      const int m = min(kWave, n_groups - r0);
      for (int j = 0; j < m; ++j) {
        const int n = __builtin_amdgcn_readlane(n_v, j), w = __builtin_amdgcn_readlane(w_v, j);
        // least work among the lists with room; equal work: the lower list (work stays far below 2^27)
        int key = (t < 8 && count + n <= cap) ? ((load << 3) | t) : 0x7fffffff;
        key = min(key, __builtin_amdgcn_update_dpp(0x7fffffff, key, 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
        key = min(key, __builtin_amdgcn_update_dpp(0x7fffffff, key, 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
        key = min(key, __builtin_amdgcn_update_dpp(0x7fffffff, key, 0x141, 0xf, 0xf, false));   // row_half_mirror
        const int best = __builtin_amdgcn_readfirstlane(key) & 7;
        const int pos = __builtin_amdgcn_readlane(count, best);
        if (t == j) {
          my_bin = best;
          my_pos = pos;
        }
        if (t == best) {
          load += w;
          count += n;
        }
      }
      if (valid) {
        g_bin[g_v] = my_bin;
        g_pos[g_v] = my_pos;
      }
    }
  }
  __syncthreads();
  if (t < n_groups) {
    for (int k = 0; k < t1 - t0; ++k) {   // heaviest tile first
      const int i = 8 * (g_pos[t] + k) + g_bin[t];
      if (i < n_wg) tasks[i] = AttnTile{gs, t1 - 1 - k, slot, S, base, Lq, gy, 0};
    }
  }
}

// Key split.  With `chunk_keys` > 0 the keys of every sequence are cut at the absolute positions chunk_keys,
// 2*chunk_keys, ... (a multiple of the 128-key stage; chunk kAttnMaxChunks - 1 is open ended) and each chunk of a
// query tile goes to a workgroup of its own (grid z), which leaves its un-normalised (max, sum, O^T) in `part_*`;
// k_attn_merge folds the chunks of a row in ascending order.  The cut points depend on absolute positions only,
// never on the batch, so a row gets the same bits whether it is scored in a long block or alone; what changes
// against the unsplit kernel is the grouping of the fp32 sums, i.e. rounding.
// Short contexts with few query tiles (region-level drafts) gain the workgroups they need to fill the chip; the
// price is 264 bytes written and read again per (row, head, chunk).
constexpr int kAttnMaxChunks = 8;
struct AttnSplit {
  int chunk_keys, total_q;
  float *part_o;     // [kAttnMaxChunks][n_q_heads][total_q][64] un-normalised O rows
  float2 *part_ml;   // [kAttnMaxChunks][n_q_heads][total_q] (integer reference point, sum)
};

union Frag8 {
  uint4 u;
  bf16x8 v;
  uint16_t h[8];
};

// QS = query sets (pairs of waves; 32 queries x one head each) per workgroup: 4 (region-level) or 8 (page-level).
// G4 = query heads of one kv head among them (1, 2 or 4); QS/G4 row sub-tiles of 32 queries.
// Waves w and w + QS form a pair: same queries, parity 0 / 1 of every stage.  Their partial (reference point, sum,
// O^T) are folded through LDS at the end, always in the same order, so results do not depend on timing.
// TREE selects the tree-ancestry mask (row_end = packed index one past each row's subtree) instead of the causal one.
// SPLIT: grid z = key chunk (see AttnSplit); results go to the partial buffers instead of `out`.
// grid: (attn_grid_size(...) tasks, 1, chunks), block 128*QS, dynamic LDS attn_smem_bytes(QS).
template <int G4, int QS, bool TREE, bool SPLIT>
__global__ void __launch_bounds__(128 * QS) k_attn_mfma(int n_q_heads, const AttnTile *__restrict__ tiles, PagedKV kv,
                                                        const bf16 *__restrict__ q, bf16 *__restrict__ out,
                                                        const int32_t *__restrict__ row_end, AttnSplit sp) {
  // staging: the 8 pages of a stage are spread over the 2*QS waves; a page's K is 128 16-byte pieces, its V^T too
  constexpr int NS = 8 / QS;                      // K pieces (and V^T pieces) per lane and stage: 2 or 1
  static_assert(QS == 4 || QS == 8, "a stage's 8 pages are staged by 8 or 16 waves");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  uint16_t *smem = reinterpret_cast<uint16_t *>(smem_raw);
  constexpr int SUB = QS / G4, QT = 32 * SUB;

  // the tile's descriptor comes through the scalar unit in one read (constant address space: written by an
  // earlier kernel, never during this one)
  typedef const int32_t __attribute__((address_space(4))) *ConstI32;
  const ConstI32 td = (ConstI32)(reinterpret_cast<const int32_t *>(tiles + blockIdx.x));
  const int s = td[0];
  if (s < 0) return;  // uniform for the whole workgroup
  const int tile_in_seq = td[1], slot = td[2], S = td[3], base = td[4], Lq = td[5], ty = td[6];

  const int group = n_q_heads / kv.n_kv_heads, hb = (group + G4 - 1) / G4;
  const int kvh = ty / hb, hgrp = ty % hb;
  const int t = threadIdx.x, lane = t & 63, half = lane >> 5, qj = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wq = wave % QS, par = wave / QS;                       // query-set index, parity of the wave
  const int head = kvh * group + hgrp * G4 + (wq % G4);
  const int row0_wg = tile_in_seq * QT;
  const int row0 = row0_wg + (wq / G4) * 32;                       // first query row (within the block) of this wave
  const bool wave_active = row0 < Lq;
  const int my_row = min(row0 + qj, Lq - 1);
  const int pos_j = S + my_row;                                    // absolute position of the lane's query
  const int wave_keys = S + min(row0 + 32, Lq);                    // keys any query of this wave can see
  const int wg_keys = S + min(row0_wg + QT, Lq);                   // ... of this workgroup
  const int n_valid = S + Lq;                                      // positions holding data of this round
  // stages kt0 .. kt1-1 of 128 keys are this workgroup's
  int key_lo = 0, key_hi = wg_keys;
  if constexpr (SPLIT) {
    key_lo = static_cast<int>(blockIdx.z) * sp.chunk_keys;
    if (key_lo >= wg_keys) return;  // uniform for the whole workgroup: no query of the tile reaches this chunk
    if (blockIdx.z + 1 < kAttnMaxChunks) key_hi = min(wg_keys, key_lo + sp.chunk_keys);
  }
  const int kt0 = key_lo / kAttnKeys, kt1 = (key_hi + kAttnKeys - 1) / kAttnKeys;
  // stages before kt_plain need no mask and no checks: every key lies in the cached prefix (tree) or at or before
  // the workgroup's first query (chain), hence holds data and is visible to every query of the workgroup
  const int kt_plain = min(kt1, (TREE ? S : S + row0_wg + 1) / kAttnKeys);
  const int qdim = n_q_heads * kHd;

  // ---- query fragments (B operand of S^T): lane holds dims 16*kk + 8*half .. +7 of its query
  Frag8 qf[4];
  {
    const bf16 *qp = q + static_cast<size_t>(base + my_row) * qdim + head * kHd + half * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) qf[kk].u = *reinterpret_cast<const uint4 *>(qp + kk * 16);
  }

  const bf16 *kpool = static_cast<const bf16 *>(kv.k_pool);
  const bf16 *vpool = static_cast<const bf16 *>(kv.v_pool);
  // Staging.  A wave stages (QS = 4) one whole page of every stage or (QS = 8) half a page: piece c of a page is
  // 16 bytes at byte offset 16*c of the K page (key c/8, dims 8*(c%8)..) and of the V^T page (dim c/2, token slots
  // 8*(c%2)..).  For V^T a lane takes piece cv = 2*(c%32) + c/32 of its 64-piece group instead of piece c, so that 16
  // consecutive lanes write 16 consecutive dims (LDS rows) and never two halves of one row.  The page id is therefore uniform per wave: it is read through the scalar unit (constant address
  // space: the table is not written while this kernel runs), one stage ahead of the data it addresses, and the page
  // offset is scalar arithmetic.
  const int pgw = (QS == 4) ? wave : (wave >> 1);                  // page of the stage this wave stages
  const int c0 = (QS == 4) ? lane : ((wave & 1) * 64 + lane);      // first K piece of the lane; piece i is c0 + 64*i
  const int cv0 = c0 - lane + 2 * (lane & 31) + (lane >> 5);       // first V^T piece
  u32x4 rk[NS], rv[NS];
  int bid;
  typedef const int32_t __attribute__((address_space(4))) *TablePtr;
  const TablePtr table_row = (TablePtr)(kv.block_table + static_cast<size_t>(slot) * kv.max_blocks_per_seq);
  const int last_entry = kv.max_blocks_per_seq - 1;
  // fetch_id only ISSUES the read (index clamped to the table row); examining the id here would stall the wave
  // for a memory latency every iteration
  auto fetch_id = [&](int kt) { bid = table_row[min(kt * (kAttnKeys / kBlk) + pgw, last_entry)]; };
  // prefetch only ISSUES the loads.  They are unconditional: an id that is out of range (a page beyond the data of
  // this round, a damaged table) reads block 0 instead; every position such a page could stand for is masked (and
  // its V zeroed) by the checked form of the loop, and the plain form only sees pages of the cached prefix.
  auto prefetch = [&]() {
    const int b = (bid >= 0 && bid < kv.n_blocks) ? bid : 0;
    const size_t off = kv_block_offset(kv, b, kvh);
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      rk[i] = *reinterpret_cast<const u32x4 *>(kpool + off + (c0 + 64 * i) * 8);
      rv[i] = *reinterpret_cast<const u32x4 *>(vpool + off + (cv0 + 64 * i) * 8);
    }
  };
  // kt = stage the staged registers belong to
  auto store_lds = [&](int stage, int kt, bool checked) {
    uint16_t *ks = smem + stage * kAttnStage, *vt = ks + kAttnKeys * kKsStride;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      const int c = c0 + 64 * i;
      *reinterpret_cast<u32x4 *>(ks + (pgw * kBlk + (c >> 3)) * kKsStride + (c & 7) * 8) = rk[i];
      u32x4 f = rv[i];
      const int cv = cv0 + 64 * i;
      const int p0 = kt * kAttnKeys + pgw * kBlk;
      if (checked && p0 + kBlk > n_valid) {
        // partly filled (or absent) page: slots of positions that hold no data of this sequence must read as 0
        // (their probability is 0, but 0 * stale-NaN would poison the product).  Element e of the piece is
        // token 4*hf + e (e < 4) or 8 + 4*hf + e - 4; two elements per 32-bit word.
        const int hf = cv & 1;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int tok0 = (w < 2) ? 4 * hf + 2 * w : 8 + 4 * hf + 2 * (w - 2);
          uint32_t keep = 0;
          if (p0 + tok0 < n_valid) keep |= 0x0000ffffu;
          if (p0 + tok0 + 1 < n_valid) keep |= 0xffff0000u;
          f[w] &= keep;
        }
      }
      *reinterpret_cast<u32x4 *>(vt + (cv >> 1) * kVtStride + pgw * kBlk + (cv & 1) * 8) = f;
    }
  };

  floatx16 o[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[i][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = 0.125f * 1.4426950408889634f;  // 1/sqrt(64) * log2(e): softmax in base 2

  // One stage of this wave: its 64 keys (parity `par`) against its 32 queries.  CHECKED adds the masks.
  auto step = [&](int kt, auto checked_tag) {
    constexpr bool CHECKED = decltype(checked_tag)::value;
    const int kb = kt * kAttnKeys + par * 64;   // first key of this wave's part of the stage
    if (CHECKED && !(wave_active && kb < wave_keys)) return;
    const uint16_t *ks = smem + (kt & 1) * kAttnStage, *vt = ks + kAttnKeys * kKsStride;
    floatx16 st[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
      for (int v = 0; v < 16; ++v) st[b][v] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        bf16x8 a = *reinterpret_cast<const bf16x8 *>(ks + (par * 64 + b * 32 + qj) * kKsStride + kk * 16 + half * 8);
        st[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk].v, st[b], 0, 0, 0);
      }
    }
    // scores stay unscaled; the softmax scale rides in the exponent's fused multiply-add
    if constexpr (CHECKED) {
      if constexpr (TREE) {
        // packed prefix tree (tree-ancestry mask): inside the block, the key in slot S + p is visible to local
        // row r iff p is r itself or an ancestor of r, i.e. p <= r < end of p's subtree (rows are in pre-order)
        if (kb + 63 >= S) {  // the wave's keys reach into the block (wave-uniform)
          // branch-free: every subtree end is fetched (index clamped into the block) before any is looked at, so
          // the 32 reads are in flight together
          int e_sub[2][16];
#pragma unroll
          for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int kpos = kb + 32 * b + 8 * (v >> 2) + 4 * half + (v & 3);
              e_sub[b][v] = row_end[base + min(max(kpos - S, 0), Lq - 1)];
            }
#pragma unroll
          for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int kpos = kb + 32 * b + 8 * (v >> 2) + 4 * half + (v & 3);
              const bool vis = (kpos <= pos_j) & ((kpos < S) | (e_sub[b][v] > base + my_row));
              st[b][v] = vis ? st[b][v] : -INFINITY;
            }
        }
      } else if (kb + 63 > S + row0) {  // the wave's keys reach past its first query: causal mask (wave-uniform)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int kpos = kb + 32 * b + 8 * (v >> 2) + 4 * half + (v & 3);
            if (kpos > pos_j) st[b][v] = -INFINITY;
          }
      }
    }
    float mx = fmaxf(st[0][0], st[1][0]);
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(fmaxf(mx, st[0][v]), st[1][v]);
    mx = half_max(mx);
    // The running reference point is kept as an INTEGER in the base-2 exponent domain (the smallest integer
    // >= max score * scale seen so far).  Every correction factor is then an exact power of two, and the bf16
    // rounding of a probability no longer depends on which stage it was computed in: rounding commutes with
    // powers of two.  Probabilities lie in (0, 1].
    const float m_new = fmaxf(m_run, ceilf(mx * sc));
    // a query that has seen no visible key yet keeps -inf (checked form only: its first keys lie in the other
    // parity); the reference point 0 then yields p = 0 and corr = 0 without producing inf - inf
    const float msc = (CHECKED && m_new == -INFINITY) ? 0.f : m_new;
    // the reference point is an integer and seldom moves after the first stages; when it moved for no lane
    // every factor is exactly 1 and the rescale is skipped (wave-uniform branch, same bits either way)
    if (__any(m_new != m_run)) {
      const float corr = (m_run == -INFINITY) ? 0.f : ldexpf(1.0f, static_cast<int>(m_run - msc));
      l_run *= corr;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] *= corr;
    }
    m_run = m_new;
    bf16x8 pf[4];
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
#pragma unroll
    for (int pg = 0; pg < 4; ++pg) {
      floatx8 pv;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // bare hardware exponential: arguments are <= 0 and results below 2^-126 may flush to zero, far
        // beneath half a bf16 unit of any probability that matters
        pv[e] = __builtin_amdgcn_exp2f(fmaf(st[pg >> 1][8 * (pg & 1) + e], sc, -msc));
      }
      pf[pg] = __builtin_convertvector(pv, bf16x8);
      // the row sum takes the probabilities as the second product will see them (rounded to bf16), two per
      // instruction: l += p0 * 1 + p1 * 1
      l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[pg], pf[pg], 0, 1), ones, l_run, false);
      l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[pg], pf[pg], 2, 3), ones, l_run, false);
      l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[pg], pf[pg], 4, 5), ones, l_run, false);
      l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[pg], pf[pg], 6, 7), ones, l_run, false);
    }
#pragma unroll
    for (int pg = 0; pg < 4; ++pg)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        bf16x8 a = *reinterpret_cast<const bf16x8 *>(vt + (i * 32 + qj) * kVtStride + (par * 4 + pg) * kBlk + half * 8);
        o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[pg], o[i], 0, 0, 0);
      }
  };

  // Pipeline: K/V of stage kt+2 and the page id of stage kt+3 are requested at the top of iteration kt, right after
  // the staging registers (stage kt+1, requested one whole iteration earlier, so long since arrived) were written to
  // the LDS stage that iteration kt-1 finished reading.  No wave ever waits for a load it has just issued, and the
  // LDS stores run ahead of the stage's arithmetic instead of between it and the barrier.
  fetch_id(kt0);
  prefetch();
  if (kt0 + 1 < kt1) fetch_id(kt0 + 1);
  store_lds(kt0 & 1, kt0, kt0 >= kt_plain);
  if (kt0 + 1 < kt1) {
    prefetch();
    if (kt0 + 2 < kt1) fetch_id(kt0 + 2);
  }
  __syncthreads();
  int kt = kt0;
  // plain stages: stage kt+1 may already be a checked one (its store then needs the zeroing of absent positions)
  for (; kt < kt_plain; ++kt) {
    if (kt + 1 < kt1) {
      if (kt + 1 < kt_plain) store_lds((kt + 1) & 1, kt + 1, false);
      else store_lds((kt + 1) & 1, kt + 1, true);
      if (kt + 2 < kt1) {
        prefetch();
        if (kt + 3 < kt1) fetch_id(kt + 3);
      }
    }
    step(kt, std::false_type{});
    __syncthreads();
  }
  for (; kt < kt1; ++kt) {
    if (kt + 1 < kt1) {
      store_lds((kt + 1) & 1, kt + 1, true);
      if (kt + 2 < kt1) {
        prefetch();
        if (kt + 3 < kt1) fetch_id(kt + 3);
      }
    }
    step(kt, std::true_type{});
    __syncthreads();
  }

  // ---- fold the two parities of each query set through LDS (stage memory is free after the last barrier):
  // parity 0 takes in parity 1
  float *mrg = reinterpret_cast<float *>(smem_raw);   // [QS query sets][34][64 lanes]
  l_run = half_sum(l_run);
  if (par == 1) {
    float *dst = mrg + wq * 34 * 64 + lane;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) dst[(i * 16 + v) * 64] = o[i][v];
    dst[32 * 64] = m_run;
    dst[33 * 64] = l_run;
  }
  __syncthreads();
  if (par == 0 && wave_active && row0 + qj < Lq) {
    {
      const float *src = mrg + wq * 34 * 64 + lane;
      const float m_b = src[32 * 64], l_b = src[33 * 64];
      // integer exponents: exact powers of two.  Unsplit, parity 0 is never empty (key 0 is in its first stage); a
      // chunk of a split pass may hold no visible key for a row in either parity
      const float m_tot = fmaxf(m_run, m_b);
      const float ca = (m_run > -INFINITY) ? ldexpf(1.0f, static_cast<int>(m_run - m_tot)) : 0.f;
      const float cb = (m_b > -INFINITY) ? ldexpf(1.0f, static_cast<int>(m_b - m_tot)) : 0.f;
      l_run = l_run * ca + l_b * cb;
      m_run = m_tot;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] = o[i][v] * ca + src[(i * 16 + v) * 64] * cb;
    }
    if constexpr (SPLIT) {
      const size_t rh = (static_cast<size_t>(blockIdx.z) * n_q_heads + head) * sp.total_q + base + row0 + qj;
      float *po = sp.part_o + rh * kHd;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          floatx4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = o[i][4 * g + e];
          *reinterpret_cast<floatx4 *>(po + i * 32 + 8 * g + 4 * half) = ov;
        }
      if (half == 0) sp.part_ml[rh] = make_float2(m_run, l_run);
    } else {
      const float inv = 1.0f / l_run;
      bf16 *op = out + static_cast<size_t>(base + row0 + qj) * qdim + head * kHd;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          floatx4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = o[i][4 * g + e] * inv;
          *reinterpret_cast<bf16x4 *>(op + i * 32 + 8 * g + 4 * half) = __builtin_convertvector(ov, bf16x4);
        }
    }
  }
}

// Folds the key chunks of a split pass: row r (cache slot row_slot[r]) has chunks 0 .. min(kAttnMaxChunks - 1,
// slot / chunk_keys), merged in ascending order with exact power-of-two factors, then normalised.
// One thread per (head, row, 4 dims); grid ceil(n_q_heads * total_q * 16 / 256), block 256.
__global__ void __launch_bounds__(256) k_attn_merge(int n_q_heads, const int32_t *__restrict__ row_slot, AttnSplit sp,
                                                    bf16 *__restrict__ out) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int rh = idx >> 4, piece = idx & 15;            // rh = head * total_q + row
  if (rh >= n_q_heads * sp.total_q) return;
  const int head = rh / sp.total_q, row = rh - head * sp.total_q;
  const int nc = min(kAttnMaxChunks, row_slot[row] / sp.chunk_keys + 1);
  const size_t cstride = static_cast<size_t>(n_q_heads) * sp.total_q;
  float2 ml = sp.part_ml[rh];
  floatx4 o = *reinterpret_cast<const floatx4 *>(sp.part_o + static_cast<size_t>(rh) * kHd + piece * 4);
  float m_run = ml.x, l_run = ml.y;
  for (int c = 1; c < nc; ++c) {
    const float2 b = sp.part_ml[c * cstride + rh];
    const floatx4 ob = *reinterpret_cast<const floatx4 *>(sp.part_o + (c * cstride + rh) * kHd + piece * 4);
    const float m_tot = fmaxf(m_run, b.x);
    const float ca = (m_run > -INFINITY) ? ldexpf(1.0f, static_cast<int>(m_run - m_tot)) : 0.f;
    const float cb = (b.x > -INFINITY) ? ldexpf(1.0f, static_cast<int>(b.x - m_tot)) : 0.f;
    l_run = l_run * ca + b.y * cb;
    m_run = m_tot;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = o[e] * ca + ob[e] * cb;
  }
  const float inv = 1.0f / l_run;
  floatx4 ov;
#pragma unroll
  for (int e = 0; e < 4; ++e) ov[e] = o[e] * inv;
  *reinterpret_cast<bf16x4 *>(out + static_cast<size_t>(row) * n_q_heads * kHd + head * kHd + piece * 4) =
      __builtin_convertvector(ov, bf16x4);
}

}  // namespace hsd
