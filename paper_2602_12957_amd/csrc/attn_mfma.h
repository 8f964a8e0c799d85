// Verification attention on the matrix cores (bf16 MFMA 32x32x16, fp32 online softmax).
//
// What it computes (paper Section 3.2, Eq. 8 in the chain case of the tree-ancestry mask): draft row r of
// sequence s at absolute position p attends to the cached positions 0..p of s -- the accepted prefix plus
// the rows before it in its own block, which the QKV epilogue appended to the pages just before.
//
// Work split.  A workgroup (4 waves) owns one (sequence, kv head, tile of query rows); its waves are the
// query heads that share the kv head (GQA) and/or 32-row sub-tiles, so every K/V tile staged in LDS is used
// by all of them.  Each wave keeps 32 queries: lane l <-> query l % 32.
//
// Orientation.  Both products are computed transposed so that a lane owns ONE query:
//   S^T = K Q^T   (MFMA i = key, j = query)  -> the lane's 16 registers per tile are 16 keys of its query:
//                 row max / row sum are in-register plus one exchange between the two lane halves;
//   O^T = V^T P^T (MFMA i = head dim, j = query) -> rescaling by the softmax correction is a per-lane scalar.
// P^T is fed straight from the S^T registers as the B operand.  Register v of lane half h holds key
// 8*(v/4) + 4h + v%4, so the contraction slots of a 16-key step are keys {4h..4h+3, 8+4h..8+4h+3}; the V
// pages are stored transposed and in exactly that token order ([dim][perm(token)], see kv_v_slot), hence the
// A operand of the second product is one 16-byte LDS read per lane and no transpose is ever done here.
#pragma once

#include "common.h"
#include "gemm_mfma.h"
#include "misc_kernels.h"

namespace hsd {

constexpr int kAttnKeys = 64;             // keys per LDS tile (4 pages)
constexpr int kKsStride = kHd + 8;        // bf16 per K row in LDS (16 B pad: conflict-free 128-bit reads)
constexpr int kVtStride = kBlk + 8;       // bf16 per (page, dim) row of V^T in LDS (48 B)
constexpr int kAttnStage = kAttnKeys * kKsStride + 4 * kHd * kVtStride;  // bf16 elements per stage

// tile_cu[s] = number of query tiles of sequences < s, with q_tile rows per tile.  One block of 1024 threads.
__global__ void __launch_bounds__(1024) k_attn_tiles(int n_seq, const int32_t *__restrict__ cu_q, int q_tile,
                                                     int32_t *__restrict__ tile_cu) {
  __shared__ int s_cnt[HSD_MAX_SEQ];
  __shared__ int s_part[1024];
  for (int s = threadIdx.x; s < n_seq; s += blockDim.x) s_cnt[s] = (cu_q[s + 1] - cu_q[s] + q_tile - 1) / q_tile;
  __syncthreads();
  int total = block_exclusive_scan_4096(s_cnt, n_seq, s_part);
  for (int s = threadIdx.x; s < n_seq; s += blockDim.x) tile_cu[s] = s_cnt[s];
  if (threadIdx.x == 0) tile_cu[n_seq] = total;
}

union Frag8 {
  uint4 u;
  bf16x8 v;
  uint16_t h[8];
};

// G4 = query heads of one kv head handled per workgroup (1, 2 or 4); 4/G4 row sub-tiles of 32 queries.
// grid: (upper bound of query tiles, n_kv_heads * ceil(group / G4)), block 256, dynamic LDS 2 * kAttnStage * 2 B.
template <int G4>
__global__ void __launch_bounds__(256) k_attn_mfma(int n_seq, int n_q_heads, const int32_t *__restrict__ cu_q,
                                                   const int32_t *__restrict__ seq_slot, int n_slots,
                                                   const int32_t *__restrict__ seq_len,
                                                   const int32_t *__restrict__ tile_cu, PagedKV kv,
                                                   const bf16 *__restrict__ q, bf16 *__restrict__ out) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  uint16_t *smem = reinterpret_cast<uint16_t *>(smem_raw);
  constexpr int SUB = 4 / G4, QT = 32 * SUB;

  const int tile = blockIdx.x;
  if (tile >= tile_cu[n_seq]) return;  // uniform for the whole workgroup
  int lo = 0, hi = n_seq - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (tile_cu[mid] <= tile) lo = mid; else hi = mid - 1;
  }
  const int s = lo, tile_in_seq = tile - tile_cu[s];
  const int slot = slot_of(seq_slot, s, n_slots);
  const int S = seq_len[slot], base = cu_q[s], Lq = cu_q[s + 1] - base;

  const int group = n_q_heads / kv.n_kv_heads, hb = (group + G4 - 1) / G4;
  const int kvh = blockIdx.y / hb, hgrp = blockIdx.y % hb;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6, half = lane >> 5, qj = lane & 31;
  const int head = kvh * group + hgrp * G4 + (wave % G4);
  const int row0 = tile_in_seq * QT + (wave / G4) * 32;          // first query row (within the block) of this wave
  const bool wave_active = row0 < Lq;
  const int my_row = min(row0 + qj, Lq - 1);
  const int pos_j = S + my_row;                                    // absolute position of the lane's query
  const int wave_keys = S + min(row0 + 32, Lq);                    // keys any query of this wave can see
  const int wg_keys = S + min(tile_in_seq * QT + QT, Lq);          // ... of this workgroup
  const int n_valid = S + Lq;                                      // positions holding data of this round
  const int n_tiles = (wg_keys + kAttnKeys - 1) / kAttnKeys;
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
  uint4 rk[2], rv[2];
  auto prefetch = [&](int kt) {
    const int kb = kt * kAttnKeys;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      // K: chunk c -> key c/8, 16-byte piece c%8
      int c = t + 256 * i, key = c >> 3, ch = c & 7;
      int blk = (kb + key < n_valid) ? kv_lookup_block(kv, slot, kb + key) : -1;
      rk[i] = make_uint4(0, 0, 0, 0);
      if (blk >= 0)
        rk[i] = *reinterpret_cast<const uint4 *>(kpool + kv_block_offset(kv, blk, kvh) + (key & 15) * kHd + ch * 8);
      // V^T: chunk c -> page c/128, dim (c%128)/2, half row c%2
      int pg = c >> 7, cc = c & 127, d = cc >> 1, hf = cc & 1;
      int vblk = (kb + pg * kBlk < n_valid) ? kv_lookup_block(kv, slot, kb + pg * kBlk) : -1;
      Frag8 f;
      f.u = make_uint4(0, 0, 0, 0);
      if (vblk >= 0) {
        f.u = *reinterpret_cast<const uint4 *>(vpool + kv_block_offset(kv, vblk, kvh) + d * kBlk + hf * 8);
        if (kb + pg * kBlk + kBlk > n_valid) {
          // last, partly filled page: slots of positions that hold no data of this sequence must read as 0
          // (their probability is 0, but 0 * stale-NaN would poison the product)
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            int tok = (e < 4) ? 4 * hf + e : 8 + 4 * hf + (e - 4);
            if (kb + pg * kBlk + tok >= n_valid) f.h[e] = 0;
          }
        }
      }
      rv[i] = f.u;
    }
  };
  auto store_lds = [&](int stage) {
    uint16_t *ks = smem + stage * kAttnStage, *vt = ks + kAttnKeys * kKsStride;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      int c = t + 256 * i, key = c >> 3, ch = c & 7;
      *reinterpret_cast<uint4 *>(ks + key * kKsStride + ch * 8) = rk[i];
      int pg = c >> 7, cc = c & 127, d = cc >> 1, hf = cc & 1;
      *reinterpret_cast<uint4 *>(vt + (pg * kHd + d) * kVtStride + hf * 8) = rv[i];
    }
  };

  floatx16 o[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[i][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = 0.125f * 1.4426950408889634f;  // 1/sqrt(64) * log2(e): softmax in base 2

  prefetch(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < n_tiles; ++kt) {
    if (kt + 1 < n_tiles) prefetch(kt + 1);
    const int kb = kt * kAttnKeys;
    if (wave_active && kb < wave_keys) {
      const uint16_t *ks = smem + (kt & 1) * kAttnStage, *vt = ks + kAttnKeys * kKsStride;
      floatx16 st[2];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
        for (int v = 0; v < 16; ++v) st[tt][v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          bf16x8 a = *reinterpret_cast<const bf16x8 *>(ks + (tt * 32 + qj) * kKsStride + kk * 16 + half * 8);
          st[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk].v, st[tt], 0, 0, 0);
        }
      }
      const bool need_mask = kb + kAttnKeys - 1 > S + row0;
      float mx = -INFINITY;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float sv = st[tt][v] * sc;
          if (need_mask) {
            int key = kb + tt * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
            if (key > pos_j) sv = -INFINITY;
          }
          st[tt][v] = sv;
          mx = fmaxf(mx, sv);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
      const float m_new = fmaxf(m_run, mx);   // finite: key 0 is visible to every query
      const float corr = exp2f(m_run - m_new);
      l_run *= corr;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] *= corr;
      Frag8 pf[2][2];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float p = exp2f(st[tt][v] - m_new);
          l_run += p;
          pf[tt][v >> 3].h[v & 7] = f32_to_bf16(p);
        }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const int pg = 2 * tt + kk;
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            bf16x8 a = *reinterpret_cast<const bf16x8 *>(vt + (pg * kHd + i * 32 + qj) * kVtStride + half * 8);
            o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[tt][kk].v, o[i], 0, 0, 0);
          }
        }
      m_run = m_new;
    }
    if (kt + 1 < n_tiles) store_lds((kt + 1) & 1);
    __syncthreads();
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
  if (wave_active && row0 + qj < Lq) {
    const float inv = 1.0f / l_tot;
    bf16 *op = out + static_cast<size_t>(base + row0 + qj) * qdim + head * kHd;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 pk;
        pk.x = f32_to_bf16(o[i][4 * g] * inv) | (static_cast<uint32_t>(f32_to_bf16(o[i][4 * g + 1] * inv)) << 16);
        pk.y = f32_to_bf16(o[i][4 * g + 2] * inv) | (static_cast<uint32_t>(f32_to_bf16(o[i][4 * g + 3] * inv)) << 16);
        *reinterpret_cast<uint2 *>(op + i * 32 + 8 * g + 4 * half) = pk;
      }
  }
}

}  // namespace hsd
