// Verification attention, plain version (fp32 debug path and cross-check of the MFMA kernel).
// Row r of sequence s at absolute position p attends to cached positions 0..p of s: the accepted prefix
// plus the draft rows before it in the same block, which the QKV epilogue has already appended to the
// pages (the chain case of the tree-ancestry mask, paper Section 3.2; with row_end given, the packed prefix tree
// itself).  Query head h reads kv head h/group.
// One wave per (row, query head): lanes own one key each for the scores and one head dimension each for
// the weighted sum of values; online softmax in fp32.
#pragma once

#include "common.h"
#include "gemm_simple.h"

namespace hsd {

// grid: (total_q, ceil(n_q_heads/4)), block 256 = 4 waves = 4 query heads of one row.
template <typename T>
__global__ void __launch_bounds__(256) k_attn_simple(int n_q_heads, RowMeta meta, PagedKV kv,
                                                     const T *__restrict__ q, T *__restrict__ out) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = blockIdx.x, head = blockIdx.y * 4 + wave;
  if (head >= n_q_heads) return;
  const int group = n_q_heads / kv.n_kv_heads, kvh = head / group;
  // keys live in cache slots 0 .. slot(r); slots before the block hold the accepted context (all visible), slot
  // S + i holds row i of the block: visible iff i is r's own row or (packed prefix tree) one of its ancestors
  const int s = meta.row_seq[r], n_keys = meta.row_slot[r] + 1;
  const int row0 = meta.row_base[r], S = meta.row_slot[r] - (r - row0);
  const T *kpool = static_cast<const T *>(kv.k_pool);
  const T *vpool = static_cast<const T *>(kv.v_pool);

  float qv[kHd];
  const T *qr = q + static_cast<size_t>(r) * (n_q_heads * kHd) + head * kHd;
#pragma unroll
  for (int d = 0; d < kHd; d += 8) load8(qr + d, qv + d);

  const float scale = 0.125f;  // 1/sqrt(64)
  float m = -INFINITY, l = 0.f, acc = 0.f;
  for (int j0 = 0; j0 < n_keys; j0 += kWave) {
    int j = j0 + lane;
    int blk = (j < n_keys) ? kv_lookup_block(kv, s, j) : -1;
    if (meta.row_end != nullptr && j >= S && j < n_keys && meta.row_end[row0 + j - S] <= r) blk = -1;  // not an ancestor
    float score = -INFINITY;
    if (blk >= 0) {
      const T *kp = kpool + kv_block_offset(kv, blk, kvh) + (j % kBlk) * kHd;
      float dot = 0.f;
#pragma unroll
      for (int d = 0; d < kHd; d += 8) {
        float kk[8];
        load8(kp + d, kk);
#pragma unroll
        for (int e = 0; e < 8; ++e) dot = fmaf(qv[d + e], kk[e], dot);
      }
      score = dot * scale;
    }
    float m_new = fmaxf(m, wave_max(score));
    if (m_new == -INFINITY) continue;  // no readable key in this chunk (wave-uniform)
    float pj = (blk >= 0) ? expf(score - m_new) : 0.f;
    float corr = (m == -INFINITY) ? 0.f : expf(m - m_new);
    l = l * corr + wave_sum(pj);
    acc *= corr;
    int lim = min(kWave, n_keys - j0);
    for (int jj = 0; jj < lim; ++jj) {
      float pb = __shfl(pj, jj, kWave);
      int bb = __shfl(blk, jj, kWave);
      if (bb >= 0) {
        const T *vp = vpool + kv_block_offset(kv, bb, kvh) + kv_v_elem((j0 + jj) % kBlk, lane);
        acc = fmaf(pb, to_f32(vp[0]), acc);
      }
    }
    m = m_new;
  }
  float o = (l > 0.f) ? acc / l : 0.f;
  out[static_cast<size_t>(r) * (n_q_heads * kHd) + head * kHd + lane] = from_f32<T>(o);
}

}  // namespace hsd
