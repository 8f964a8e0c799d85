// Small kernels around the GEMMs and the attention: row metadata + rotary table, embedding gather,
// RMSNorm, KV block reservation, LM-head arg-max reduction, acceptance scan, KV commit/rollback.
#pragma once

#include "common.h"

namespace hsd {

// ------------------------------------------------------------------------------------------------
// Row metadata of every packed row: sequence, rotary position and (cos, sin) table, cache slot, and the packed
// tree it belongs to.  A chain block is the tree in which every row's subtree is the rest of the block.
//   row_pos  = seq_len + depth   (position on the row's own root-to-node path: what the rotary embedding sees)
//   row_slot = seq_len + local index (where its K/V are stored until commit)
//   row_end  = GLOBAL row index one past the row's subtree, clamped into (row, end of the sequence's block]
//   row_par  = GLOBAL row index of the parent (nearest earlier row whose subtree contains this one), -1 for a root
// The angle is formed in fp64 (position * theta^(-2i/64)) so that positions of many thousands lose
// nothing before the fp32 rounding of cos/sin themselves.
// grid: ceil(T*32 / 256) blocks of 256 threads; thread -> (row, frequency index i)
// ------------------------------------------------------------------------------------------------
__global__ void k_row_meta(int n_seq, int total_q, const int32_t *__restrict__ cu_q,
                           const int32_t *__restrict__ seq_slot, int n_slots,
                           const int32_t *__restrict__ seq_len, float rope_theta, int32_t *__restrict__ row_seq,
                           int32_t *__restrict__ row_pos, int32_t *__restrict__ row_slot,
                           int32_t *__restrict__ row_base, float2 *__restrict__ rope_cs,
                           const int32_t *__restrict__ tree_end,
                           const int32_t *__restrict__ tree_depth, int32_t *__restrict__ row_end,
                           int32_t *__restrict__ row_par, float *__restrict__ want_logit,
                           int32_t *__restrict__ status) {
  int gid = blockIdx.x * blockDim.x + threadIdx.x;
  int r = gid >> 5, i = gid & 31;
  if (r >= total_q) return;
  // binary search: largest s with cu_q[s] <= r
  int lo = 0, hi = n_seq - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (cu_q[mid] <= r) lo = mid; else hi = mid - 1;
  }
  const int base = cu_q[lo], stop = cu_q[lo + 1], local = r - base;
  int slot = slot_of(seq_slot, lo, n_slots);
  int depth = local;
  if (tree_depth != nullptr) {
    depth = tree_depth[r];
    if (depth < 0 || depth > local || (local > 0 && depth == 0)) {
      depth = local > 0 ? 1 : 0;
      if (i == 0) atomicOr(status, HSD_STATUS_BAD_TREE);
    }
  }
  int pos = seq_len[slot] + depth;
  if (i == 0) {
    row_seq[r] = slot;
    row_pos[r] = pos;
    row_slot[r] = seq_len[slot] + local;
    row_base[r] = base;
    int e = stop;
    if (tree_end != nullptr) {
      e = base + tree_end[r];
      if (e <= r || e > stop || (local == 0 && e != stop)) {
        e = local == 0 ? stop : r + 1;
        atomicOr(status, HSD_STATUS_BAD_TREE);
      }
    }
    row_end[r] = e;
    if (row_par != nullptr) {
      // nearest earlier row whose (clamped) subtree reaches past r; row `base` (the root) always qualifies
      int p = -1;
      if (local > 0) {
        p = base;
        if (tree_end == nullptr) {
          p = r - 1;
        } else {
          for (int j = r - 1; j > base; --j) {
            int ej = base + tree_end[j];
            if (ej > r && ej <= stop) { p = j; break; }
          }
        }
      }
      row_par[r] = p;
      want_logit[r] = -INFINITY;
    }
  }
  double inv_freq = pow(static_cast<double>(rope_theta), -2.0 * i / static_cast<double>(kHd));
  double ang = static_cast<double>(pos) * inv_freq;
  double sn, cs;
  sincos(ang, &sn, &cs);
  rope_cs[static_cast<size_t>(r) * 32 + i] = make_float2(static_cast<float>(cs), static_cast<float>(sn));
}

// Where each packed row's key and value land in the paged pools: 16 * block id + slot within the block, or -1
// when the table holds no valid block for the row's position (reservation failed).  Block ids are the same in
// every layer, so the projection epilogues of all layers read this one array instead of walking
// row -> sequence -> table themselves.  Runs after the reservation kernel.
// grid: ceil(T / 256) blocks of 256 threads
__global__ void k_row_kv(int total_q, const int32_t *__restrict__ row_seq, const int32_t *__restrict__ row_slot,
                         const int32_t *__restrict__ block_table, int max_blocks_per_seq, int n_blocks,
                         int32_t *__restrict__ row_kv) {
  int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= total_q) return;
  const int pos = row_slot[r], bi = pos / kBlk;
  int b = -1;
  if (bi < max_blocks_per_seq) b = block_table[static_cast<size_t>(row_seq[r]) * max_blocks_per_seq + bi];
  row_kv[r] = (b >= 0 && b < n_blocks) ? b * kBlk + pos % kBlk : -1;
}

// dump_slot[r] = index into logits_dump for row r, or -1.  Two launches: fill -1, then scatter.
__global__ void k_fill_i32(int32_t *p, int n, int32_t v) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
__global__ void k_dump_slots(const int32_t *__restrict__ dump_rows, int n_dump, int total_q,
                             int32_t *__restrict__ dump_slot) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_dump) {
    int r = dump_rows[i];
    if (r >= 0 && r < total_q) dump_slot[r] = i;
  }
}

// ------------------------------------------------------------------------------------------------
// Embedding gather: x[r,:] = tok_embed[tokens[r],:] (widened to fp32) or embeds[r,:] if tokens[r] < 0.
// grid: T blocks; block 256 threads strided over d.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void k_embed(int d, int vocab, const int32_t *__restrict__ tokens, const float *__restrict__ embeds,
                        const T *__restrict__ table, float *__restrict__ x) {
  int r = blockIdx.x;
  int t = tokens[r];
  float *xr = x + static_cast<size_t>(r) * d;
  if (t >= 0) {
    if (t >= vocab) t = vocab - 1;  // ids are validated by the caller; clamp keeps the read in bounds
    const T *src = table + static_cast<size_t>(t) * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) xr[c] = to_f32(src[c]);
  } else if (embeds != nullptr) {
    const float *src = embeds + static_cast<size_t>(r) * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) xr[c] = src[c];
  } else {
    for (int c = threadIdx.x; c < d; c += blockDim.x) xr[c] = 0.f;
  }
}

// ------------------------------------------------------------------------------------------------
// RMSNorm: h[r,:] = x[r,:] * rsqrt(mean(x^2) + eps) * gain, fp32 math, output in the GEMM operand type.
// One wave per row, 4 rows per 256-thread block; d is a multiple of 128 so every lane reads float4s.  The
// first kNormCache float4 of a lane (rows up to 2048 wide) stay in registers between the two passes.
// ------------------------------------------------------------------------------------------------
constexpr int kNormCache = 8;

__device__ __forceinline__ float sumsq4(const floatx4 &v) { return v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3]; }

__device__ __forceinline__ void norm_store4(float *dst, const floatx4 &v, float rstd, const floatx4 &g) {
  floatx4 o = {v[0] * rstd * g[0], v[1] * rstd * g[1], v[2] * rstd * g[2], v[3] * rstd * g[3]};
  *reinterpret_cast<floatx4 *>(dst) = o;
}
__device__ __forceinline__ void norm_store4(bf16 *dst, const floatx4 &v, float rstd, const floatx4 &g) {
  floatx4 o = {v[0] * rstd * g[0], v[1] * rstd * g[1], v[2] * rstd * g[2], v[3] * rstd * g[3]};
  *reinterpret_cast<bf16x4 *>(dst) = __builtin_convertvector(o, bf16x4);   // round-to-nearest-even, 8-byte store
}

// second pass of both kernels: scale the row (cached part from registers, the rest re-read) and store it
template <typename T>
__device__ __forceinline__ void norm_write_row(const floatx4 *xr, const floatx4 (&cache)[kNormCache], int n4, int lane,
                                               float ss, int d, float eps, const float *gain, T *hr) {
  ss = wave_sum(ss);
  const float rstd = 1.0f / sqrtf(ss / static_cast<float>(d) + eps);
  const floatx4 *g4 = reinterpret_cast<const floatx4 *>(gain);
#pragma unroll
  for (int i = 0; i < kNormCache; ++i) {
    const int c = lane + kWave * i;
    if (c < n4) norm_store4(hr + 4 * c, cache[i], rstd, g4[c]);
  }
  for (int c = lane + kWave * kNormCache; c < n4; c += kWave) norm_store4(hr + 4 * c, xr[c], rstd, g4[c]);
}

template <typename T>
__global__ void k_rmsnorm(int n_rows, int d, float eps, const float *__restrict__ x, const float *__restrict__ gain,
                          T *__restrict__ h) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + wave;
  if (r >= n_rows) return;
  const floatx4 *xr = reinterpret_cast<const floatx4 *>(x + static_cast<size_t>(r) * d);
  const int n4 = d >> 2;
  floatx4 cache[kNormCache];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < kNormCache; ++i) {
    const int c = lane + kWave * i;
    if (c < n4) {
      cache[i] = xr[c];
      ss += sumsq4(cache[i]);
    }
  }
  for (int c = lane + kWave * kNormCache; c < n4; c += kWave) ss += sumsq4(xr[c]);
  norm_write_row<T>(xr, cache, n4, lane, ss, d, eps, gain, h + static_cast<size_t>(r) * d);
}

// ------------------------------------------------------------------------------------------------
// Block-wide exclusive scan of up to HSD_MAX_SEQ ints held in LDS (1024 threads, 4 items each).
// On return s_val[i] holds the exclusive prefix and the function returns the grand total.
// ------------------------------------------------------------------------------------------------
__device__ inline int block_exclusive_scan_4096(int *s_val, int n, int *s_part /*[1024]*/) {
  int t = threadIdx.x;
  int base = t * 4;
  int v[4], sum = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    v[j] = (base + j < n) ? s_val[base + j] : 0;
    sum += v[j];
  }
  s_part[t] = sum;
  __syncthreads();
  // Hillis-Steele inclusive scan over the 1024 partial sums
  for (int off = 1; off < 1024; off <<= 1) {
    int add = (t >= off) ? s_part[t - off] : 0;
    __syncthreads();
    s_part[t] += add;
    __syncthreads();
  }
  int total = s_part[1023];
  int run = s_part[t] - sum;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (base + j < n) s_val[base + j] = run;
    run += v[j];
  }
  __syncthreads();
  return total;
}

// ------------------------------------------------------------------------------------------------
// KV block reservation for the speculative append.  For every sequence, every block-table slot that
// covers positions seq_len .. seq_len+q_len-1 and holds no block gets one popped from the free stack.
// Deterministic: sequence s takes its blocks after all sequences < s, slots in increasing order.
// One block of 1024 threads (16 waves; waves stride over sequences, lanes over slots).
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024) k_kv_reserve(int n_seq, const int32_t *__restrict__ cu_q,
                                                     const int32_t *__restrict__ seq_slot, int n_slots,
                                                     const int32_t *__restrict__ seq_len,
                                                     int32_t *__restrict__ block_table, int maxb, int n_blocks,
                                                     int32_t *__restrict__ free_list, int32_t *__restrict__ free_count,
                                                     int32_t *__restrict__ status) {
  __shared__ int s_cnt[HSD_MAX_SEQ];
  __shared__ int s_part[1024];
  __shared__ int s_flags;
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (threadIdx.x == 0) s_flags = 0;
  __syncthreads();
  for (int s = wave; s < n_seq; s += 16) {
    int sl = slot_of(seq_slot, s, n_slots);
    if (lane == 0 && seq_slot != nullptr && seq_slot[s] != sl) atomicOr(&s_flags, HSD_STATUS_BAD_SLOT);
    int S = seq_len[sl], Lq = cu_q[s + 1] - cu_q[s];
    int lo = S / kBlk, hi = (S + Lq + kBlk - 1) / kBlk;
    if (hi > maxb) {
      if (lane == 0) atomicOr(&s_flags, HSD_STATUS_TABLE_OVERFLOW);
      hi = maxb;
    }
    int cnt = 0;
    for (int i = lo + lane; i < hi; i += kWave) cnt += (block_table[static_cast<size_t>(sl) * maxb + i] < 0);
    cnt = wave_sum_i(cnt);
    if (lane == 0) s_cnt[s] = cnt;
  }
  __syncthreads();
  int total = block_exclusive_scan_4096(s_cnt, n_seq, s_part);
  int avail = *free_count;
  if (avail > n_blocks) avail = n_blocks;
  if (total > avail) {
    if (threadIdx.x == 0) atomicOr(status, s_flags | HSD_STATUS_POOL_EXHAUSTED);
    return;  // nothing is taken; slots stay -1 and every later kernel skips them
  }
  for (int s = wave; s < n_seq; s += 16) {
    int sl = slot_of(seq_slot, s, n_slots);
    int S = seq_len[sl], Lq = cu_q[s + 1] - cu_q[s];
    int lo = S / kBlk, hi = (S + Lq + kBlk - 1) / kBlk;
    if (hi > maxb) hi = maxb;
    int taken = s_cnt[s];  // exclusive prefix = blocks taken by earlier sequences
    for (int i0 = lo; i0 < hi; i0 += kWave) {
      int i = i0 + lane;
      bool need = (i < hi) && (block_table[static_cast<size_t>(sl) * maxb + i] < 0);
      unsigned long long m = __ballot(need);
      int rank = __popcll(m & ((1ull << lane) - 1ull));
      if (need) block_table[static_cast<size_t>(sl) * maxb + i] = free_list[avail - 1 - (taken + rank)];
      taken += __popcll(m);
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    *free_count = avail - total;
    if (s_flags) atomicOr(status, s_flags);
  }
}

// ------------------------------------------------------------------------------------------------
// KV commit / rollback.  seq_len += 1 + alpha (alpha >= 0), or += q_len when commit_all (prefill);
// slots wholly beyond the new length are pushed back on the free stack in (sequence, slot) order.
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024) k_kv_commit(int n_seq, const int32_t *__restrict__ cu_q,
                                                    const int32_t *__restrict__ seq_slot, int n_slots,
                                                    int32_t *__restrict__ seq_len, int32_t *__restrict__ block_table,
                                                    int maxb, int n_blocks, int32_t *__restrict__ free_list,
                                                    int32_t *__restrict__ free_count,
                                                    const int32_t *__restrict__ accept_len,
                                                    const int32_t *__restrict__ bonus, int32_t *__restrict__ pending_out,
                                                    int commit_all) {
  __shared__ int s_cnt[HSD_MAX_SEQ];
  __shared__ int s_new[HSD_MAX_SEQ];
  __shared__ int s_part[1024];
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int s = wave; s < n_seq; s += 16) {
    int sl = slot_of(seq_slot, s, n_slots);
    int S = seq_len[sl], Lq = cu_q[s + 1] - cu_q[s];
    int new_len = S;
    if (commit_all) {
      new_len = S + Lq;
    } else {
      int a = accept_len[s];
      if (a > Lq - 1) a = Lq - 1;
      if (a >= 0) new_len = S + 1 + a;
    }
    int keep = (new_len + kBlk - 1) / kBlk, hi = (S + Lq + kBlk - 1) / kBlk;
    if (hi > maxb) hi = maxb;
    int cnt = 0;
    for (int i = keep + lane; i < hi; i += kWave) {
      int b = block_table[static_cast<size_t>(sl) * maxb + i];
      cnt += (b >= 0 && b < n_blocks);
    }
    cnt = wave_sum_i(cnt);
    if (lane == 0) {
      s_cnt[s] = cnt;
      s_new[s] = new_len;
    }
  }
  __syncthreads();
  int total = block_exclusive_scan_4096(s_cnt, n_seq, s_part);
  int height = *free_count;
  if (height < 0) height = 0;
  if (height + total > n_blocks) total = 0, height = -1;  // corrupted accounting: free nothing
  for (int s = wave; s < n_seq; s += 16) {
    int sl = slot_of(seq_slot, s, n_slots);
    int S = seq_len[sl], Lq = cu_q[s + 1] - cu_q[s];
    int new_len = s_new[s];
    int keep = (new_len + kBlk - 1) / kBlk, hi = (S + Lq + kBlk - 1) / kBlk;
    if (hi > maxb) hi = maxb;
    int pushed = s_cnt[s];
    if (height >= 0) {
      for (int i0 = keep; i0 < hi; i0 += kWave) {
        int i = i0 + lane;
        int b = (i < hi) ? block_table[static_cast<size_t>(sl) * maxb + i] : -1;
        bool has = (b >= 0 && b < n_blocks);
        unsigned long long m = __ballot(has);
        int rank = __popcll(m & ((1ull << lane) - 1ull));
        if (has) {
          free_list[height + pushed + rank] = b;
          block_table[static_cast<size_t>(sl) * maxb + i] = -1;
        }
        pushed += __popcll(m);
      }
    }
  }
  __syncthreads();
  for (int s = threadIdx.x; s < n_seq; s += blockDim.x) {
    bool advanced = commit_all || accept_len[s] >= 0;
    seq_len[slot_of(seq_slot, s, n_slots)] = s_new[s];
    if (!commit_all && advanced && pending_out != nullptr) pending_out[s] = bonus[s];
  }
  if (threadIdx.x == 0 && height >= 0) *free_count = height + total;
}

__global__ void k_pool_init(int n_blocks, int32_t *__restrict__ free_list, int32_t *__restrict__ free_count) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_blocks) free_list[i] = n_blocks - 1 - i;  // popping from the top hands out 0, 1, 2, ...
  if (i == 0) *free_count = n_blocks;
}

// ------------------------------------------------------------------------------------------------
// LM-head arg-max, second stage: merge the per-(row, column tile) Top2 partials of the LM-head GEMM.
// One wave per row.  Output u_hat (Eq. 10: arg-max over the vocabulary; arg-max of logits equals
// arg-max of probabilities) and the top-1/top-2 logit margin.
// ------------------------------------------------------------------------------------------------
__global__ void k_lm_reduce(int n_rows, int n_tiles, const Top2 *__restrict__ part, int32_t *__restrict__ argmax,
                            float *__restrict__ margin, float *__restrict__ row_max) {
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int r = blockIdx.x * 4 + wave;
  if (r >= n_rows) return;
  Top2 t = top2_init();
  for (int c = lane; c < n_tiles; c += kWave) t = top2_merge(t, part[static_cast<size_t>(r) * n_tiles + c]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    Top2 u;
    u.m1 = __shfl_xor(t.m1, o, kWave);
    u.i1 = __shfl_xor(t.i1, o, kWave);
    u.m2 = __shfl_xor(t.m2, o, kWave);
    t = top2_merge(t, u);
  }
  if (lane == 0) {
    argmax[r] = t.i1;
    if (margin != nullptr) margin[r] = t.m1 - t.m2;
    if (row_max != nullptr) row_max[r] = t.m1;
  }
}

// Relaxed acceptance (Eq. 11) in logits: log p(u*) - log p(u_hat) = logit(u*) - max logit, both taken at the PARENT
// row of the candidate.  draft_gap[r] = (logit of row r's own token at its parent's row) - (parent's row maximum);
// -inf for root rows.  One thread per row.
__global__ void k_draft_gap(int n_rows, const int32_t *__restrict__ row_par, const float *__restrict__ want_logit,
                            const float *__restrict__ row_max, float *__restrict__ draft_gap) {
  int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_rows) return;
  const int p = row_par[r];
  draft_gap[r] = p < 0 ? -INFINITY : want_logit[r] - row_max[p];
}

// ------------------------------------------------------------------------------------------------
// Draft compare + longest-prefix acceptance on chain blocks (Eq. 9, 11; Eq. 12 bonus; alpha of Eq. 15).
// One wave per sequence: lanes test 64 draft positions at a time, a ballot finds the first rejection.
// Exact rule (log_tau == 0): reject_i = (tokens[base+i] != argmax[base+i-1]) for i = 1..k.
// Relaxed rule (log_tau < 0): reject_i = !(draft_gap[base+i] >= log_tau).
// ------------------------------------------------------------------------------------------------
__global__ void k_accept(int n_seq, const int32_t *__restrict__ cu_q, const int32_t *__restrict__ tokens,
                         const int32_t *__restrict__ argmax, const float *__restrict__ draft_gap, float log_tau,
                         int32_t *__restrict__ accept_len, int32_t *__restrict__ bonus) {
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int s = blockIdx.x * 4 + wave;
  if (s >= n_seq) return;
  int base = cu_q[s], k = cu_q[s + 1] - base - 1;
  const bool relaxed = log_tau < 0.f && draft_gap != nullptr;
  int alpha = k;
  for (int i0 = 1; i0 <= k; i0 += kWave) {
    int i = i0 + lane;
    bool reject = false;
    if (i <= k) reject = relaxed ? !(draft_gap[base + i] >= log_tau) : (tokens[base + i] != argmax[base + i - 1]);
    unsigned long long m = __ballot(reject);
    if (m != 0ull) {
      alpha = i0 + (__ffsll(static_cast<long long>(m)) - 1) - 1;  // accepted = index of first rejection - 1
      break;
    }
  }
  if (lane == 0) {
    accept_len[s] = alpha;
    bonus[s] = argmax[base + alpha];
  }
}

// ------------------------------------------------------------------------------------------------
// Greedy traversal of a packed prefix tree (Eq. 9-12).  One thread per sequence (trees are small: the candidate
// continuations of one matching step).  At node s the children are s+1, row_end[s+1], ... while < row_end[s].
// Exact rule: enter the child whose token is the row's arg-max token, if there is one (then u* = u_hat).
// Relaxed rule: u* = the child with the largest logit at row s (lowest row among equals); enter it iff
// draft_gap[u*] >= log_tau.  Outputs alpha = depth reached, the bonus token (arg-max at the stop node) and the
// stop node's local row.
// ------------------------------------------------------------------------------------------------
__global__ void k_accept_tree(int n_seq, const int32_t *__restrict__ cu_q, const int32_t *__restrict__ tokens,
                              const int32_t *__restrict__ argmax, const int32_t *__restrict__ row_end,
                              const float *__restrict__ want_logit, const float *__restrict__ draft_gap,
                              float log_tau, int32_t *__restrict__ accept_len, int32_t *__restrict__ bonus,
                              int32_t *__restrict__ stop_row) {
  int sq = blockIdx.x * blockDim.x + threadIdx.x;
  if (sq >= n_seq) return;
  const int base = cu_q[sq];
  const bool relaxed = log_tau < 0.f && draft_gap != nullptr;
  int s = base, alpha = 0;
  for (;;) {
    int best = -1;
    float best_v = -INFINITY;
    for (int c = s + 1; c < row_end[s]; c = row_end[c]) {
      if (relaxed) {
        float v = want_logit[c];
        if (best < 0 || v > best_v) best = c, best_v = v;
      } else if (tokens[c] == argmax[s]) {
        best = c;
        break;
      }
    }
    if (best < 0) break;
    if (relaxed && !(draft_gap[best] >= log_tau)) break;
    s = best;
    ++alpha;
  }
  accept_len[sq] = alpha;
  bonus[sq] = argmax[s];
  stop_row[sq] = s - base;
}

// ------------------------------------------------------------------------------------------------
// Commit of a packed tree: the accepted root-to-stop path becomes ordinary context.  Its node at depth d was stored
// at cache slot S + (local row) and moves to slot S + d, d = 1..alpha (a node's pre-order row is never smaller
// than its depth, and no target slot is the source of a later move, so the moves are independent).
// grid: (n_seq, n_layers * n_kv_heads), block 64: lane = head dimension.  Runs BEFORE the length update.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void k_kv_compact(const int32_t *__restrict__ cu_q, const int32_t *__restrict__ seq_slot, int n_slots,
                             const int32_t *__restrict__ seq_len, const int32_t *__restrict__ block_table, int maxb,
                             int n_blocks, int n_kv_heads, const int32_t *__restrict__ tree_end,
                             const int32_t *__restrict__ accept_len, const int32_t *__restrict__ stop_row,
                             T *__restrict__ k_pool, T *__restrict__ v_pool) {
  const int sq = blockIdx.x, layer = blockIdx.y / n_kv_heads, kvh = blockIdx.y % n_kv_heads, dim = threadIdx.x;
  const int base = cu_q[sq], Lq = cu_q[sq + 1] - base;
  const int sl = slot_of(seq_slot, sq, n_slots);
  const int S = seq_len[sl];
  int alpha = accept_len[sq], stop = stop_row[sq];
  if (alpha < 1 || stop < 1 || stop >= Lq) return;
  auto end_of = [&](int i) {   // same clamping as the row metadata kernel
    int e = tree_end[base + i];
    return (e <= i || e > Lq) ? i + 1 : e;
  };
  int s = 0;
  for (int d = 1; d <= alpha; ++d) {
    // the child of s whose subtree contains the stop node
    int c = s + 1;
    while (c < Lq && !(c <= stop && stop < end_of(c))) c = end_of(c);
    if (c >= Lq) return;   // malformed tree: nothing sensible to move
    s = c;
    if (c == d) continue;  // already in place
    const int src = S + c, dst = S + d;
    if (src / kBlk >= maxb) return;
    const int bs = block_table[static_cast<size_t>(sl) * maxb + src / kBlk];
    const int bd = block_table[static_cast<size_t>(sl) * maxb + dst / kBlk];
    if (bs < 0 || bs >= n_blocks || bd < 0 || bd >= n_blocks) return;
    const size_t os = ((static_cast<size_t>(layer) * n_blocks + bs) * n_kv_heads + kvh) * (kBlk * kHd);
    const size_t od = ((static_cast<size_t>(layer) * n_blocks + bd) * n_kv_heads + kvh) * (kBlk * kHd);
    k_pool[od + (dst % kBlk) * kHd + dim] = k_pool[os + (src % kBlk) * kHd + dim];
    v_pool[od + kv_v_elem(dst % kBlk, dim)] = v_pool[os + kv_v_elem(src % kBlk, dim)];
  }
}

}  // namespace hsd
