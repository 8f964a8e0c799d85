// GEMM epilogues of the verification forward.  Every GEMM kernel (plain fp32-FMA and bf16 MFMA) hands
// its accumulators to one of these functors as column PAIRS (n, n+32) of the same row: a 64-aligned group
// of output columns is exactly one attention head, so the rotate-half partner of dimension i (i + 32) is
// always in the same thread.  For the SwiGLU GEMM the kernel accumulates the gate and the up projection
// of the same output column side by side.
#pragma once

#include <type_traits>

#include "common.h"

namespace hsd {

// RMSNorm folded into the GEMMs around it.  The projection that completes a residual row (EpiResidualNorm below)
// leaves, besides x itself, the row times the next norm's gain (the next GEMM's operand) and the row's sum of
// squares in pieces of 64 columns; the next GEMM multiplies its accumulators by the row's
// rstd = rsqrt(mean(x^2) + eps), which commutes with the contraction: (x g rstd) W^T = rstd (x g) W^T.
// The pieces are added in ascending column order by every reader, so a row's rstd has the same bits everywhere.
struct RowScale {
  const float *ss;   // [rows][n_parts] partial sums of squares, or nullptr: the operand is already normalised
  int n_parts;       // d_model / 64
  float inv_d, eps;
  __device__ __forceinline__ float at(int m) const {
    if (ss == nullptr) return 1.0f;
    const float *p = ss + static_cast<size_t>(m) * n_parts;
    float s = 0.f;
    for (int i = 0; i < n_parts; ++i) s += p[i];
    return 1.0f / sqrtf(s * inv_d + eps);
  }
};

// C = A W^T for the QKV projection, then rotary embedding on q and k heads, q to the packed q buffer,
// k and v appended to the paged cache at the row's absolute position (speculative append).
template <typename T>
struct EpiQKV {
  static constexpr bool kDual = false;
  static constexpr bool kRowScale = true;
  int n_q_heads, n_kv_heads;
  RowMeta meta;
  PagedKV kv;
  T *q_out;  // [T, n_q_heads*64]
  RowScale rs;

  // One (row, column pair) at a time, given the row's rotary pair cs = rope_cs[m][n & 31] and cache destination
  // kvd = row_kv[m].
  __device__ __forceinline__ void pair_rw(int m, int n, float lo, float hi, float2 cs, int kvd) const {
    const int head = n >> 6, dim = n & 63;  // dim in [0, 32)
    if (head < n_q_heads + n_kv_heads) {
      const float rlo = lo * cs.x - hi * cs.y;
      const float rhi = hi * cs.x + lo * cs.y;
      lo = rlo;
      hi = rhi;
    }
    if (head < n_q_heads) {
      T *dst = q_out + static_cast<size_t>(m) * (n_q_heads * kHd) + head * kHd + dim;
      dst[0] = from_f32<T>(lo);
      dst[32] = from_f32<T>(hi);
      return;
    }
    if (kvd < 0) return;
    const int b = kvd / kBlk, tok = kvd % kBlk;
    if (head < n_q_heads + n_kv_heads) {
      T *dst = static_cast<T *>(kv.k_pool) + kv_block_offset(kv, b, head - n_q_heads) + tok * kHd + dim;
      dst[0] = from_f32<T>(lo);
      dst[32] = from_f32<T>(hi);
    } else {
      T *dst = static_cast<T *>(kv.v_pool) + kv_block_offset(kv, b, head - n_q_heads - n_kv_heads) + kv_v_elem(tok, dim);
      dst[0] = from_f32<T>(lo);
      dst[32 * kBlk] = from_f32<T>(hi);
    }
  }
  // Row-piece form used by the MFMA kernels: kPiece consecutive columns n .. n+7 (lo; n % 64 < 32) of row m and
  // their rotary partners n+32 .. n+39 (hi).  All loads first, then 16-byte stores.  The head index is the same
  // for a whole wave (wave-uniform branches).
  static constexpr int kPiece = 8;
  __device__ __forceinline__ void piece(int m, int n, float (&lo)[8], float (&hi)[8]) const {
    const int head = n >> 6, dim = n & 63;
    const bool rot = head < n_q_heads + n_kv_heads;
    const int kvd = (head >= n_q_heads) ? meta.row_kv[m] : 0;
    if (rot) {
      const floatx4 *cp = reinterpret_cast<const floatx4 *>(meta.rope_cs + static_cast<size_t>(m) * 32 + dim);
      floatx4 cs[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) cs[q] = cp[q];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float c = cs[e >> 1][2 * (e & 1)], sn = cs[e >> 1][2 * (e & 1) + 1];
        const float rlo = lo[e] * c - hi[e] * sn;
        hi[e] = hi[e] * c + lo[e] * sn;
        lo[e] = rlo;
      }
    }
    if (head < n_q_heads) {
      T *dst = q_out + static_cast<size_t>(m) * (n_q_heads * kHd) + head * kHd + dim;
      store_row(dst, lo);
      store_row(dst + 32, hi);
      return;
    }
    if (kvd < 0) return;
    const int b = kvd / kBlk, tok = kvd % kBlk;
    if (rot) {
      T *dst = static_cast<T *>(kv.k_pool) + kv_block_offset(kv, b, head - n_q_heads) + tok * kHd + dim;
      store_row(dst, lo);
      store_row(dst + 32, hi);
    } else {
      T *dst = static_cast<T *>(kv.v_pool) + kv_block_offset(kv, b, head - n_q_heads - n_kv_heads) + kv_v_elem(tok, dim);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        dst[e * kBlk] = from_f32<T>(lo[e]);
        dst[(32 + e) * kBlk] = from_f32<T>(hi[e]);
      }
    }
  }
  __device__ __forceinline__ void pair(int m, int n, float lo, float hi) const {
    pair_rw(m, n, lo, hi, meta.rope_cs[static_cast<size_t>(m) * 32 + (n & 31)], meta.row_kv[m]);
  }
};

// x += A W^T (fp32 residual stream, each element owned by one thread: deterministic).  Plain-kernel path; the MFMA
// kernels use EpiResidualNorm.
struct EpiResidual {
  static constexpr bool kDual = false;
  static constexpr bool kRowScale = false;
  float *x;
  int ld;
  static constexpr int kPiece = 4;
  __device__ __forceinline__ void piece(int m, int n, float (&lo)[4], float (&hi)[4]) const {
    float *p = x + static_cast<size_t>(m) * ld + n;
    const floatx4 a = *reinterpret_cast<const floatx4 *>(p), b = *reinterpret_cast<const floatx4 *>(p + 32);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      lo[e] += a[e];
      hi[e] += b[e];
    }
    store_row(p, lo);
    store_row(p + 32, hi);
  }
  __device__ __forceinline__ void pair(int m, int n, float lo, float hi) const {
    float *p = x + static_cast<size_t>(m) * ld + n;
    p[0] += lo;
    p[32] += hi;
  }
};

// Sum over the 8 adjacent lanes that hold one 64-column piece of a row (lanes 8k .. 8k+7), by lane-crossing moves
// inside the vector unit; every lane ends up with the same bits (the additions pair up commutatively).
__device__ __forceinline__ float sum8_lanes(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, true));   // quad_perm [2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, true));  // row_half_mirror
  return v;
}

// x += A W^T as EpiResidual, and everything the RMSNorm after it needs (see RowScale): h = x * gain
// in the GEMM operand type and the sum of squares of each 64-column piece of the row.  With gain == nullptr (no
// norm follows: last layer of a prefill) only x is updated.  MFMA kernels only.
struct EpiResidualNorm {
  static constexpr bool kDual = false;
  static constexpr bool kRowScale = false;
  float *x;
  int ld;
  const float *gain;  // [ld] gain of the norm that follows, or nullptr
  bf16 *h;            // [M][ld]
  float *ss;          // [M][ld / 64]
  static constexpr int kPiece = 4;
  __device__ __forceinline__ void piece(int m, int n, float (&lo)[4], float (&hi)[4]) const {
    float *p = x + static_cast<size_t>(m) * ld + n;
    const floatx4 a = *reinterpret_cast<const floatx4 *>(p), b = *reinterpret_cast<const floatx4 *>(p + 32);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      lo[e] += a[e];
      hi[e] += b[e];
    }
    store_row(p, lo);
    store_row(p + 32, hi);
    if (gain == nullptr) return;
    const floatx4 g0 = *reinterpret_cast<const floatx4 *>(gain + n), g1 = *reinterpret_cast<const floatx4 *>(gain + n + 32);
    floatx4 h0, h1;
    float sq = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      h0[e] = lo[e] * g0[e];
      h1[e] = hi[e] * g1[e];
      sq += lo[e] * lo[e];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) sq += hi[e] * hi[e];
    bf16 *hp = h + static_cast<size_t>(m) * ld + n;
    *reinterpret_cast<bf16x4 *>(hp) = __builtin_convertvector(h0, bf16x4);
    *reinterpret_cast<bf16x4 *>(hp + 32) = __builtin_convertvector(h1, bf16x4);
    // the 8 lanes n % 64 / 4 = 0..7 of this row hold the 64-column piece between them
    sq = sum8_lanes(sq);
    if ((n & 63) == 0) ss[static_cast<size_t>(m) * (ld >> 6) + (n >> 6)] = sq;
  }
};

// u = silu(A Wg^T) * (A Wu^T), written in the GEMM operand type.
template <typename T>
struct EpiSwiGLU {
  static constexpr bool kDual = true;
  static constexpr bool kRowScale = true;
  T *u;
  int ld;
  RowScale rs;
  // silu(g) * up with the hardware exp2 and reciprocal (each within 1 ulp; the result is rounded to the operand
  // type right after).  g -> -inf gives exp2 = +inf, rcp = 0, result -0.
  __device__ __forceinline__ static float f(float g, float up) {
    if constexpr (std::is_same<T, float>::value) {
      return g / (1.0f + expf(-g)) * up;   // fp32 debug path: full-precision library routines
    } else {
      return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g)) * up;
    }
  }
  // Row-piece form used by the MFMA kernels: eight consecutive output columns n .. n+7 of row m
  static constexpr int kPiece = 8;
  __device__ __forceinline__ void piece_dual(int m, int n, const float (&g)[8], const float (&up)[8]) const {
    float r[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = f(g[e], up[e]);
    store_row(u + static_cast<size_t>(m) * ld + n, r);
  }
  __device__ __forceinline__ void one2(int m, int n, float g, float up) const {
    u[static_cast<size_t>(m) * ld + n] = from_f32<T>(f(g, up));
  }
  __device__ __forceinline__ void pair2(int m, int n, float g_lo, float g_hi, float u_lo, float u_hi) const {
    T *p = u + static_cast<size_t>(m) * ld + n;
    p[0] = from_f32<T>(f(g_lo, u_lo));
    p[32] = from_f32<T>(f(g_hi, u_hi));
  }
};

// LM head: logits never reach memory.  Each thread folds its accumulators into a Top2 record; the
// kernel reduces the records of one row within the column tile and stores one record per (row, tile).
struct EpiLMHead {
  static constexpr bool kDual = false;
  static constexpr bool kRowScale = true;
  Top2 *part;  // [T][n_tiles]
  int n_tiles;
  int vocab;
  const int32_t *dump_slot;  // [T] or nullptr
  float *logits_dump;        // [n_dump][vocab]
  // Relaxed acceptance needs, for every candidate row c, the logit of c's own token at its PARENT row m.  The
  // children of row m in the packed pre-order tree are m+1, row_end[m+1], ... while < row_end[m] (a chain: just m+1).
  const int32_t *tokens;     // [T] packed token ids
  const int32_t *row_end;    // [T] packed index one past each row's subtree
  float *want_logit;         // [T] out, indexed by the CANDIDATE row, pre-filled with -inf; nullptr = exact rule
  RowScale rs;
  // called with the logits v[0..count) of row m at vocabulary ids n[e]: every (row, id) pair is computed by exactly
  // one thread of the launch, so each wanted logit is written once, from the accumulator that feeds the arg-max
  template <typename F>
  __device__ __forceinline__ void capture(int m, F &&match) const {
    for (int c = m + 1; c < row_end[m]; c = row_end[c]) {
      const int want = tokens[c];
      float v;
      if (want >= 0 && match(want, v)) want_logit[c] = v;
    }
  }
  __device__ __forceinline__ void dump(int m, int n, float lo, float hi) const {
    if (dump_slot != nullptr) {
      int sl = dump_slot[m];
      if (sl >= 0) {
        float *p = logits_dump + static_cast<size_t>(sl) * vocab + n;
        p[0] = lo;
        p[32] = hi;
      }
    }
  }
};

}  // namespace hsd
