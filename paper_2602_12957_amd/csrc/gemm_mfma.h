// bf16 MFMA GEMM for gfx950: C[m,n] = sum_k A[m,k] * W[n,k], fp32 accumulation, fused epilogues.
//
// Both operands are K-contiguous (activations [M,K], weights [N,K]), which is what the MFMA operand
// layout wants: lane l of v_mfma_f32_32x32x16_bf16 supplies 8 consecutive k of row (l % 32), k-group
// (l / 32).  A 256-thread workgroup (4 waves, 2x2) computes a 128x128 tile; each wave a 64x64 tile as
// 2x2 MFMA tiles of 32x32, accumulators 64 fp32 registers per lane.  K is consumed in slices of BK
// staged through LDS (rows padded by 16 bytes so that the 128-bit operand reads of 8 consecutive lanes
// cover all banks), double buffered: global loads of slice k+1 are issued before the MFMAs of slice k.
//
// The kernel is written on two K-contiguous matrices P (MFMA "i" side) and Q ("j" side).  In the 32x32
// result tile, lane l holds column j = l % 32 and rows i = 8*(v/4) + 4*(l/32) + v%4 for register v.
//  - normal mode  (P = activations, Q = weights): a lane owns one output column and many rows; the two
//    N sub-tiles of a wave are columns n and n+32 of the same head -> rotary pairs stay in one lane.
//  - swapped mode (P = weights, Q = activations): a lane owns one token and many vocabulary entries, so
//    the LM-head arg-max folds in registers with no cross-lane traffic.
//  - dual mode: the Q tile interleaves 32 gate rows and 32 up rows per wave, so gate and up of the same
//    output element sit in the same lane and register (SwiGLU in place).
//
// Workgroups are numbered so that the 8 XCDs (round-robin over workgroup ids) each walk a contiguous
// range of tiles, M-tile fastest: consecutive tiles on one XCD share the weight tile in that XCD's L2.
#pragma once

#include "common.h"
#include "epilogues.h"

namespace hsd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kGemmBM = 128, kGemmBN = 128;

template <int BK>
struct GemmSmem {
  static constexpr int kStride = BK + 8;  // bf16 elements per LDS row
  static constexpr int kTile = 128 * kStride;
  static constexpr int kBytes = 2 /*stages*/ * 2 /*P,Q*/ * kTile * 2;
};

__device__ __forceinline__ void xcd_tile(int pid, int tiles_fast, int n_tiles, int &t_fast, int &t_slow) {
  int full = (n_tiles / 8) * 8;
  int p = pid;
  if (pid < full) p = (pid % 8) * (full / 8) + pid / 8;
  t_fast = p % tiles_fast;
  t_slow = p / tiles_fast;
}

enum GemmMode { kModeNormal = 0, kModeDual = 1, kModeSwapLM = 2 };

// grid: 1-D, ceil(M/128) * (N_tiles) workgroups; N_tiles = N/128 (normal, swapped; N padded up) or
// N/64 (dual, N = number of output columns).
template <int BK, int MODE, typename Epi>
__global__ void __launch_bounds__(256) k_gemm_mfma(int M, int N, int K, const bf16 *__restrict__ A,
                                                   const bf16 *__restrict__ W, Epi epi) {
  using S = GemmSmem<BK>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  uint16_t *smem = reinterpret_cast<uint16_t *>(smem_raw);

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int tiles_m = (M + kGemmBM - 1) / kGemmBM;
  const int tiles_n = (MODE == kModeDual) ? N / 64 : (N + kGemmBN - 1) / kGemmBN;
  int tm, tn;
  xcd_tile(blockIdx.x, tiles_m, tiles_m * tiles_n, tm, tn);
  const int m0 = tm * kGemmBM;
  const int n0 = tn * ((MODE == kModeDual) ? 64 : kGemmBN);

  // ---- which global row feeds tile row r of P and of Q
  auto act_row = [&](int r) { return min(m0 + r, M - 1); };
  auto w_row = [&](int r) {
    if (MODE == kModeDual) {
      int wn = r >> 6, sub = (r >> 5) & 1, j = r & 31;
      return (sub ? N : 0) + n0 + wn * 32 + j;
    }
    return min(n0 + r, N - 1);
  };

  constexpr int kChunks = BK / 8;                 // 16-byte chunks per tile row
  constexpr int kLoads = 128 * kChunks / 256;     // per thread per matrix
  const bf16 *srcP[kLoads], *srcQ[kLoads];
  int dst[kLoads];
#pragma unroll
  for (int i = 0; i < kLoads; ++i) {
    int c = t + 256 * i, r = c / kChunks, kc = c % kChunks;
    int ra = act_row(r), rw = w_row(r);
    const bf16 *pa = A + static_cast<size_t>(ra) * K + kc * 8;
    const bf16 *pw = W + static_cast<size_t>(rw) * K + kc * 8;
    srcP[i] = (MODE == kModeSwapLM) ? pw : pa;
    srcQ[i] = (MODE == kModeSwapLM) ? pa : pw;
    dst[i] = r * S::kStride + kc * 8;
  }

  uint4 regP[kLoads], regQ[kLoads];
  auto load_global = [&](int k0) {
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      regP[i] = *reinterpret_cast<const uint4 *>(srcP[i] + k0);
      regQ[i] = *reinterpret_cast<const uint4 *>(srcQ[i] + k0);
    }
  };
  auto store_lds = [&](int stage) {
    uint16_t *ps = smem + stage * 2 * S::kTile, *qs = ps + S::kTile;
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      *reinterpret_cast<uint4 *>(ps + dst[i]) = regP[i];
      *reinterpret_cast<uint4 *>(qs + dst[i]) = regQ[i];
    }
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int wi = wave >> 1, wj = wave & 1;
  const int frag_off_p = (wi * 64 + (lane & 31)) * S::kStride + (lane >> 5) * 8;
  const int frag_off_q = (wj * 64 + (lane & 31)) * S::kStride + (lane >> 5) * 8;

  const int nk = K / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk) load_global((kt + 1) * BK);
    const uint16_t *ps = smem + (kt & 1) * 2 * S::kTile, *qs = ps + S::kTile;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = *reinterpret_cast<const bf16x8 *>(ps + frag_off_p + i * 32 * S::kStride + kk * 16);
        b[i] = *reinterpret_cast<const bf16x8 *>(qs + frag_off_q + i * 32 * S::kStride + kk * 16);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_lds((kt + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue
  const int col = lane & 31, half = lane >> 5;
  if constexpr (MODE == kModeSwapLM) {
    // i side = vocabulary rows, j side = tokens: fold the lane's 2x16 values per token, merge the two lane halves
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int m = m0 + wj * 64 + j * 32 + col;
      Top2 tp = top2_init();
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int n = n0 + wi * 64 + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
          top2_push(tp, acc[i][j][v], n);
        }
      if (epi.dump_slot != nullptr && m < M) {
        int sl = epi.dump_slot[m];
        if (sl >= 0) {
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              int n = n0 + wi * 64 + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
              epi.logits_dump[static_cast<size_t>(sl) * epi.vocab + n] = acc[i][j][v];
            }
        }
      }
      Top2 other;
      other.m1 = __shfl_xor(tp.m1, 32, kWave);
      other.i1 = __shfl_xor(tp.i1, 32, kWave);
      other.m2 = __shfl_xor(tp.m2, 32, kWave);
      tp = top2_merge(tp, other);
      if (half == 0 && m < M) epi.part[static_cast<size_t>(m) * epi.n_tiles + tn * 2 + wi] = tp;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        int m = m0 + wi * 64 + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
        if (m >= M) continue;
        if constexpr (MODE == kModeDual) {
          epi.one2(m, n0 + wj * 32 + col, acc[i][0][v], acc[i][1][v]);
        } else {
          int n = n0 + wj * 64 + col;
          if (n < N) epi.pair(m, n, acc[i][0][v], acc[i][1][v]);
        }
      }
  }
}

}  // namespace hsd
