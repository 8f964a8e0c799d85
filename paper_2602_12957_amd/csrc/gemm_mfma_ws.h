// bf16 MFMA GEMM with eight waves in two roles: waves 0-3 multiply (a 2x2 arrangement of wave tiles, as the 4-wave
// configurations of gemm_mfma.h: 128x128 tile with 64x64 wave tiles, or 64x128 with 32x64), waves 4-7 only move the
// operands (global -> registers -> LDS).
//
// Why.  With one workgroup per CU -- all a launch over ~2 k rows offers for the narrow projections -- a 4-wave
// workgroup has one wave per SIMD, and that wave's instruction stream serialises fragment reads + MFMAs (0.31 us
// per K slice), operand loads (0.07), LDS stores (0.14) and the barrier (0.08): measured by removing each part in
// turn, the parts add up to the 0.6 us a slice takes.  Giving the data movement to waves of its own puts two waves
// on every SIMD whose stalls are independent: the stores and load waits of one hide behind the MFMAs of the other.
//
// Same pipeline as the generic kernel (two LDS stages, two register sets, a slice requested two iterations before
// it is stored), same tile order, same epilogue (multiplying waves only), same K order in every accumulator, so
// results are bit-identical to every other tile configuration.  Modes: normal and dual (the swapped LM-head mode
// has its own kernel).
// Every wave executes exactly 1 + K/64 workgroup barriers, whichever role it has.
#pragma once

#include "gemm_mfma.h"

namespace hsd {

using GemmCfgWS = GemmCfg<128, 128, 64, 2, 2>;
using GemmCfgWS64 = GemmCfg<64, 128, 64, 2, 2>;

// Cfg: a configuration with four (multiplying) waves.
// grid: 1-D, tiles_act * tiles_w workgroups of 512 threads, Cfg::kSmemBytes + kRowScaleBytes dynamic LDS.
template <typename Cfg, int MODE, typename Epi>
__global__ void __launch_bounds__(512) k_gemm_mfma_ws(int M, int N, int K, const bf16 *__restrict__ A,
                                                      const bf16 *__restrict__ W, Epi epi) {
  static_assert(Cfg::kThreads == 256 && Cfg::BK == 64, "four multiplying waves, 64-wide K slices");
  static_assert(MODE == kModeNormal || MODE == kModeDual, "normal or dual mode");
  constexpr int BP = Cfg::BP, BQ = Cfg::BQ, BK = Cfg::BK, TM = Cfg::TM, TN = Cfg::TN, LS = Cfg::kStride;
  constexpr int NT = 256, CH = Cfg::kChunks, LP = Cfg::kLoadsP, LQ = Cfg::kLoadsQ;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  uint16_t *smem = reinterpret_cast<uint16_t *>(smem_raw);

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const bool mover = wave >= 4;
  int tiles_act, tiles_w, ta, tw;
  gemm_tiles<Cfg, MODE>(M, N, tiles_act, tiles_w);
  gemm_tile_of(blockIdx.x, M, (MODE == kModeDual) ? 2 * N : N, tiles_act, tiles_w, ta, tw);
  const int m0 = ta * BP, n0 = tw * ((MODE == kModeDual) ? BQ / 2 : BQ);
  const int nk = K / BK;

  if (mover) {
    const int tp = t - NT;
    const bf16 *srcP[LP];
    const bf16 *srcQ[LQ];
#pragma unroll
    for (int i = 0; i < LP; ++i) {
      const int c = tp + NT * i, r = c / CH, kc = c % CH;
      srcP[i] = A + static_cast<size_t>(min(m0 + r, M - 1)) * K + kc * 8;
    }
#pragma unroll
    for (int i = 0; i < LQ; ++i) {
      const int c = tp + NT * i, r = c / CH, kc = c % CH;
      int row;
      if (MODE == kModeDual) {
        // Q row r: wave column r / WNC, 32-row sub-tile (r % WNC) / 32 (even: gate, odd: up), lane row r % 32
        constexpr int WNC = BQ / Cfg::WN;
        const int wq = r / WNC, tn = (r % WNC) >> 5, j = r & 31;
        row = min(((tn & 1) ? N : 0) + n0 + wq * (WNC / 2) + (tn >> 1) * 32 + j, 2 * N - 1);
      } else {
        row = min(n0 + r, N - 1);
      }
      srcQ[i] = W + static_cast<size_t>(row) * K + kc * 8;
    }
    u32x4 regP[2][LP], regQ[2][LQ];
    // requests are unconditional (past the last slice they re-read the last one; the LDS store that follows fills a
    // stage nobody multiplies from), so every store waits for exactly the older of the two sets in flight
#define HSD_WS_LOAD(set, slice)                                                                     \
  {                                                                                                 \
    const int k0 = min((slice), nk - 1) * BK;                                                       \
    _Pragma("unroll") for (int i = 0; i < LP; ++i)                                                  \
        regP[set][i] = *reinterpret_cast<const u32x4 *>(srcP[i] + k0);                              \
    _Pragma("unroll") for (int i = 0; i < LQ; ++i)                                                  \
        regQ[set][i] = *reinterpret_cast<const u32x4 *>(srcQ[i] + k0);                              \
  }
#define HSD_WS_STORE(set, stage)                                                                    \
  {                                                                                                 \
    uint16_t *sd = smem + (stage) * Cfg::kStage;                                                    \
    _Pragma("unroll") for (int i = 0; i < LP; ++i) {                                                \
      const int c = tp + NT * i;                                                                    \
      *reinterpret_cast<u32x4 *>(sd + (c / CH) * LS + (c % CH) * 8) = regP[set][i];                 \
    }                                                                                               \
    _Pragma("unroll") for (int i = 0; i < LQ; ++i) {                                                \
      const int c = tp + NT * i;                                                                    \
      *reinterpret_cast<u32x4 *>(sd + BP * LS + (c / CH) * LS + (c % CH) * 8) = regQ[set][i];       \
    }                                                                                               \
  }
    HSD_WS_LOAD(0, 0)
    HSD_WS_LOAD(1, 1)
    HSD_WS_STORE(0, 0)
    HSD_WS_LOAD(0, 2)
    __syncthreads();                                   // barrier 1: slice 0 is in stage 0
    // iteration kt: slice kt+1 (set and stage (kt+1) & 1) goes to LDS, slice kt+3 is requested into its set
    // (four sets, i.e. requests four iterations ahead, were measured and change nothing)
    int kt = 0;
    for (; kt + 2 <= nk; kt += 2) {
      HSD_WS_STORE(1, 1)
      HSD_WS_LOAD(1, kt + 3)
      __syncthreads();
      HSD_WS_STORE(0, 0)
      HSD_WS_LOAD(0, kt + 4)
      __syncthreads();
    }
    if (kt < nk) {
      HSD_WS_STORE(1, 1)
      __syncthreads();
    }
#undef HSD_WS_LOAD
#undef HSD_WS_STORE
    return;                                            // 1 + nk barriers executed
  }

  // ---- multiplying waves
  const int wi = wave / Cfg::WN, wj = wave % Cfg::WN;
  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  const int frag_p = (wi * (BP / Cfg::WM) + (lane & 31)) * LS + (lane >> 5) * 8;
  const int frag_q = BP * LS + (wj * (BQ / Cfg::WN) + (lane & 31)) * LS + (lane >> 5) * 8;
  gemm_row_scales<Cfg, MODE>(epi, M, m0, t, NT, smem_raw);   // while the moving waves fetch the first slices
  __syncthreads();                                     // barrier 1
  for (int kt = 0; kt < nk; ++kt) {
    const uint16_t *sp = smem + (kt & 1) * Cfg::kStage;
    bf16x8 fa[2][TM], fb[2][TN];
#define HSD_WS_FRAG(buf, kk)                                                                        \
  _Pragma("unroll") for (int i = 0; i < TM; ++i) fa[buf][i] =                                       \
      *reinterpret_cast<const bf16x8 *>(sp + frag_p + i * 32 * LS + (kk) * 16);                     \
  _Pragma("unroll") for (int j = 0; j < TN; ++j) fb[buf][j] =                                       \
      *reinterpret_cast<const bf16x8 *>(sp + frag_q + j * 32 * LS + (kk) * 16);
#define HSD_WS_MMA(buf)                                                                             \
  _Pragma("unroll") for (int i = 0; i < TM; ++i) _Pragma("unroll") for (int j = 0; j < TN; ++j)     \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
    HSD_WS_FRAG(0, 0)
    HSD_WS_FRAG(1, 1)
    HSD_WS_MMA(0)
    HSD_WS_FRAG(0, 2)
    HSD_WS_MMA(1)
    HSD_WS_FRAG(1, 3)
    HSD_WS_MMA(0)
    HSD_WS_MMA(1)
#undef HSD_WS_FRAG
#undef HSD_WS_MMA
    __syncthreads();
  }
  // the moving waves have left; their last LDS stores came before the last barrier, so the stages are free for
  // the epilogue's staging
  gemm_epilogue<Cfg, MODE>(acc, M, N, m0, n0, tw, wi, wj, lane, epi,
                                  reinterpret_cast<float *>(smem_raw));
}

}  // namespace hsd
