// bf16 MFMA GEMM, large-tile variant for the wide projections (gate/up, LM head): 256x256x64 tiles, 8 waves.
//
// Why this shape.  On MI355X the L2 -> CU path sustains about 15 TB/s in aggregate for tile loads (measured),
// i.e. ~58 GB/s per CU.  A 128x128x64 step moves 32 KB for 2.1 MFLOP: at the MFMA rate that is 2.5x more bytes
// than the path delivers.  A 256x256x64 step moves 64 KB for 8.4 MFLOP, which balances the two.  Eight waves
// (2 x 4, wave tile 128x64, 128 accumulator registers) keep two waves per SIMD so that one wave's LDS reads
// and address arithmetic hide behind the other's MFMAs.
//
// Pipeline per K slice: the 8 buffer loads a thread owns for slice k+2 are issued in two groups between the
// MFMA groups of the first two k-steps of slice k (so that load issue never blocks a long MFMA run) into one of
// two register sets; the other set, holding slice k+1, is written to the free LDS stage after the last k-step.
// Loads are raw buffer loads: rows past the end of a matrix read as zero in hardware, no clamping needed.
//
// Operand roles (P = MFMA i side, Q = j side), modes and the epilogue are those of gemm_mfma.h.
#pragma once

#include "gemm_mfma.h"

namespace hsd {

using GemmCfg8 = GemmCfg<256, 256, 64, 2, 4>;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, size_t bytes) {
  // raw buffer: stride 0, num_records = bytes (capped to what 32 bits hold), data format word for gfx9-class chips
  const uint32_t n = bytes > 0xFFFFFFFFull ? 0xFFFFFFFFu : static_cast<uint32_t>(bytes);
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, static_cast<int>(n), 0x00020000);
}

// grid: 1-D, tiles_act * tiles_w workgroups of 512 threads, GemmCfg8::kSmemBytes dynamic LDS.
// K a multiple of 128 and at least 256 (an even number, >= 4, of K slices); both matrices below 2 GiB.
template <int MODE, typename Epi>
__global__ void __launch_bounds__(512) k_gemm_mfma8(int M, int N, int K, const bf16 *__restrict__ A,
                                                    const bf16 *__restrict__ W, Epi epi) {
  using Cfg = GemmCfg8;
  constexpr int BP = Cfg::BP, BQ = Cfg::BQ, BK = Cfg::BK, TM = Cfg::TM, TN = Cfg::TN, LS = Cfg::kStride;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  uint16_t *smem = reinterpret_cast<uint16_t *>(smem_raw);

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wi = wave / Cfg::WN, wj = wave % Cfg::WN;
  int tiles_act, tiles_w, ta, tw;
  gemm_tiles<Cfg, MODE>(M, N, tiles_act, tiles_w);
  gemm_tile_of(blockIdx.x, M, (MODE == kModeDual) ? 2 * N : N, tiles_act, tiles_w, ta, tw);
  const int m0 = ta * ((MODE == kModeSwapLM) ? BQ : BP);
  const int n0 = tw * ((MODE == kModeSwapLM) ? BP : ((MODE == kModeDual) ? BQ / 2 : BQ));
  gemm_row_scales<Cfg, MODE>(epi, M, m0, t, 512, smem_raw);

  // ---- staging map: chunk c = t + 512*i covers tile row t/8 + 64*i, 16-byte piece t%8
  const int r8 = t >> 3, kc = t & 7;
  const size_t w_rows = (MODE == kModeDual) ? 2 * static_cast<size_t>(N) : static_cast<size_t>(N);
  const __amdgpu_buffer_rsrc_t rs_act = make_rsrc(A, static_cast<size_t>(M) * K * 2);
  const __amdgpu_buffer_rsrc_t rs_w = make_rsrc(W, w_rows * K * 2);
  const __amdgpu_buffer_rsrc_t rs_p = (MODE == kModeSwapLM) ? rs_w : rs_act;
  const __amdgpu_buffer_rsrc_t rs_q = (MODE == kModeSwapLM) ? rs_act : rs_w;
  // Byte offset of the thread's piece in row group 0 of the tile.  The whole row offset sits in the VECTOR offset,
  // because the hardware range check of a raw buffer looks at the vector offset only: rows at or past the end of
  // the matrix then read as zero.  The scalar offset carries just the K-slice offset (less than one row).
  int voff_p = ((((MODE == kModeSwapLM) ? n0 : m0) + r8) * K + kc * 8) * 2;
  int voff_q, q_step;                                        // group i of Q is q_step bytes further
  if (MODE == kModeSwapLM) {
    voff_q = ((m0 + r8) * K + kc * 8) * 2;
    q_step = 64 * K * 2;
  } else if (MODE == kModeDual) {
    // Q row r = 64*i + r8: wave column i, sub-tile (r8 >> 5) (0 gate, 1 up), lane row r8 & 31
    voff_q = ((((r8 >> 5) ? N : 0) + n0 + (r8 & 31)) * K + kc * 8) * 2;
    q_step = 32 * K * 2;
  } else {
    voff_q = ((n0 + r8) * K + kc * 8) * 2;
    q_step = 64 * K * 2;
  }
  const int p_step = 64 * K * 2;
  const int lds_dst = r8 * LS + kc * 8;   // + i * 64 * LS

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int frag_p = (wi * (BP / Cfg::WM) + (lane & 31)) * LS + (lane >> 5) * 8;
  const int frag_q = BP * LS + (wj * (BQ / Cfg::WN) + (lane & 31)) * LS + (lane >> 5) * 8;

  // Two register sets hold the slices in flight: while slice kt is multiplied out of LDS, slice kt+1 (set X,
  // requested one iteration earlier) is landing and is written to the other LDS stage at the end of the
  // iteration, and the requests for slice kt+2 go out into set Y.  A request therefore has two full
  // iterations to come back.
  u32x4 regP[2][4], regQ[2][4];
  const int nk = K / BK;

#define HSD_G8_LOAD(set, i, kbyte)                                                                    \
  regP[set][i] = __builtin_amdgcn_raw_buffer_load_b128(rs_p, voff_p + (i) * p_step, (kbyte), 0);      \
  regQ[set][i] = __builtin_amdgcn_raw_buffer_load_b128(rs_q, voff_q + (i) * q_step, (kbyte), 0);
#define HSD_G8_STORE(set, stage, i0, i1)                                                              \
  {                                                                                                   \
    uint16_t *sd = smem + (stage) * Cfg::kStage;                                                      \
    _Pragma("unroll") for (int i = (i0); i < (i1); ++i) {                                             \
      *reinterpret_cast<u32x4 *>(sd + lds_dst + i * 64 * LS) = regP[set][i];                          \
      *reinterpret_cast<u32x4 *>(sd + BP * LS + lds_dst + i * 64 * LS) = regQ[set][i];                \
    }                                                                                                 \
  }
  // Operand fragments are double buffered in registers: the LDS reads of k-step kk+1 are issued before the MFMAs
  // of k-step kk, so their latency hides behind the matrix pipe instead of opening every k-step.
#define HSD_G8_FRAG(buf, kk)                                                                          \
  _Pragma("unroll") for (int i = 0; i < TM; ++i) fa[buf][i] =                                         \
      *reinterpret_cast<const bf16x8 *>(sp + frag_p + i * 32 * LS + (kk) * 16);                       \
  _Pragma("unroll") for (int j = 0; j < TN; ++j) fb[buf][j] =                                         \
      *reinterpret_cast<const bf16x8 *>(sp + frag_q + j * 32 * LS + (kk) * 16);
#define HSD_G8_MMA(buf)                                                                               \
  _Pragma("unroll") for (int i = 0; i < TM; ++i) _Pragma("unroll") for (int j = 0; j < TN; ++j)       \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
  // one iteration: multiply slice kt (LDS stage kt & 1); request slice kt+2 into set `ld`; store set `st` (kt+1)
  // REQ / PUT are compile-time so that the compiler can count the loads in flight exactly (a run-time condition
  // around the requests would force a wait for ALL loads before every LDS store)
#define HSD_G8_ITER(kt, ld, st, REQ, PUT)                                                             \
  {                                                                                                   \
    const uint16_t *sp = smem + ((kt) & 1) * Cfg::kStage;                                             \
    const int kbyte = ((kt) + 2) * BK * 2;                                                            \
    bf16x8 fa[2][TM], fb[2][TN];                                                                      \
    HSD_G8_FRAG(0, 0)                                                                                 \
    if (REQ) { HSD_G8_LOAD(ld, 0, kbyte) HSD_G8_LOAD(ld, 1, kbyte) }                                  \
    HSD_G8_FRAG(1, 1)                                                                                 \
    HSD_G8_MMA(0)                                                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    if (REQ) { HSD_G8_LOAD(ld, 2, kbyte) HSD_G8_LOAD(ld, 3, kbyte) }                                  \
    HSD_G8_FRAG(0, 2)                                                                                 \
    HSD_G8_MMA(1)                                                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    if (PUT) HSD_G8_STORE(st, ((kt) + 1) & 1, 0, 2)                                                   \
    HSD_G8_FRAG(1, 3)                                                                                 \
    HSD_G8_MMA(0)                                                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    if (PUT) HSD_G8_STORE(st, ((kt) + 1) & 1, 2, 4)                                                   \
    HSD_G8_MMA(1)                                                                                     \
    __syncthreads();                                                                                  \
  }

  HSD_G8_LOAD(0, 0, 0) HSD_G8_LOAD(0, 1, 0) HSD_G8_LOAD(0, 2, 0) HSD_G8_LOAD(0, 3, 0)
  HSD_G8_LOAD(1, 0, BK * 2) HSD_G8_LOAD(1, 1, BK * 2) HSD_G8_LOAD(1, 2, BK * 2) HSD_G8_LOAD(1, 3, BK * 2)
  HSD_G8_STORE(0, 0, 0, 4)
  __syncthreads();
  // slice kt+1 lives in set (kt+1) & 1; requests for slice kt+2 reuse set kt & 1 (stored one iteration ago).
  // The host only launches this kernel with an even number (>= 4) of K slices: full iterations in pairs, then the
  // fixed two-iteration tail (keeping the control flow this simple keeps the kernel free of register spills)
  int kt = 0;
  for (; kt + 3 < nk; kt += 2) {
    HSD_G8_ITER(kt, 0, 1, true, true)
    HSD_G8_ITER(kt + 1, 1, 0, true, true)
  }
  HSD_G8_ITER(kt, 0, 1, false, true)
  HSD_G8_ITER(kt + 1, 1, 0, false, false)
  gemm_epilogue<Cfg, MODE>(acc, M, N, m0, n0, tw, wi, wj, lane, epi, reinterpret_cast<float *>(smem_raw));
#undef HSD_G8_LOAD
#undef HSD_G8_STORE
#undef HSD_G8_FRAG
#undef HSD_G8_MMA
#undef HSD_G8_ITER
}

}  // namespace hsd
