// bf16 MFMA GEMM for the narrow projections (QKV, O, down) at a few thousand rows: small tiles, four multiplying
// waves and a fifth wave that does nothing but request operands, which the loads write straight into LDS.
//
// Why.  With ~2 k rows these projections have only a few hundred tiles of 64x128 or 128x128, about one workgroup per
// compute unit, each walking 16 to 64 K slices.  Measured on such a workgroup (one K slice of a 64x128 tile): the
// compute unit's load path takes in 64 bytes per cycle, so the 24 KB of a slice occupy it for ~380 cycles and a wave
// that issues the loads sits in the issue stall for that long; the 12 fragment reads and 8 MFMAs of a multiplying wave
// take ~390 cycles.  Waves that do both, in step with each other from barrier to barrier, pay the sum (0.36 us a
// slice in every arrangement tried: loads to registers and LDS stores by the multiplying waves, by four moving waves,
// LDS-direct loads issued by the multiplying waves in one batch or between the MFMAs).  Here the two run side by
// side: wave 4 issues `buffer_load_dwordx4 ... lds` (lane l's 16 bytes land at LDS address M0 + 16 l, so one
// instruction fills 8 tile rows of 64 bf16; no staging registers, no LDS store instructions, nothing to wait for
// but a counter) into a ring of stages, several slices ahead; waves 0-3 only read fragments and multiply.  Per slice
// every wave passes one barrier: behind it the next slice is complete in LDS and the oldest stage is free.
//
// The 16-byte pieces of a row are stored XOR-swizzled instead of padded (piece c of tile row r at position
// c ^ ((r >> 1) & 7)): the requesting lanes choose which global piece they fetch, the fragment reads apply the same
// XOR, and the 128-bit reads of 16 consecutive rows cover all 64 banks once.
//
// Operand roles, modes (normal, dual), K order per accumulator (ascending 16-wide steps) and the epilogue are those
// of gemm_mfma.h, so results are bit-identical to every other tile configuration.
#pragma once

#include "gemm_mfma.h"
#include "gemm_mfma8.h"

namespace hsd {

template <int BP_, int BQ_, int STAGES_, int LW_ = 1, int WM_ = 2, int WN_ = 2>
struct GemmCfgD : GemmCfg<BP_, BQ_, 64, WM_, WN_> {
  static constexpr int kStages = STAGES_;
  static constexpr int kLoaderWaves = LW_;                         // requesting waves: 1, 2 or 4
  static constexpr int kStageBytes = (BP_ + BQ_) * 64 * 2;         // P rows, then Q rows, 128 bytes each
  static constexpr int kSmemBytes = STAGES_ * kStageBytes;         // operand stages; kRowScaleBytes more follow them
  static constexpr int kLoads = (BP_ + BQ_) / 8;                   // load instructions per slice (8 rows each)
  static constexpr int kMulWaves = WM_ * WN_;                      // multiplying waves: 2 x 2, or 1 x 1 for tiny row counts
  static constexpr int kThreadsD = 64 * (WM_ * WN_ + LW_);         // the multiplying waves and the requesting ones
  static_assert((LW_ == 1 || LW_ == 2 || LW_ == 4) && ((BP_ + BQ_) / 8) % LW_ == 0, "requests divide evenly over the waves");
  static_assert((BP_ / 8) % LW_ == 0, "every request slot of a wave is all P or all Q");
  static_assert(STAGES_ >= 3 && STAGES_ <= 12, "a slice being multiplied, one complete behind it, one to nine in flight");
  static_assert(WM_ * WN_ * 32 * GemmCfg<BP_, BQ_, 64, WM_, WN_>::kEpiStride * 4 <= kSmemBytes, "epilogue staging must fit in the stages");
};

typedef __attribute__((address_space(3))) unsigned char *LdsBytePtr;

// One LDS-direct load: lane l's 16 bytes at buffer offset voff(l) + soff go to LDS address dst + 16 l (dst is wave
// uniform).  A plain function on purpose: called with template-dependent arguments the builtin itself makes the host
// pass drop the enclosing kernel's instantiation without a diagnostic.
__device__ __forceinline__ void lds_load16(__amdgpu_buffer_rsrc_t rs, LdsBytePtr dst, int voff, int soff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, dst, 16, voff, soff, 0, 0);
}

// s_waitcnt vmcnt(N) with the other counters left alone (N < 64)
#define HSD_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 15) | (7 << 4) | (15 << 8) | (((N) >> 4) << 14))

// grid: 1-D, tiles_act * tiles_w workgroups of Cfg::kThreadsD threads, Cfg::kSmemBytes + kRowScaleBytes dynamic LDS; the tiles
// cover rows m_base .. M-1 (a caller that gave the rows before m_base to another kernel passes their count, a
// multiple of the tile height; otherwise 0).
// K must be a multiple of 64; both matrices below 2 GiB (32-bit buffer offsets).
// Every wave executes exactly K/64 + 1 workgroup barriers, whichever role it has.
template <typename Cfg, int MODE, typename Epi>
__global__ void __launch_bounds__(Cfg::kThreadsD) k_gemm_mfma_d(int M, int N, int K, int m_base, const bf16 *__restrict__ A,
                                                     const bf16 *__restrict__ W, Epi epi) {
  static_assert(MODE == kModeNormal || MODE == kModeDual, "normal or dual mode");
  constexpr int BP = Cfg::BP, BQ = Cfg::BQ, BK = Cfg::BK, TM = Cfg::TM, TN = Cfg::TN, S = Cfg::kStages;
  constexpr int ROWB = BK * 2, LW = Cfg::kLoaderWaves, NL = Cfg::kLoads / LW;   // NL: requests per wave and slice
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  int tiles_act, tiles_w, ta, tw;
  gemm_tiles<Cfg, MODE>(M - m_base, N, tiles_act, tiles_w);
  gemm_tile_of(blockIdx.x, M - m_base, (MODE == kModeDual) ? 2 * N : N, tiles_act, tiles_w, ta, tw);
  const int m0 = m_base + ta * BP, n0 = tw * ((MODE == kModeDual) ? BQ / 2 : BQ);
  const int nk = K / BK;

  if (wave >= Cfg::kMulWaves) {
    // ---- a requesting wave.  Instruction i of a slice covers tile rows 8 i .. 8 i + 7 (P rows, then Q rows); lane l
    // fetches, for row 8 i + l / 8, the piece that belongs at position l & 7.  Rows past the end of a matrix re-read
    // its last row (their products are never stored).  With LW requesting waves, wave w takes the instructions
    // i = w, w + LW, ...: each wave's loads return in order, so several waves are several independent streams.
    const int lw = wave - Cfg::kMulWaves;
    const LdsBytePtr lds = (LdsBytePtr)smem_raw;
    const int w_rows = (MODE == kModeDual) ? 2 * N : N;
    const __amdgpu_buffer_rsrc_t rs_p = make_rsrc(A, static_cast<size_t>(M) * K * 2);
    const __amdgpu_buffer_rsrc_t rs_q = make_rsrc(W, static_cast<size_t>(w_rows) * K * 2);
    int voff[NL];
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const int i = j * LW + lw;
      const int r = (i < BP / 8 ? 8 * i : 8 * i - BP) + (lane >> 3);   // row of the P or of the Q tile
      const int kc = (lane & 7) ^ ((r >> 1) & 7);
      int row;
      if (i < BP / 8) {
        row = min(m0 + r, M - 1);
      } else if (MODE == kModeDual) {
        // Q row r: wave column r / WNC, 32-row sub-tile (r % WNC) / 32 (even: gate, odd: up), lane row r % 32
        constexpr int WNC = BQ / Cfg::WN;
        const int wq = r / WNC, tn = (r % WNC) >> 5;
        row = min(((tn & 1) ? N : 0) + n0 + wq * (WNC / 2) + (tn >> 1) * 32 + (r & 31), 2 * N - 1);
      } else {
        row = min(n0 + r, N - 1);
      }
      voff[j] = (row * K + kc * 8) * 2;
    }
#define HSD_GD_ISSUE(stage, slice)                                                                   \
  {                                                                                                  \
    const int kbyte = (slice) * BK * 2;                                                              \
    const LdsBytePtr dst = lds + (stage) * Cfg::kStageBytes;                                         \
    _Pragma("unroll") for (int j = 0; j < NL; ++j)                                                   \
        lds_load16(j < BP / 8 / LW ? rs_p : rs_q, dst + (j * LW + lw) * 1024, voff[j], kbyte);      \
  }
    // Wait until all but the `n_ahead` most recent slices have landed (the counter holds 63 loads at most: asking
    // for more to stay in flight than it can count only waits for a few loads more than necessary)
#define HSD_GD_WAIT_CASE(n) case n: HSD_VMCNT((n) * NL < 63 ? (n) * NL : 63); break;
#define HSD_GD_WAIT(n_ahead)                                                                         \
  switch (n_ahead) {                                                                                 \
    HSD_GD_WAIT_CASE(0) HSD_GD_WAIT_CASE(1) HSD_GD_WAIT_CASE(2) HSD_GD_WAIT_CASE(3) HSD_GD_WAIT_CASE(4)  \
    HSD_GD_WAIT_CASE(5) HSD_GD_WAIT_CASE(6) HSD_GD_WAIT_CASE(7) HSD_GD_WAIT_CASE(8)                  \
    default: HSD_VMCNT(9 * NL < 63 ? 9 * NL : 63); break;                                            \
  }
#pragma unroll
    for (int s = 0; s < S - 1; ++s)
      if (s < nk) HSD_GD_ISSUE(s, s)
    int st_free = S - 1;   // stage of slice kt - 1, free once everyone is past barrier kt
    for (int kt = 0; kt < nk; ++kt) {
      // behind barrier kt the multiplying waves read slice kt and the first fragments of slice kt+1: both must have
      // landed; slices kt+2 .. kt+S-2 (requested so far) may stay in flight
      const int left = nk - 2 - kt;   // slices after kt+1
      const int ahead = left < 0 ? 0 : (left < S - 3 ? left : S - 3);
      HSD_GD_WAIT(ahead)
      __builtin_amdgcn_s_barrier();
      if (kt + S - 1 < nk) HSD_GD_ISSUE(st_free, kt + S - 1)
      st_free = st_free + 1 == S ? 0 : st_free + 1;
    }
    __builtin_amdgcn_s_barrier();   // every load has landed (the last wait was for all of them)
#undef HSD_GD_ISSUE
#undef HSD_GD_WAIT
#undef HSD_GD_WAIT_CASE
    return;
  }

  // ---- the multiplying waves
  const int wi = wave / Cfg::WN, wj = wave % Cfg::WN;
  gemm_row_scales<Cfg, MODE>(epi, M, m0, t, 64 * Cfg::kMulWaves, smem_raw);
  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // fragment addresses: row (lane & 31) of a 32-row sub-tile, logical piece 2 kk + lane / 32, swizzled
  const int fr = lane & 31, sw = (fr >> 1) & 7, kg = lane >> 5;
  int off_p[4], off_q[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const int phys = ((2 * kk + kg) ^ sw) * 16;
    off_p[kk] = (wi * (BP / Cfg::WM) + fr) * ROWB + phys;
    off_q[kk] = BP * ROWB + (wj * (BQ / Cfg::WN) + fr) * ROWB + phys;
  }

  // Operand fragments are double buffered in registers: the LDS reads of k-step kk+1 (for the last step: of the next
  // slice's first step, which is complete behind the same barrier) are issued before the MFMAs of k-step kk.
  bf16x8 fa[2][TM], fb[2][TN];
#define HSD_GD_FRAG(buf, sp, kk)                                                                     \
  _Pragma("unroll") for (int i = 0; i < TM; ++i) fa[buf][i] =                                        \
      *reinterpret_cast<const bf16x8 *>(sp + off_p[kk] + i * 32 * ROWB);                             \
  _Pragma("unroll") for (int j = 0; j < TN; ++j) fb[buf][j] =                                        \
      *reinterpret_cast<const bf16x8 *>(sp + off_q[kk] + j * 32 * ROWB);
#define HSD_GD_MMA(buf)                                                                              \
  _Pragma("unroll") for (int i = 0; i < TM; ++i) _Pragma("unroll") for (int j = 0; j < TN; ++j)      \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
  __builtin_amdgcn_s_barrier();   // barrier 0: slices 0 and 1 are complete
  __builtin_amdgcn_sched_barrier(0);
  HSD_GD_FRAG(0, smem_raw, 0)
  int st = 0;   // stage of slice kt
  for (int kt = 0; kt < nk; ++kt) {
    if (kt > 0) {
      __builtin_amdgcn_s_barrier();   // barrier kt
      __builtin_amdgcn_sched_barrier(0);
    }
    const int st1 = st + 1 == S ? 0 : st + 1;
    const unsigned char *sp = smem_raw + st * Cfg::kStageBytes;
    const unsigned char *spn = smem_raw + st1 * Cfg::kStageBytes;
    HSD_GD_FRAG(1, sp, 1)
    HSD_GD_MMA(0)
    __builtin_amdgcn_sched_barrier(0);
    HSD_GD_FRAG(0, sp, 2)
    HSD_GD_MMA(1)
    __builtin_amdgcn_sched_barrier(0);
    HSD_GD_FRAG(1, sp, 3)
    HSD_GD_MMA(0)
    __builtin_amdgcn_sched_barrier(0);
    if (kt + 1 < nk) { HSD_GD_FRAG(0, spn, 0) }
    HSD_GD_MMA(1)
    __builtin_amdgcn_sched_barrier(0);
    st = st1;
  }
#undef HSD_GD_FRAG
#undef HSD_GD_MMA
  __builtin_amdgcn_s_barrier();   // the epilogue stages through the operand stages
  gemm_epilogue<Cfg, MODE>(acc, M, N, m0, n0, tw, wi, wj, lane, epi,
                           reinterpret_cast<float *>(smem_raw));
}

}  // namespace hsd
