// bf16 MFMA GEMM for gfx950: C[m,n] = sum_k A[m,k] * W[n,k], fp32 accumulation, fused epilogues.
//
// Both operands are K-contiguous (activations [M,K], weights [N,K]), which is what the MFMA operand
// layout wants: lane l of v_mfma_f32_32x32x16_bf16 supplies 8 consecutive k of row (l % 32), k-group
// (l / 32).  A workgroup of WM x WN waves computes a BP x BQ tile; each wave a (BP/WM) x (BQ/WN) tile made
// of 32x32 MFMA tiles.  K is consumed in slices of BK staged through LDS (rows padded by 16 bytes so that
// the 128-bit operand reads of 8 consecutive lanes cover all banks), double buffered: the global loads of
// slice k+1 are issued before the MFMAs of slice k and written to the other LDS stage after them.
//
// The kernel is written on two K-contiguous matrices P (MFMA "i" side) and Q ("j" side).  In the 32x32
// result tile, lane l holds column j = l % 32 and rows i = 8*(v/4) + 4*(l/32) + v%4 for register v.
//  - normal mode  (P = activations, Q = weights): a lane owns one output column and many rows; two adjacent
//    N sub-tiles of a wave are columns n and n+32 of the same head -> rotary pairs stay in one lane.
//  - swapped mode (P = weights, Q = activations): a lane owns one token and many vocabulary entries, so
//    the LM-head arg-max folds in registers with no cross-lane traffic.
//  - dual mode: the Q tile alternates 32 gate rows and 32 up rows, so gate and up of the same output
//    element sit in the same lane and register index of adjacent sub-tiles (SwiGLU in place).
//
// Workgroups are numbered so that the 8 XCDs (round-robin over workgroup ids) each walk a contiguous
// range of tiles: activation tile fastest while the weights are the larger operand (consecutive tiles on one XCD
// share the weight tile in its L2), weight tile fastest for passes over many rows (see gemm_tile_of).
#pragma once

#include "common.h"
#include "epilogues.h"

namespace hsd {


enum GemmMode { kModeNormal = 0, kModeDual = 1, kModeSwapLM = 2 };

template <int BP_, int BQ_, int BK_, int WM_, int WN_>
struct GemmCfg {
  static constexpr int BP = BP_, BQ = BQ_, BK = BK_, WM = WM_, WN = WN_;
  static constexpr int kThreads = 64 * WM * WN;
  static constexpr int TM = BP / WM / 32, TN = BQ / WN / 32;  // 32x32 MFMA tiles per wave
  static constexpr int kStride = BK + 8;                      // bf16 elements per LDS row
  static constexpr int kStage = (BP + BQ) * kStride;          // bf16 elements per stage
  static constexpr int kSmemBytes = 2 * kStage * 2;            // operand stages; kRowScaleBytes more follow them
  static constexpr int kChunks = BK / 8;                      // 16-byte chunks per tile row
  static constexpr int kLoadsP = BP * kChunks / kThreads, kLoadsQ = BQ * kChunks / kThreads;
  static constexpr int kEpiStride = TN * 32 + 4;              // floats per row of a wave's epilogue staging region
  static_assert(WM * WN * 32 * kEpiStride * 4 <= kSmemBytes, "epilogue staging must fit in the operand stages");
  static_assert(BP % (WM * 32) == 0 && BQ % (WN * 64) == 0, "wave tile must be made of 32-row / 64-col groups");
  static_assert(BP * kChunks % kThreads == 0 && BQ * kChunks % kThreads == 0, "tile loads must divide evenly");
};

__device__ __forceinline__ void xcd_tile(int pid, int tiles_fast, int n_tiles, int &t_fast, int &t_slow) {
  int full = (n_tiles / 8) * 8;
  int p = pid;
  if (pid < full) p = (pid % 8) * (full / 8) + pid / 8;
  t_fast = p % tiles_fast;
  t_slow = p / tiles_fast;
}

// Workgroup -> (activation tile, weight tile).  Workgroups go to the 8 XCDs round robin; xcd_tile gives each XCD
// a contiguous run of the tile order, so the operand whose tile index is the SLOW one is fetched into one L2 only,
// the other into all of them.  With few rows the weights are the big operand (each XCD takes a few weight tiles and
// every activation tile); with many rows it is the activations (each XCD takes a band of rows and every weight
// tile).  `w_rows` = rows of the weight matrix.
__device__ __forceinline__ void gemm_tile_of(int pid, int M, int w_rows, int tiles_act, int tiles_w, int &ta, int &tw) {
  if (M >= 4 * w_rows) xcd_tile(pid, tiles_w, tiles_act * tiles_w, tw, ta);
  else xcd_tile(pid, tiles_act, tiles_act * tiles_w, ta, tw);
}

// Tile counts for (M, N) in a mode: activation tiles first, weight tiles second.
template <typename Cfg, int MODE>
__host__ __device__ inline void gemm_tiles(int M, int N, int &tiles_act, int &tiles_w) {
  if (MODE == kModeSwapLM) {
    tiles_act = (M + Cfg::BQ - 1) / Cfg::BQ;
    tiles_w = (N + Cfg::BP - 1) / Cfg::BP;
  } else if (MODE == kModeDual) {
    tiles_act = (M + Cfg::BP - 1) / Cfg::BP;
    tiles_w = (2 * N + Cfg::BQ - 1) / Cfg::BQ;
  } else {
    tiles_act = (M + Cfg::BP - 1) / Cfg::BP;
    tiles_w = (N + Cfg::BQ - 1) / Cfg::BQ;
  }
}

// Row scales (the rstd of a folded RMSNorm, see RowScale) of a tile's activation rows live in LDS behind the operand
// stages: computed once per workgroup while the first K slices are on their way, read by the epilogue.
constexpr int kRowScaleBytes = 256 * 4;   // up to 256 activation rows per tile

template <typename Cfg, int MODE, typename Epi>
__device__ __forceinline__ void gemm_row_scales(const Epi &epi, int M, int m0, int t, int n_threads,
                                                unsigned char *smem_raw) {
  if constexpr (Epi::kRowScale) {
    constexpr int ROWS = (MODE == kModeSwapLM) ? Cfg::BQ : Cfg::BP;
    static_assert(ROWS * 4 <= kRowScaleBytes, "row scales must fit their LDS region");
    float *rsl = reinterpret_cast<float *>(smem_raw + Cfg::kSmemBytes);
    for (int r = t; r < ROWS; r += n_threads) rsl[r] = (m0 + r < M) ? epi.rs.at(m0 + r) : 1.0f;
  }
}

// Hands the accumulators of one wave to the epilogue functor (see the mode descriptions above).  A barrier must lie
// between gemm_row_scales and this call (every K loop has one).
template <typename Cfg, int MODE, typename Epi>
__device__ __forceinline__ void gemm_epilogue(floatx16 (&acc)[Cfg::TM][Cfg::TN], int M, int N, int m0, int n0, int tw,
                                              int wi, int wj, int lane, const Epi &epi, float *stage) {
  const float *rsl = reinterpret_cast<const float *>(reinterpret_cast<const unsigned char *>(stage) + Cfg::kSmemBytes);
  constexpr int BP = Cfg::BP, BQ = Cfg::BQ, TM = Cfg::TM, TN = Cfg::TN;
  const int col = lane & 31, half = lane >> 5;
  if constexpr (MODE == kModeSwapLM) {
    // i side = vocabulary rows, j side = tokens: fold the lane's TM*16 values per token, merge the lane halves
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int m = m0 + wj * (BQ / Cfg::WN) + j * 32 + col;
      if (epi.rs.ss != nullptr && m < M) {   // fold in the row's rstd before anything looks at the logits
        const float rsc = rsl[wj * (BQ / Cfg::WN) + j * 32 + col];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[i][j][v] *= rsc;
      }
      Top2 tp = top2_init();
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int n = n0 + wi * (BP / Cfg::WM) + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
          top2_push(tp, acc[i][j][v], n);
        }
      if (epi.want_logit != nullptr && m < M) {
        // this lane holds row m's logits at ids nb + 32*i + 8*(v/4) + 4*half + v%4, i < TM, v < 16
        const int nb = n0 + wi * (BP / Cfg::WM);
        epi.capture(m, [&](int want, float &out) {
          const int rel = want - nb;
          if (rel < 0 || rel >= TM * 32 || ((rel >> 2) & 1) != half) return false;
          const int i = rel >> 5, vv = ((rel & 31) >> 3) * 4 + (rel & 3);
          bool hit = false;
#pragma unroll
          for (int ii = 0; ii < TM; ++ii)
#pragma unroll
            for (int v = 0; v < 16; ++v)
              if (ii == i && v == vv) out = acc[ii][j][v], hit = true;
          return hit;
        });
      }
      if (epi.dump_slot != nullptr && m < M) {
        int sl = epi.dump_slot[m];
        if (sl >= 0) {
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              int n = n0 + wi * (BP / Cfg::WM) + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
              epi.logits_dump[static_cast<size_t>(sl) * epi.vocab + n] = acc[i][j][v];
            }
        }
      }
      Top2 other;
      other.m1 = __shfl_xor(tp.m1, 32, kWave);
      other.i1 = __shfl_xor(tp.i1, 32, kWave);
      other.m2 = __shfl_xor(tp.m2, 32, kWave);
      tp = top2_merge(tp, other);
      if (half == 0 && m < M) epi.part[static_cast<size_t>(m) * epi.n_tiles + tw * Cfg::WM + wi] = tp;
    }
  } else {
    // Accumulators go through LDS to turn the MFMA result layout (a lane owns one COLUMN of 16 scattered rows)
    // into row pieces of PC = Epi::kPiece columns: in every 64-column group of a 32-row sub-tile, the 32/PC lanes
    // l % (32/PC) of a row own columns PC*(l % (32/PC)) .. +PC-1 and their partners 32 further on (rotary pairs;
    // gate/up pairs in dual mode), so that adjacent lanes write adjacent 16-byte pieces of one row.  Each wave
    // uses a private region (32 rows of TN*32 + 4 floats); LDS executes a wave's accesses in program order, so
    // only the compiler has to be kept from reordering them (wave-scope fences).
    constexpr int ST = Cfg::kEpiStride, PC = Epi::kPiece, LPR = 32 / PC, RPI = 64 / LPR;  // lanes per row, rows per pass
    float *wst = stage + (wi * Cfg::WN + wj) * 32 * ST;
    const int pc = lane % LPR, pr = lane / LPR;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) wst[(8 * (v >> 2) + 4 * half + (v & 3)) * ST + j * 32 + col] = acc[i][j][v];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int it = 0; it < 32 / RPI; ++it) {
        const int r = it * RPI + pr;
        const int m = m0 + wi * (BP / Cfg::WM) + i * 32 + r;
        float rsc = 1.0f;
        if constexpr (Epi::kRowScale) rsc = rsl[wi * (BP / Cfg::WM) + i * 32 + r];
#pragma unroll
        for (int jg = 0; jg < TN / 2; ++jg) {
          float lo[PC], hi[PC];
          const float *src = wst + r * ST + jg * 64 + PC * pc;
#pragma unroll
          for (int q = 0; q < PC / 4; ++q) {
            const floatx4 a = *reinterpret_cast<const floatx4 *>(src + 4 * q);
            const floatx4 b = *reinterpret_cast<const floatx4 *>(src + 32 + 4 * q);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              lo[4 * q + e] = Epi::kRowScale ? a[e] * rsc : a[e];
              hi[4 * q + e] = Epi::kRowScale ? b[e] * rsc : b[e];
            }
          }
          if (m >= M) continue;
          if constexpr (MODE == kModeDual) {
            epi.piece_dual(m, n0 + wj * (BQ / Cfg::WN / 2) + jg * 32 + PC * pc, lo, hi);
          } else {
            const int n = n0 + wj * (BQ / Cfg::WN) + jg * 64 + PC * pc;
            if (n < N) epi.piece(m, n, lo, hi);
          }
        }
      }
    }
  }
}

// grid: 1-D, tiles_act * tiles_w workgroups of Cfg::kThreads threads, Cfg::kSmemBytes dynamic LDS.
// N is the number of output columns (for dual mode the weight matrix has 2N rows: gate | up).
template <typename Cfg, int MODE, typename Epi>
__global__ void __launch_bounds__(Cfg::kThreads) k_gemm_mfma(int M, int N, int K, const bf16 *__restrict__ A,
                                                             const bf16 *__restrict__ W, Epi epi) {
  constexpr int BP = Cfg::BP, BQ = Cfg::BQ, BK = Cfg::BK, TM = Cfg::TM, TN = Cfg::TN, LS = Cfg::kStride;
  constexpr int NT = Cfg::kThreads, CH = Cfg::kChunks;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  uint16_t *smem = reinterpret_cast<uint16_t *>(smem_raw);

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wi = wave / Cfg::WN, wj = wave % Cfg::WN;
  int tiles_act, tiles_w, ta, tw;
  gemm_tiles<Cfg, MODE>(M, N, tiles_act, tiles_w);
  gemm_tile_of(blockIdx.x, M, (MODE == kModeDual) ? 2 * N : N, tiles_act, tiles_w, ta, tw);
  // first activation row / first output column of this tile
  const int m0 = ta * ((MODE == kModeSwapLM) ? BQ : BP);
  const int n0 = tw * ((MODE == kModeSwapLM) ? BP : ((MODE == kModeDual) ? BQ / 2 : BQ));
  gemm_row_scales<Cfg, MODE>(epi, M, m0, t, NT, smem_raw);

  // ---- global source of every 16-byte chunk this thread stages (fixed over the K loop)
  const bf16 *srcP[Cfg::kLoadsP];
  const bf16 *srcQ[Cfg::kLoadsQ];
#pragma unroll
  for (int i = 0; i < Cfg::kLoadsP; ++i) {
    int c = t + NT * i, r = c / CH, kc = c % CH;
    int row = (MODE == kModeSwapLM) ? min(n0 + r, N - 1) : min(m0 + r, M - 1);
    srcP[i] = ((MODE == kModeSwapLM) ? W : A) + static_cast<size_t>(row) * K + kc * 8;
  }
#pragma unroll
  for (int i = 0; i < Cfg::kLoadsQ; ++i) {
    int c = t + NT * i, r = c / CH, kc = c % CH;
    int row;
    if (MODE == kModeSwapLM) {
      row = min(m0 + r, M - 1);
    } else if (MODE == kModeDual) {
      constexpr int WNC = BQ / Cfg::WN;  // Q rows per wave column
      int wq = r / WNC, tn = (r % WNC) >> 5, j = r & 31;
      row = min(((tn & 1) ? N : 0) + n0 + wq * (WNC / 2) + (tn >> 1) * 32 + j, 2 * N - 1);
    } else {
      row = min(n0 + r, N - 1);
    }
    srcQ[i] = ((MODE == kModeSwapLM) ? A : W) + static_cast<size_t>(row) * K + kc * 8;
  }

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int frag_p = (wi * (BP / Cfg::WM) + (lane & 31)) * LS + (lane >> 5) * 8;
  const int frag_q = BP * LS + (wj * (BQ / Cfg::WN) + (lane & 31)) * LS + (lane >> 5) * 8;

  // Two register sets hold the K slices in flight: while slice kt is multiplied out of LDS stage kt & 1, slice
  // kt+1 (requested one iteration earlier) is written from its set to the other stage, and the requests for slice
  // kt+2 go out into the set that was stored last iteration.  Loads and LDS stores are issued between the MFMA
  // groups of the four k-steps so that neither blocks a long MFMA run.
  u32x4 regP[2][Cfg::kLoadsP], regQ[2][Cfg::kLoadsQ];
  static_assert(BK == 64 && Cfg::kLoadsP % 2 == 0 && Cfg::kLoadsQ % 2 == 0, "pipeline is written for 4 k-steps");
  const int nk = K / BK;

#define HSD_GEMM_LOAD(set, k0, h)                                                                   \
  _Pragma("unroll") for (int i = (h) * (Cfg::kLoadsP / 2); i < ((h) + 1) * (Cfg::kLoadsP / 2); ++i) \
      regP[set][i] = *reinterpret_cast<const u32x4 *>(srcP[i] + (k0));                              \
  _Pragma("unroll") for (int i = (h) * (Cfg::kLoadsQ / 2); i < ((h) + 1) * (Cfg::kLoadsQ / 2); ++i) \
      regQ[set][i] = *reinterpret_cast<const u32x4 *>(srcQ[i] + (k0));
#define HSD_GEMM_STORE(set, stage, h)                                                               \
  {                                                                                                 \
    uint16_t *sd = smem + (stage) * Cfg::kStage;                                                    \
    _Pragma("unroll") for (int i = (h) * (Cfg::kLoadsP / 2); i < ((h) + 1) * (Cfg::kLoadsP / 2); ++i) { \
      int c = t + NT * i;                                                                           \
      *reinterpret_cast<u32x4 *>(sd + (c / CH) * LS + (c % CH) * 8) = regP[set][i];                 \
    }                                                                                               \
    _Pragma("unroll") for (int i = (h) * (Cfg::kLoadsQ / 2); i < ((h) + 1) * (Cfg::kLoadsQ / 2); ++i) { \
      int c = t + NT * i;                                                                           \
      *reinterpret_cast<u32x4 *>(sd + BP * LS + (c / CH) * LS + (c % CH) * 8) = regQ[set][i];       \
    }                                                                                               \
  }
#define HSD_GEMM_KSTEP(kk)                                                                          \
  {                                                                                                 \
    bf16x8 a[TM], b[TN];                                                                            \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) a[i] =                                           \
        *reinterpret_cast<const bf16x8 *>(sp + frag_p + i * 32 * LS + (kk) * 16);                   \
    _Pragma("unroll") for (int j = 0; j < TN; ++j) b[j] =                                           \
        *reinterpret_cast<const bf16x8 *>(sp + frag_q + j * 32 * LS + (kk) * 16);                   \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) _Pragma("unroll") for (int j = 0; j < TN; ++j)   \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);         \
  }
  // REQ / PUT are compile-time: a run-time condition around the loads would make the compiler count the loads
  // in flight for the path WITHOUT them, i.e. wait for everything before each LDS store, and the two-slice
  // look-ahead would collapse to none.  The loop below therefore peels the last two iterations.
#define HSD_GEMM_ITER(kt, ld, st, REQ, PUT)                                                         \
  {                                                                                                 \
    const uint16_t *sp = smem + ((kt) & 1) * Cfg::kStage;                                           \
    const int knext = ((kt) + 2) * BK;                                                              \
    if (REQ) { HSD_GEMM_LOAD(ld, knext, 0) }                                                        \
    HSD_GEMM_KSTEP(0)                                                                               \
    __builtin_amdgcn_sched_barrier(0);                                                              \
    if (REQ) { HSD_GEMM_LOAD(ld, knext, 1) }                                                        \
    HSD_GEMM_KSTEP(1)                                                                               \
    __builtin_amdgcn_sched_barrier(0);                                                              \
    if (PUT) HSD_GEMM_STORE(st, ((kt) + 1) & 1, 0)                                                  \
    HSD_GEMM_KSTEP(2)                                                                               \
    __builtin_amdgcn_sched_barrier(0);                                                              \
    if (PUT) HSD_GEMM_STORE(st, ((kt) + 1) & 1, 1)                                                  \
    HSD_GEMM_KSTEP(3)                                                                               \
    __syncthreads();                                                                                \
  }

  HSD_GEMM_LOAD(0, 0, 0) HSD_GEMM_LOAD(0, 0, 1)
  if (nk > 1) { HSD_GEMM_LOAD(1, BK, 0) HSD_GEMM_LOAD(1, BK, 1) }
  HSD_GEMM_STORE(0, 0, 0) HSD_GEMM_STORE(0, 0, 1)
  __syncthreads();
  // slice kt is in LDS stage kt & 1 and came through register set kt & 1; iteration kt requests slice kt+2
  // into set kt & 1 and stores set (kt+1) & 1.  Full iterations run while kt + 2 < nk.
  int kt = 0;
  for (; kt + 3 < nk; kt += 2) {
    HSD_GEMM_ITER(kt, 0, 1, true, true)
    HSD_GEMM_ITER(kt + 1, 1, 0, true, true)
  }
  if (kt + 2 < nk) {  // one more full iteration, then the two-iteration tail on swapped sets
    HSD_GEMM_ITER(kt, 0, 1, true, true)
    HSD_GEMM_ITER(kt + 1, 1, 0, false, true)
    HSD_GEMM_ITER(kt + 2, 0, 1, false, false)
  } else if (kt + 1 < nk) {
    HSD_GEMM_ITER(kt, 0, 1, false, true)
    HSD_GEMM_ITER(kt + 1, 1, 0, false, false)
  } else {
    HSD_GEMM_ITER(kt, 0, 1, false, false)
  }
#undef HSD_GEMM_LOAD
#undef HSD_GEMM_STORE
#undef HSD_GEMM_KSTEP
#undef HSD_GEMM_ITER
  gemm_epilogue<Cfg, MODE>(acc, M, N, m0, n0, tw, wi, wj, lane, epi, reinterpret_cast<float *>(smem_raw));
}

}  // namespace hsd
