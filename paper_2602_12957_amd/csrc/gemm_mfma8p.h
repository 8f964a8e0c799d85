// Persistent form of the 256x256 8-wave GEMM (k_gemm_mfma8) for launches of several rounds of tiles: a workgroup
// walks tiles pid, pid + grid, pid + 2 grid, ... and requests the first two K slices of its NEXT tile during the last
// two iterations of the current one, so that they travel while the epilogue runs instead of opening the next tile
// with an idle wait.  Same tile order per workgroup index (workgroup b stays on XCD b % 8 and grid is a multiple of
// 8, so a tile is computed on the XCD it would be launched on), same pipeline, same K order, same epilogue: results
// are bit-identical to k_gemm_mfma8.
#pragma once

#include "gemm_mfma8.h"

namespace hsd {

// grid: 1-D, a multiple of 8 workgroups (at most tiles_act * tiles_w) of 512 threads, GemmCfg8::kSmemBytes +
// kRowScaleBytes dynamic LDS.  K a multiple of 128 and at least 256; both matrices below 2 GiB.
template <int MODE, typename Epi>
__global__ void __launch_bounds__(512) k_gemm_mfma8p(int M, int N, int K, const bf16 *__restrict__ A,
                                                     const bf16 *__restrict__ W, Epi epi) {
  using Cfg = GemmCfg8;
  constexpr int BP = Cfg::BP, BQ = Cfg::BQ, BK = Cfg::BK, TM = Cfg::TM, TN = Cfg::TN, LS = Cfg::kStride;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  uint16_t *smem = reinterpret_cast<uint16_t *>(smem_raw);

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wi = wave / Cfg::WN, wj = wave % Cfg::WN;
  int tiles_act, tiles_w;
  gemm_tiles<Cfg, MODE>(M, N, tiles_act, tiles_w);
  const int n_tiles = tiles_act * tiles_w;
  const int w_rows_i = (MODE == kModeDual) ? 2 * N : N;

  const int r8 = t >> 3, kc = t & 7;
  const __amdgpu_buffer_rsrc_t rs_act = make_rsrc(A, static_cast<size_t>(M) * K * 2);
  const __amdgpu_buffer_rsrc_t rs_w = make_rsrc(W, static_cast<size_t>(w_rows_i) * K * 2);
  const __amdgpu_buffer_rsrc_t rs_p = (MODE == kModeSwapLM) ? rs_w : rs_act;
  const __amdgpu_buffer_rsrc_t rs_q = (MODE == kModeSwapLM) ? rs_act : rs_w;
  const int p_step = 64 * K * 2;
  const int q_step = (MODE == kModeDual ? 32 : 64) * K * 2;
  const int lds_dst = r8 * LS + kc * 8;   // + i * 64 * LS

  // first row / first column and the thread's operand offsets (as in k_gemm_mfma8) of tile `pid`
  auto tile_of = [&](int pid, int &m0, int &n0, int &tw, int &vp, int &vq) {
    int ta;
    gemm_tile_of(pid, M, w_rows_i, tiles_act, tiles_w, ta, tw);
    m0 = ta * ((MODE == kModeSwapLM) ? BQ : BP);
    n0 = tw * ((MODE == kModeSwapLM) ? BP : ((MODE == kModeDual) ? BQ / 2 : BQ));
    vp = ((((MODE == kModeSwapLM) ? n0 : m0) + r8) * K + kc * 8) * 2;
    if (MODE == kModeSwapLM) vq = ((m0 + r8) * K + kc * 8) * 2;
    else if (MODE == kModeDual) vq = ((((r8 >> 5) ? N : 0) + n0 + (r8 & 31)) * K + kc * 8) * 2;
    else vq = ((n0 + r8) * K + kc * 8) * 2;
  };

  const int frag_p = (wi * (BP / Cfg::WM) + (lane & 31)) * LS + (lane >> 5) * 8;
  const int frag_q = BP * LS + (wj * (BQ / Cfg::WN) + (lane & 31)) * LS + (lane >> 5) * 8;
  u32x4 regP[2][4], regQ[2][4];
  const int nk = K / BK;

#define HSD_G8P_LOAD(set, i, vp, vq, kbyte)                                                           \
  regP[set][i] = __builtin_amdgcn_raw_buffer_load_b128(rs_p, (vp) + (i) * p_step, (kbyte), 0);        \
  regQ[set][i] = __builtin_amdgcn_raw_buffer_load_b128(rs_q, (vq) + (i) * q_step, (kbyte), 0);
#define HSD_G8P_STORE(set, stage, i0, i1)                                                             \
  {                                                                                                   \
    uint16_t *sd = smem + (stage) * Cfg::kStage;                                                      \
    _Pragma("unroll") for (int i = (i0); i < (i1); ++i) {                                             \
      *reinterpret_cast<u32x4 *>(sd + lds_dst + i * 64 * LS) = regP[set][i];                          \
      *reinterpret_cast<u32x4 *>(sd + BP * LS + lds_dst + i * 64 * LS) = regQ[set][i];                \
    }                                                                                                 \
  }
#define HSD_G8P_FRAG(buf, kk)                                                                         \
  _Pragma("unroll") for (int i = 0; i < TM; ++i) fa[buf][i] =                                         \
      *reinterpret_cast<const bf16x8 *>(sp + frag_p + i * 32 * LS + (kk) * 16);                       \
  _Pragma("unroll") for (int j = 0; j < TN; ++j) fb[buf][j] =                                         \
      *reinterpret_cast<const bf16x8 *>(sp + frag_q + j * 32 * LS + (kk) * 16);
#define HSD_G8P_MMA(buf)                                                                              \
  _Pragma("unroll") for (int i = 0; i < TM; ++i) _Pragma("unroll") for (int j = 0; j < TN; ++j)       \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
  // one iteration: multiply slice kt (LDS stage kt & 1); request into set `ld` the slice at (vp, vq, kbyte); store
  // set `st` (slice kt+1) if PUT
#define HSD_G8P_ITER(kt, ld, st, vp, vq, kbyte, PUT)                                                  \
  {                                                                                                   \
    const uint16_t *sp = smem + ((kt) & 1) * Cfg::kStage;                                             \
    bf16x8 fa[2][TM], fb[2][TN];                                                                      \
    HSD_G8P_FRAG(0, 0)                                                                                \
    HSD_G8P_LOAD(ld, 0, vp, vq, kbyte) HSD_G8P_LOAD(ld, 1, vp, vq, kbyte)                             \
    HSD_G8P_FRAG(1, 1)                                                                                \
    HSD_G8P_MMA(0)                                                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    HSD_G8P_LOAD(ld, 2, vp, vq, kbyte) HSD_G8P_LOAD(ld, 3, vp, vq, kbyte)                             \
    HSD_G8P_FRAG(0, 2)                                                                                \
    HSD_G8P_MMA(1)                                                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    if (PUT) HSD_G8P_STORE(st, ((kt) + 1) & 1, 0, 2)                                                  \
    HSD_G8P_FRAG(1, 3)                                                                                \
    HSD_G8P_MMA(0)                                                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    if (PUT) HSD_G8P_STORE(st, ((kt) + 1) & 1, 2, 4)                                                  \
    HSD_G8P_MMA(1)                                                                                    \
    __syncthreads();                                                                                  \
  }

  int pid = blockIdx.x;
  int m0, n0, tw, voff_p, voff_q;
  tile_of(pid, m0, n0, tw, voff_p, voff_q);
  HSD_G8P_LOAD(0, 0, voff_p, voff_q, 0) HSD_G8P_LOAD(0, 1, voff_p, voff_q, 0)
  HSD_G8P_LOAD(0, 2, voff_p, voff_q, 0) HSD_G8P_LOAD(0, 3, voff_p, voff_q, 0)
  HSD_G8P_LOAD(1, 0, voff_p, voff_q, BK * 2) HSD_G8P_LOAD(1, 1, voff_p, voff_q, BK * 2)
  HSD_G8P_LOAD(1, 2, voff_p, voff_q, BK * 2) HSD_G8P_LOAD(1, 3, voff_p, voff_q, BK * 2)
  for (;;) {
    // sets 0 and 1 hold (or are about to receive) slices 0 and 1 of tile `pid`
    gemm_row_scales<Cfg, MODE>(epi, M, m0, t, 512, smem_raw);
    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    HSD_G8P_STORE(0, 0, 0, 4)
    __syncthreads();
    // the tile after this one (the last tile requests its own first slices once more: loads that nobody uses, so
    // that the number of loads in flight never depends on a run-time condition)
    const int next = pid + static_cast<int>(gridDim.x);
    const bool has_next = next < n_tiles;
    int m0n, n0n, twn, vpn, vqn;
    tile_of(has_next ? next : pid, m0n, n0n, twn, vpn, vqn);
    int kt = 0;
    for (; kt + 3 < nk; kt += 2) {
      HSD_G8P_ITER(kt, 0, 1, voff_p, voff_q, (kt + 2) * BK * 2, true)
      HSD_G8P_ITER(kt + 1, 1, 0, voff_p, voff_q, (kt + 3) * BK * 2, true)
    }
    HSD_G8P_ITER(kt, 0, 1, vpn, vqn, 0, true)
    HSD_G8P_ITER(kt + 1, 1, 0, vpn, vqn, BK * 2, false)
    gemm_epilogue<Cfg, MODE>(acc, M, N, m0, n0, tw, wi, wj, lane, epi,
                             reinterpret_cast<float *>(smem_raw));
    if (!has_next) break;
    pid = next;
    m0 = m0n, n0 = n0n, tw = twn, voff_p = vpn, voff_q = vqn;
    __syncthreads();   // the epilogue staged through the LDS the next tile's first slice is about to be written to
  }
#undef HSD_G8P_LOAD
#undef HSD_G8P_STORE
#undef HSD_G8P_FRAG
#undef HSD_G8P_MMA
#undef HSD_G8P_ITER
}

}  // namespace hsd
