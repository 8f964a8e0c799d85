// C ABI of the HSD verification hot path: argument validation, workspace carving, launch sequencing.
// All device work is enqueued on the caller's stream; nothing here synchronises or allocates device memory.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <type_traits>
#include <vector>

#include "../../include/hsd.h"
#include "attn_mfma.h"
#include "attn_simple.h"
#include "common.h"
#include "epilogues.h"
#include "gemm_mfma.h"
#include "gemm_mfma8.h"
#include "gemm_mfma8p.h"
#include "gemm_mfma_ws.h"
#include "gemm_mfma_d.h"
#include "probes.h"
#include "gemm_simple.h"
#include "misc_kernels.h"

using namespace hsd;

// Scratch for hsd_verify_region_batch_noalloc: the workspace of a verify call lives in this file-scope device array
// instead of caller memory.  Every GPU the library runs on holds its own copy until the process ends; host code never
// uses the array's name as an address, only the pointer hipGetSymbolAddress returns for the current device.
constexpr size_t kStaticWsBytes = size_t{16} << 20;
static __device__ __align__(256) unsigned char g_static_ws[kStaticWsBytes];

struct hsd_ctx {
  hsd_model_desc desc;
  void *static_ws = nullptr;  // device address of g_static_ws on the context's device
  const void *tok_embed;
  const float *final_norm;
  const void *lm_head;
  std::vector<const float *> attn_norm, ffn_norm;
  std::vector<const void *> wqkv, wo, w_gate_up, w_down;
  int n_cu;
  // hsd_debug_set knobs (defaults are what production runs use)
  bool sync_layers = false;  // wait for the stream after every layer (bounds the launches in flight for tools that
                             // track each dispatch; never set in timed runs)
  bool force_simple;  // run the plain kernels also for bf16 (cross-check of the MFMA path)
  bool gemm_cfg_forced = false;  // a tile configuration was set by hand: use it for every row count
  int gemm_cfg[5];    // tile configuration of the MFMA GEMM per call site (qkv, o, gate_up, down, lm_head)
  // per-kernel timing (hsd_profile_*)
  int prof_which = HSD_PROF_NONE;
  int prof_used = 0;
  std::vector<hipEvent_t> prof_events;  // 2 per timed launch
};

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Workspace {
  float *x;
  void *h, *q, *a, *u;
  int32_t *row_seq, *row_pos, *row_kv, *row_slot, *row_base, *row_end, *row_par, *dump_slot;
  AttnTile *attn_tiles;
  float *want_logit, *row_max;
  float2 *rope_cs;
  Top2 *lm_part;
  float *ss;    // [T][d_model / 64] sums of squares of the residual rows, in 64-column pieces (see RowScale)
  float *attn_part_o;    // key-split attention: un-normalised partial rows and their (reference point, sum)
  float2 *attn_part_ml;
  size_t total;
};

// Carves the workspace; with base == nullptr only the size is computed.
Workspace carve(const hsd_model_desc &d, int64_t T, int64_t n_seq, void *base) {
  const size_t es = d.dtype == HSD_BF16 ? 2 : 4;
  const size_t qdim = static_cast<size_t>(d.n_q_heads) * d.head_dim;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += align_up(bytes);
    return base ? static_cast<char *>(base) + o : nullptr;
  };
  Workspace w;
  w.x = reinterpret_cast<float *>(take(T * d.d_model * sizeof(float)));
  w.h = take(T * d.d_model * es);
  w.q = take(T * qdim * es);
  w.a = take(T * qdim * es);
  w.u = take(T * d.d_ffn * es);
  w.row_seq = reinterpret_cast<int32_t *>(take(T * sizeof(int32_t)));
  w.row_pos = reinterpret_cast<int32_t *>(take(T * sizeof(int32_t)));
  w.row_kv = reinterpret_cast<int32_t *>(take(T * sizeof(int32_t)));
  w.row_slot = reinterpret_cast<int32_t *>(take(T * sizeof(int32_t)));
  w.row_base = reinterpret_cast<int32_t *>(take(T * sizeof(int32_t)));
  w.row_end = reinterpret_cast<int32_t *>(take(T * sizeof(int32_t)));
  w.row_par = reinterpret_cast<int32_t *>(take(T * sizeof(int32_t)));
  w.want_logit = reinterpret_cast<float *>(take(T * sizeof(float)));
  w.row_max = reinterpret_cast<float *>(take(T * sizeof(float)));
  w.dump_slot = reinterpret_cast<int32_t *>(take(T * sizeof(int32_t)));
  // the largest task table any attention launch over T rows can need (32-row tiles, one head group per kv head)
  w.attn_tiles = reinterpret_cast<AttnTile *>(take(static_cast<size_t>(attn_grid_size(static_cast<int>(T / 32 + n_seq), d.n_q_heads, 8)) * sizeof(AttnTile)));
  w.rope_cs = reinterpret_cast<float2 *>(take(T * 32 * sizeof(float2)));
  w.lm_part = reinterpret_cast<Top2 *>(take(T * (d.vocab / 64) * sizeof(Top2)));
  w.ss = reinterpret_cast<float *>(take(T * (d.d_model / 64) * sizeof(float)));
  const size_t split_rh = (d.dtype == HSD_BF16 && d.attn_key_chunk > 0) ? kAttnMaxChunks * T * d.n_q_heads : 0;
  w.attn_part_o = reinterpret_cast<float *>(take(split_rh * d.head_dim * sizeof(float)));
  w.attn_part_ml = reinterpret_cast<float2 *>(take(split_rh * sizeof(float2)));
  w.total = off;
  return w;
}

#define HSD_LAUNCH_CHECK()                         \
  do {                                             \
    if (hipGetLastError() != hipSuccess) return HSD_EHIP; \
  } while (0)

// Brackets one launch with events when its class is being timed.
struct ProfScope {
  hsd_ctx *ctx;
  hipStream_t st;
  bool on;
  ProfScope(hsd_ctx *c, hipStream_t s, int which) : ctx(c), st(s) {
    on = c->prof_which == which && which != HSD_PROF_NONE &&
         static_cast<size_t>(2 * c->prof_used + 1) < c->prof_events.size();
    if (on) (void)hipEventRecord(c->prof_events[2 * c->prof_used], st);
  }
  ~ProfScope() {
    if (on) {
      (void)hipEventRecord(ctx->prof_events[2 * ctx->prof_used + 1], st);
      ctx->prof_used++;
    }
  }
};

enum { kSiteQKV = 0, kSiteO = 1, kSiteGateUp = 2, kSiteDown = 3, kSiteLM = 4 };

template <typename Epi>
struct GemmModeOf {
  static constexpr int value = Epi::kDual ? kModeDual : (std::is_same<Epi, EpiLMHead>::value ? kModeSwapLM : kModeNormal);
};

template <typename Cfg, typename Epi>
int launch_gemm_mfma(hipStream_t st, int M, int N, int K, const void *A, const void *W, Epi epi) {
  constexpr int MODE = GemmModeOf<Epi>::value;
  auto kern = k_gemm_mfma<Cfg, MODE, Epi>;
  constexpr int smem = Cfg::kSmemBytes + kRowScaleBytes;
  // set once per instantiation (initialisation of a function-local static is thread safe)
  static const hipError_t attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (attr_rc != hipSuccess) return HSD_EHIP;
  if constexpr (MODE == kModeSwapLM) epi.n_tiles = (N / Cfg::BP) * Cfg::WM;
  int tiles_act, tiles_w;
  gemm_tiles<Cfg, MODE>(M, N, tiles_act, tiles_w);
  hipLaunchKernelGGL(kern, dim3(tiles_act * tiles_w), dim3(Cfg::kThreads), smem, st, M, N, K,
                     static_cast<const bf16 *>(A), static_cast<const bf16 *>(W), epi);
  HSD_LAUNCH_CHECK();
  return HSD_OK;
}

template <typename Epi>
int launch_gemm_mfma8(hipStream_t st, int M, int N, int K, const void *A, const void *W, Epi epi, int n_cu) {
  constexpr int MODE = GemmModeOf<Epi>::value;
  using Cfg = GemmCfg8;
  auto kern = k_gemm_mfma8<MODE, Epi>;
  constexpr int smem = Cfg::kSmemBytes + kRowScaleBytes;
  static const hipError_t attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (attr_rc != hipSuccess) return HSD_EHIP;
  if constexpr (MODE == kModeSwapLM) epi.n_tiles = (N / Cfg::BP) * Cfg::WM;
  int tiles_act, tiles_w;
  gemm_tiles<Cfg, MODE>(M, N, tiles_act, tiles_w);
  // A launch of several rounds of tiles goes to the persistent form: one workgroup per compute unit (a multiple of
  // 8, so that tiles stay on the XCD the tile order gives them) walks its tiles and requests the next tile's first
  // K slices while the epilogue of the current one runs.  Not for the LM head: with the arg-max epilogue's state the
  // slices in flight no longer fit the registers (67 spilled, 153 -> 184 us at 1856 rows).
  if constexpr (MODE != kModeSwapLM) {
    const int grid_p = n_cu / 8 * 8;
    if (grid_p >= 8 && tiles_act * tiles_w > grid_p) {
      auto kern_p = k_gemm_mfma8p<MODE, Epi>;
      static const hipError_t attr_rc_p = hipFuncSetAttribute(reinterpret_cast<const void *>(kern_p),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, smem);
      if (attr_rc_p != hipSuccess) return HSD_EHIP;
      hipLaunchKernelGGL(kern_p, dim3(grid_p), dim3(512), smem, st, M, N, K, static_cast<const bf16 *>(A),
                         static_cast<const bf16 *>(W), epi);
      HSD_LAUNCH_CHECK();
      return HSD_OK;
    }
  }
  hipLaunchKernelGGL(kern, dim3(tiles_act * tiles_w), dim3(512), smem, st, M, N, K, static_cast<const bf16 *>(A),
                     static_cast<const bf16 *>(W), epi);
  HSD_LAUNCH_CHECK();
  return HSD_OK;
}

template <typename Cfg, typename Epi>
int launch_gemm_mfma_ws(hipStream_t st, int M, int N, int K, const void *A, const void *W, Epi epi) {
  constexpr int MODE = GemmModeOf<Epi>::value;
  auto kern = k_gemm_mfma_ws<Cfg, MODE, Epi>;
  constexpr int smem = Cfg::kSmemBytes + kRowScaleBytes;
  static const hipError_t attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (attr_rc != hipSuccess) return HSD_EHIP;
  int tiles_act, tiles_w;
  gemm_tiles<Cfg, MODE>(M, N, tiles_act, tiles_w);
  hipLaunchKernelGGL(kern, dim3(tiles_act * tiles_w), dim3(512), smem, st, M, N, K, static_cast<const bf16 *>(A),
                     static_cast<const bf16 *>(W), epi);
  HSD_LAUNCH_CHECK();
  return HSD_OK;
}

template <typename Cfg, typename Epi>
int launch_gemm_mfma_d(hipStream_t st, int M, int N, int K, const void *A, const void *W, Epi epi, int m_base = 0) {
  constexpr int MODE = GemmModeOf<Epi>::value;
  auto kern = k_gemm_mfma_d<Cfg, MODE, Epi>;
  constexpr int smem = Cfg::kSmemBytes + kRowScaleBytes;
  static const hipError_t attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (attr_rc != hipSuccess) return HSD_EHIP;
  int tiles_act, tiles_w;
  gemm_tiles<Cfg, MODE>(M - m_base, N, tiles_act, tiles_w);
  hipLaunchKernelGGL(kern, dim3(tiles_act * tiles_w), dim3(Cfg::kThreadsD), smem, st, M, N, K, m_base,
                     static_cast<const bf16 *>(A), static_cast<const bf16 *>(W), epi);
  HSD_LAUNCH_CHECK();
  return HSD_OK;
}

// Tile configurations of the MFMA GEMM (hsd_debug_set selects one for experiments; default per call site).
using GemmCfg0 = GemmCfg<128, 128, 64, 2, 2>;
using GemmCfg1 = GemmCfg<256, 128, 64, 2, 2>;
using GemmCfg4 = GemmCfg<128, 256, 64, 2, 2>;
using GemmCfg6 = GemmCfg<256, 128, 64, 4, 2>;   // 8 waves, wave tile 64x64
using GemmCfg2 = GemmCfg<64, 128, 64, 2, 2>;    // small tiles for narrow projections (more workgroups)
using GemmCfg3 = GemmCfg<128, 64, 64, 2, 1>;
using GemmCfg5 = GemmCfg<128, 128, 64, 4, 2>;   // 8 waves, wave tile 32x64
// configurations 7 and 9 = k_gemm_mfma_ws (128x128 / 64x128 tile, four multiplying and four moving waves),
// 8 = k_gemm_mfma8, 10 and 11 = k_gemm_mfma_d (64x128 / 128x128 tile, a requesting wave and LDS-direct loads)
using GemmCfgD64 = GemmCfgD<64, 128, 5, 2>;    // two requesting waves: two independent in-order load streams
using GemmCfgD128 = GemmCfgD<128, 128, 4, 4>;
// 12 = the same kernel with ONE multiplying wave on a 32x64 tile (token-by-token decoding, see effective_gemm_cfg)
using GemmCfgD32 = GemmCfgD<32, 64, 6, 2, 1, 1>;
using GemmCfgD64n = GemmCfgD<64, 64, 6, 2, 2, 1>;   // 13: two multiplying waves on a 64x64 tile


// Tile configuration actually used at a call site for a given problem (the launch and everything sized from the
// tile shape, like the LM-head partial records, must agree on it).  -1 = plain kernels.
template <typename T>
int effective_gemm_cfg(const hsd_ctx *ctx, int site, int M, int N, int K) {
  if (!std::is_same<T, bf16>::value || ctx->force_simple || K % 64 != 0) return -1;
  int cfg = ctx->gemm_cfg[site];
  if (cfg < 0 || cfg > 13) cfg = 0;
  // The tile shape never changes a result bit (every output element sums its K slices in the same order), so it
  // may follow the row count and the path stays batch-invariant.  A kernel's time is set by one workgroup's walk
  // over K plus fixed costs as long as the launch fits the chip in one round, so fewer rows take smaller tiles: more
  // workgroups, each with less arithmetic per K slice (measured per site on the 24-layer model at 16 to 1856 rows).
  if (!ctx->gemm_cfg_forced) {
    // 9 / 7: 64x128 / 128x128 tiles with four operand-moving waves; 10: the 64x128 tile fed by a requesting wave
    // (k_gemm_mfma_d).  Measured with operands that come from HBM, as they do inside a pass (24 layers of weights
    // do not stay in any cache): the requesting-wave kernel wins up to ~512 rows (16 rows, K = 4096: 19.5 us against
    // 23.7; 512 rows: 20.7 against 25.4) and loses from ~1 k to ~2 k rows (1856 rows: 35.8 against 32.0), although
    // it wins there too when the operands are cache resident (25.7 against 28.3).
    // At ~4 k rows the 128x128 tile of the same kernel (11) yields one workgroup per compute unit on the square
    // projections and wins there (4096 x 1024, K = 4096: 47.3 us against 56.5).
    // With few rows the weights are all there is to read, from HBM, and a compute unit streams them at a rate that
    // neither deeper rings nor more requesting waves raise (the down projection's 8 workgroups of 64x128 tiles at 16
    // rows: 0.34 TB/s): what helps is more compute units, i.e. narrower tiles, as long as the launch stays within one
    // workgroup per unit -- 32x64 tiles with one multiplying wave (12), else 64x64 with two (13).  Measured with
    // operands from HBM, K = 4096, N = 1024: 16 rows 15.6 us (64x128: 24.5), 512 rows 18.6 (31.0), 1024 rows 23.6 with
    // 64x64 (32.4; two-role kernel 30.0); K = 1024, N = 1536: 256 rows 6.8 (8.3), 512 rows 9.9 with 64x64 (12.3).
    const int64_t cu_n = ctx->n_cu > 0 ? ctx->n_cu : 256;
    const int64_t cols64 = ((site == kSiteGateUp ? 2 * static_cast<int64_t>(N) : N) + 63) / 64;
    if (site == kSiteLM) cfg = M <= 128 ? 0 : cfg;
    else if (static_cast<int64_t>((M + 31) / 32) * cols64 <= cu_n) cfg = 12;
    else if (static_cast<int64_t>((M + 63) / 64) * cols64 <= cu_n) cfg = 13;
    else if (M <= 64) cfg = 10;                                        // one row tile
    else if (site != kSiteGateUp && M <= 512) cfg = 10;
    else if ((site == kSiteO || site == kSiteDown) && M >= 3072) cfg = 11;
    else if (site == kSiteQKV) cfg = M <= 1024 ? 9 : 7;
    else if (site == kSiteO || site == kSiteDown) cfg = 9;   // down walks all of K in one workgroup: small tiles,
                                                             // so that a pass over ~2 k rows still fills the chip
    else if (site == kSiteGateUp) cfg = M <= 256 ? 9 : (M <= 1024 ? 7 : cfg);
  }
  // ... and a pass over many rows (prefill chunks, long-document blocks) has enough row tiles to fill the chip with
  // the 256x256 tile also on the narrower projections (measured crossover: about 6 k rows at N = 1536)
  if ((site == kSiteQKV || site == kSiteO || site == kSiteDown) && M >= 6144 && !ctx->gemm_cfg_forced) {
    // 256x256 tiles, unless their count leaves the last round over the CUs nearly empty and 256x128 tiles (8 waves,
    // one workgroup per CU as well, 0.575 of the time per tile) fill the rounds better
    const int64_t rt = (M + 255) / 256, cu = ctx->n_cu > 0 ? ctx->n_cu : 256;
    const int64_t t8 = rt * ((N + 255) / 256), t6 = rt * ((N + 127) / 128);
    cfg = ((t6 + cu - 1) / cu) * 575 < ((t8 + cu - 1) / cu) * 900 ? 6 : 8;   // only on a clear (10 %) advantage
  }
  // the two-role kernels: not for the swapped LM-head mode
  if ((cfg == 7 || cfg == 9) && site == kSiteLM) cfg = cfg == 7 ? 0 : 2;
  // the LDS-direct kernels: not the swapped mode, 32-bit operand offsets
  if ((cfg == 10 || cfg == 11 || cfg == 12 || cfg == 13) &&
      (site == kSiteLM || static_cast<int64_t>(M) * K * 2 >= (int64_t{1} << 31) ||
       (site == kSiteGateUp ? 2 : 1) * static_cast<int64_t>(N) * K * 2 >= (int64_t{1} << 31)))
    cfg = cfg == 11 ? 0 : 2;
  // the 8-wave kernel needs an even number (>= 4) of 64-wide K slices
  if (cfg == 8 && (K % 128 != 0 || K < 256)) cfg = 0;
  // ... and addresses its operands with 32-bit byte offsets (buffer loads): both matrices must stay below 2 GiB
  // (in dual mode the weight matrix has 2N rows)
  const int64_t w_rows = site == kSiteGateUp ? 2 * static_cast<int64_t>(N) : N;
  if (cfg == 8 && (static_cast<int64_t>(M) * K * 2 >= (int64_t{1} << 31) || w_rows * K * 2 >= (int64_t{1} << 31))) cfg = 0;
  if (site == kSiteLM) {
    // the partial-record buffer holds vocab/64 records per row: at least 64 vocabulary rows per wave, and the
    // vocabulary must be a whole number of tiles (it is a multiple of 128 by validation)
    if (cfg == 2 || cfg == 3 || cfg == 5) cfg = 0;
    if ((cfg == 1 || cfg == 6 || cfg == 8) && N % 256 != 0) cfg = 0;
  }
  return cfg;
}

template <typename T, typename Epi>
int launch_gemm(const hsd_ctx *ctx, hipStream_t st, int site, int M, int N, int K, const void *A, const void *W,
                const Epi &epi) {
  if constexpr (std::is_same<T, bf16>::value) {
    const int cfg = effective_gemm_cfg<T>(ctx, site, M, N, K);
    if constexpr (GemmModeOf<Epi>::value != kModeSwapLM) {
      // Rounds over the chip.  The 256x256 kernel runs one tile per compute unit at a time, so a tile count just
      // above a multiple of the number of units costs a whole extra round (4 pages of 8193 rows: 129 x 4 tiles of
      // the down projection = 2.02 rounds; a prefill of 16,880 rows: 66 x 4 = 1.03 rounds).  When leaving out at most
      // 512 rows saves that round, those rows go to the small-tile kernel in a launch of their own (rows are
      // independent in every epilogue).  Costs in us from the measured per-tile times: a 256x256 tile 6 + 1.9 per K
      // slice, a round of 64x128 tiles 6 + 0.3 per slice, a 256x128 tile 0.64 of a 256x256 one.
      if ((cfg == 8 || cfg == 6) && !ctx->gemm_cfg_forced && K % 128 == 0 && K >= 256) {
        const int64_t cu = ctx->n_cu > 0 ? ctx->n_cu : 256;
        const int64_t w_cols = site == kSiteGateUp ? 2 * static_cast<int64_t>(N) : N;
        const int64_t tw8 = (w_cols + 255) / 256, tw_small = (w_cols + 127) / 128;
        const int64_t r_all = (M + 255) / 256, rounds_all = (r_all * tw8 + cu - 1) / cu;
        const int64_t r_main = std::min<int64_t>(M / 256, (rounds_all - 1) * cu / tw8);
        const int64_t rem = M - 256 * r_main;
        if (rounds_all >= 2 && r_main >= 1 && rem > 0 && rem <= 512 &&
            static_cast<int64_t>(M) * K * 2 < (int64_t{1} << 31) && w_cols * K * 2 < (int64_t{1} << 31)) {
          const double t8 = 6.0 + 1.9 * (K / 64), t_small = 6.0 + 0.3 * (K / 64);
          const double cost_all = cfg == 8 ? rounds_all * t8 : ((r_all * tw_small + cu - 1) / cu) * 0.64 * t8;
          const double cost_split = ((r_main * tw8 + cu - 1) / cu) * t8 +
                                    ((((rem + 63) / 64) * tw_small + cu - 1) / cu) * t_small;
          if (cost_split < 0.9 * cost_all) {
            const int m_main = static_cast<int>(256 * r_main);
            const int rc = launch_gemm_mfma8(st, m_main, N, K, A, W, epi, ctx->n_cu);
            if (rc != HSD_OK) return rc;
            // the narrowest tile that still gives at most one workgroup per compute unit (see effective_gemm_cfg)
            const int64_t cols64 = (w_cols + 63) / 64;
            if (((rem + 31) / 32) * cols64 <= cu) return launch_gemm_mfma_d<GemmCfgD32>(st, M, N, K, A, W, epi, m_main);
            if (((rem + 63) / 64) * cols64 <= cu) return launch_gemm_mfma_d<GemmCfgD64n>(st, M, N, K, A, W, epi, m_main);
            return launch_gemm_mfma_d<GemmCfgD64>(st, M, N, K, A, W, epi, m_main);
          }
        }
      }
    }
    switch (cfg) {
      case -1: break;
      case 1: return launch_gemm_mfma<GemmCfg1>(st, M, N, K, A, W, epi);
      case 2: return launch_gemm_mfma<GemmCfg2>(st, M, N, K, A, W, epi);
      case 3: return launch_gemm_mfma<GemmCfg3>(st, M, N, K, A, W, epi);
      case 4: return launch_gemm_mfma<GemmCfg4>(st, M, N, K, A, W, epi);
      case 5: return launch_gemm_mfma<GemmCfg5>(st, M, N, K, A, W, epi);
      case 6: return launch_gemm_mfma<GemmCfg6>(st, M, N, K, A, W, epi);
      case 7:
        if constexpr (GemmModeOf<Epi>::value != kModeSwapLM)
          return launch_gemm_mfma_ws<GemmCfgWS>(st, M, N, K, A, W, epi);
        break;
      case 9:
        if constexpr (GemmModeOf<Epi>::value != kModeSwapLM)
          return launch_gemm_mfma_ws<GemmCfgWS64>(st, M, N, K, A, W, epi);
        break;
      case 8: return launch_gemm_mfma8(st, M, N, K, A, W, epi, ctx->n_cu);
      case 10:
        if constexpr (GemmModeOf<Epi>::value != kModeSwapLM)
          return launch_gemm_mfma_d<GemmCfgD64>(st, M, N, K, A, W, epi);
        break;
      case 11:
        if constexpr (GemmModeOf<Epi>::value != kModeSwapLM)
          return launch_gemm_mfma_d<GemmCfgD128>(st, M, N, K, A, W, epi);
        break;
      case 12:
        if constexpr (GemmModeOf<Epi>::value != kModeSwapLM)
          return launch_gemm_mfma_d<GemmCfgD32>(st, M, N, K, A, W, epi);
        break;
      case 13:
        if constexpr (GemmModeOf<Epi>::value != kModeSwapLM)
          return launch_gemm_mfma_d<GemmCfgD64n>(st, M, N, K, A, W, epi);
        break;
      default: return launch_gemm_mfma<GemmCfg0>(st, M, N, K, A, W, epi);
    }
  }
  if constexpr (std::is_same<Epi, EpiResidualNorm>::value) {
    return HSD_EINVAL;   // this epilogue exists for the MFMA kernels only (the caller never gets here with it)
  } else {
    dim3 grid(N / 64, (M + 63) / 64);
    hipLaunchKernelGGL((k_gemm_simple<T, Epi>), grid, dim3(256), 0, st, M, N, K, static_cast<const T *>(A),
                       static_cast<const T *>(W), epi);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
  }
}

// Number of (row, column-tile) partial records the LM-head GEMM writes per row.
template <typename T>
int lm_head_tiles(const hsd_ctx *ctx, int M) {
  const int V = ctx->desc.vocab;
  switch (effective_gemm_cfg<T>(ctx, kSiteLM, M, V, ctx->desc.d_model)) {
    case -1: return V / 64;
    case 1: return V / GemmCfg1::BP * GemmCfg1::WM;
    case 4: return V / GemmCfg4::BP * GemmCfg4::WM;
    case 6: return V / GemmCfg6::BP * GemmCfg6::WM;
    case 8: return V / GemmCfg8::BP * GemmCfg8::WM;
    default: return V / GemmCfg0::BP * GemmCfg0::WM;
  }
}

// Verification attention: bf16 goes to the MFMA kernel when the GQA group size fits its wave mapping.
// A compute unit has 160 KB of LDS; a request above half of it keeps a workgroup alone on its compute unit.
constexpr size_t kLdsExclusive = 84 * 1024;

template <int G4, int QS, bool TREE, bool SPLIT>
int launch_attn_mfma(hipStream_t st, dim3 grid, int n_cu, int n_q_heads, const AttnTile *tiles, const PagedKV &kv,
                     const bf16 *q, bf16 *o, const int32_t *row_end, const AttnSplit &sp) {
  constexpr size_t smem = attn_smem_bytes(QS);
  auto kern = k_attn_mfma<G4, QS, TREE, SPLIT>;
  // set once per instantiation (initialisation of a function-local static is thread safe)
  static const hipError_t attr_rc =
      hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          smem > kLdsExclusive ? smem : kLdsExclusive);
  if (attr_rc != hipSuccess) return HSD_EHIP;
  // Two workgroups fit a compute unit, and the dispatcher does pair them up while other units are still empty:
  // with about one workgroup per unit (measured on the 16-region workload: 30 of 256 units held two, 30 none) the
  // paired ones run 1.7 times as long and set the launch's duration (31 us against 22 us).  A launch with no more
  // workgroups than the chip has units therefore asks for more LDS than half a unit has, which spreads it one
  // workgroup per unit.  (With a few more workgroups than units pairing is the better deal: a second round would
  // cost more.)  Scheduling only: no result depends on it.
  const size_t n_wg = static_cast<size_t>(grid.x) * grid.y * grid.z;
  const size_t lds = (n_cu > 0 && n_wg <= static_cast<size_t>(n_cu) && smem < kLdsExclusive) ? kLdsExclusive : smem;
  hipLaunchKernelGGL(kern, grid, dim3(128 * QS), lds, st, n_q_heads, tiles, kv, q, o, row_end, sp);
  HSD_LAUNCH_CHECK();
  return HSD_OK;
}

template <typename T>
int launch_attention(const hsd_ctx *ctx, hipStream_t st, const hsd_batch *b, const RowMeta &meta, const PagedKV &kv,
                     const Workspace &ws, bool page_mode) {
  const hsd_model_desc &d = ctx->desc;
  const int group = d.n_q_heads / d.n_kv_heads;
  if constexpr (std::is_same<T, bf16>::value) {
    if (!ctx->force_simple && (group == 1 || group == 2 || group % 4 == 0)) {
      // Work split, fixed per model and entry point (never chosen from the batch; and one row's arithmetic is the
      // same in both, so results stay bitwise batch-invariant): g4 query heads of a kv head among the query sets of
      // a workgroup; 4 query sets for region-level batches (many short blocks: more, smaller workgroups), 8 for
      // page-level ones (few long blocks: each K/V stage in LDS serves twice the queries).
      const int g4 = group >= 4 ? 4 : group, qs = page_mode ? 8 : 4;
      const int q_tile = 32 * (qs / g4);
      const int max_tiles = b->total_q / q_tile + b->n_seq;
      const int n_y = d.n_kv_heads * ((group + g4 - 1) / g4);
      const int sub_tiles = 256 / q_tile;   // tiles of one sequence and head group that share an XCD: 256 rows
      const int n_wg = attn_grid_size(max_tiles, n_y, sub_tiles);
      const dim3 grid(n_wg, 1);
      const bf16 *q = static_cast<const bf16 *>(ws.q);
      bf16 *o = static_cast<bf16 *>(ws.a);
      if (kv.layer == 0) {  // the task table depends on the batch only: built once per pass
        hipLaunchKernelGGL(k_attn_tiles, dim3(1), dim3(1024), 0, st, b->n_seq, b->cu_q, b->seq_slot, b->n_slots,
                           b->seq_len, q_tile, n_y, sub_tiles, n_wg, ws.attn_tiles);
        HSD_LAUNCH_CHECK();
      }
      // Key split (desc.attn_key_chunk > 0): one workgroup per (query tile, chunk of keys); no sequence can hold
      // more keys than its block-table row addresses, which bounds the chunks worth launching.
      const int chunk = d.attn_key_chunk;
      int n_chunks = 1;
      if (chunk > 0) {
        const int64_t max_keys = static_cast<int64_t>(b->max_blocks_per_seq) * HSD_KV_BLOCK_TOKENS;
        n_chunks = static_cast<int>(std::min<int64_t>(kAttnMaxChunks, (max_keys + chunk - 1) / chunk));
      }
      const dim3 grid_z(grid.x, grid.y, n_chunks);
      const AttnSplit sp{chunk, b->total_q, ws.attn_part_o, ws.attn_part_ml};
      const bool tree = meta.row_end != nullptr;
      int rc = HSD_OK;
#define HSD_ATTN_CASE(G4, QS)                                                                                      \
  if (g4 == G4 && qs == QS) {                                                                                      \
    if (tree && chunk > 0) rc = launch_attn_mfma<G4, QS, true, true>(st, grid_z, ctx->n_cu, d.n_q_heads, ws.attn_tiles, kv, q, o, meta.row_end, sp);       \
    else if (tree) rc = launch_attn_mfma<G4, QS, true, false>(st, grid_z, ctx->n_cu, d.n_q_heads, ws.attn_tiles, kv, q, o, meta.row_end, sp);             \
    else if (chunk > 0) rc = launch_attn_mfma<G4, QS, false, true>(st, grid_z, ctx->n_cu, d.n_q_heads, ws.attn_tiles, kv, q, o, meta.row_end, sp);        \
    else rc = launch_attn_mfma<G4, QS, false, false>(st, grid_z, ctx->n_cu, d.n_q_heads, ws.attn_tiles, kv, q, o, meta.row_end, sp);                      \
  }
      HSD_ATTN_CASE(4, 4) HSD_ATTN_CASE(4, 8) HSD_ATTN_CASE(2, 4) HSD_ATTN_CASE(2, 8) HSD_ATTN_CASE(1, 4) HSD_ATTN_CASE(1, 8)
#undef HSD_ATTN_CASE
      if (rc != HSD_OK) return rc;
      if (chunk > 0) {
        const int64_t n_thr = static_cast<int64_t>(d.n_q_heads) * b->total_q * 16;
        hipLaunchKernelGGL(k_attn_merge, dim3(static_cast<unsigned>((n_thr + 255) / 256)), dim3(256), 0, st,
                           d.n_q_heads, meta.row_slot, sp, o);
        HSD_LAUNCH_CHECK();
      }
      return HSD_OK;
    }
  }
  hipLaunchKernelGGL((k_attn_simple<T>), dim3(b->total_q, (d.n_q_heads + 3) / 4), dim3(256), 0, st, d.n_q_heads, meta,
                     kv, static_cast<const T *>(ws.q), static_cast<T *>(ws.a));
  HSD_LAUNCH_CHECK();
  return HSD_OK;
}

template <typename T>
int forward(hsd_ctx *ctx, hipStream_t st, const hsd_kv_pool *pool, const hsd_batch *b, void *ws_base, bool page_mode,
            bool with_head) {
  const hsd_model_desc &d = ctx->desc;
  const int Tq = b->total_q;
  Workspace ws = carve(d, Tq, b->n_seq, ws_base);
  const int qdim = d.n_q_heads * d.head_dim, kvdim = d.n_kv_heads * d.head_dim;
  const bool relaxed = with_head && b->log_tau < 0.f;   // Eq. 11 with tau < 1: needs the draft tokens' own logits
  int rc;

  hipLaunchKernelGGL(k_row_meta, dim3((Tq * 32 + 255) / 256), dim3(256), 0, st, b->n_seq, Tq, b->cu_q, b->seq_slot,
                     b->n_slots, b->seq_len, d.rope_theta, ws.row_seq, ws.row_pos, ws.row_slot, ws.row_base, ws.rope_cs,
                     b->tree_end, b->tree_depth, ws.row_end, relaxed ? ws.row_par : nullptr, ws.want_logit, b->status);
  HSD_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_kv_reserve, dim3(1), dim3(1024), 0, st, b->n_seq, b->cu_q, b->seq_slot, b->n_slots,
                     b->seq_len, b->block_table, b->max_blocks_per_seq, pool->n_blocks, pool->free_list,
                     pool->free_count, b->status);
  HSD_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_row_kv, dim3((Tq + 255) / 256), dim3(256), 0, st, Tq, ws.row_seq, ws.row_slot, b->block_table,
                     b->max_blocks_per_seq, pool->n_blocks, ws.row_kv);
  HSD_LAUNCH_CHECK();
  hipLaunchKernelGGL((k_embed<T>), dim3(Tq), dim3(256), 0, st, d.d_model, d.vocab, b->tokens, b->embeds,
                     static_cast<const T *>(ctx->tok_embed), ws.x);
  HSD_LAUNCH_CHECK();

  const bool tree = b->tree_end != nullptr;
  RowMeta meta{ws.row_seq, ws.row_pos, ws.rope_cs, ws.row_kv, ws.row_slot, ws.row_base, tree ? ws.row_end : nullptr};
  const bool mfma_path = std::is_same<T, bf16>::value && !ctx->force_simple;

  // RMSNorm as a kernel of its own: the first norm of a pass, and every norm of the plain-kernel path
  auto norm = [&](const float *gain) -> int {
    ProfScope ps(ctx, st, HSD_PROF_RMSNORM);
    hipLaunchKernelGGL((k_rmsnorm<T>), dim3((Tq + 3) / 4), dim3(256), 0, st, Tq, d.d_model, d.rms_eps, ws.x, gain,
                       static_cast<T *>(ws.h));
    HSD_LAUNCH_CHECK();
    return HSD_OK;
  };
  // x += A W^T.  MFMA path: the epilogue also prepares the norm that follows (operand x * gain and the row sums of
  // squares, see RowScale), so that norm never runs as a kernel; plain path: residual only, then the norm kernel.
  auto residual_proj = [&](int site, int prof, const void *A, const void *W, int K, const float *next_gain) -> int {
    {
      ProfScope ps(ctx, st, prof);
      int rc2;
      if constexpr (std::is_same<T, bf16>::value) {
        if (mfma_path) {
          EpiResidualNorm en{ws.x, d.d_model, next_gain, static_cast<bf16 *>(ws.h), ws.ss};
          rc2 = launch_gemm<T>(ctx, st, site, Tq, d.d_model, K, A, W, en);
          return rc2;
        }
      }
      EpiResidual er{ws.x, d.d_model};
      if ((rc2 = launch_gemm<T>(ctx, st, site, Tq, d.d_model, K, A, W, er))) return rc2;
    }
    return next_gain != nullptr ? norm(next_gain) : HSD_OK;
  };
  const RowScale rs_none{nullptr, 0, 0.f, 0.f};
  const RowScale rs_fused{mfma_path ? ws.ss : nullptr, d.d_model / 64, 1.0f / static_cast<float>(d.d_model), d.rms_eps};

  if ((rc = norm(ctx->attn_norm[0]))) return rc;
  for (int l = 0; l < d.n_layers; ++l) {
    PagedKV kv{pool->k_pool, pool->v_pool, b->block_table, b->max_blocks_per_seq, pool->n_blocks, d.n_kv_heads, l};
    // layer 0 reads the operand the norm kernel normalised; later layers the one the previous down projection left
    EpiQKV<T> eq{d.n_q_heads, d.n_kv_heads, meta, kv, static_cast<T *>(ws.q), l == 0 ? rs_none : rs_fused};
    {
      ProfScope ps(ctx, st, HSD_PROF_GEMM_QKV);
      if ((rc = launch_gemm<T>(ctx, st, kSiteQKV, Tq, qdim + 2 * kvdim, d.d_model, ws.h, ctx->wqkv[l], eq))) return rc;
    }
    {
      ProfScope ps(ctx, st, HSD_PROF_ATTENTION);
      if ((rc = launch_attention<T>(ctx, st, b, meta, kv, ws, page_mode))) return rc;
    }
    if ((rc = residual_proj(kSiteO, HSD_PROF_GEMM_O, ws.a, ctx->wo[l], qdim, ctx->ffn_norm[l]))) return rc;
    EpiSwiGLU<T> es{static_cast<T *>(ws.u), d.d_ffn, rs_fused};
    {
      ProfScope ps(ctx, st, HSD_PROF_GEMM_GATE_UP);
      if ((rc = launch_gemm<T>(ctx, st, kSiteGateUp, Tq, d.d_ffn, d.d_model, ws.h, ctx->w_gate_up[l], es))) return rc;
    }
    // the norm that follows: next layer's attention norm, or the final norm before the LM head (none for prefill)
    const float *next_gain = (l + 1 < d.n_layers) ? ctx->attn_norm[l + 1] : (with_head ? ctx->final_norm : nullptr);
    if ((rc = residual_proj(kSiteDown, HSD_PROF_GEMM_DOWN, ws.u, ctx->w_down[l], d.d_ffn, next_gain))) return rc;
    if (ctx->sync_layers && hipStreamSynchronize(st) != hipSuccess) return HSD_EHIP;
  }
  if (!with_head) return HSD_OK;

  const int32_t *dump_slot = nullptr;
  if (b->n_dump > 0 && b->logits_dump != nullptr) {
    hipLaunchKernelGGL(k_fill_i32, dim3((Tq + 255) / 256), dim3(256), 0, st, ws.dump_slot, Tq, -1);
    HSD_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_dump_slots, dim3((b->n_dump + 255) / 256), dim3(256), 0, st, b->dump_rows, b->n_dump, Tq,
                       ws.dump_slot);
    HSD_LAUNCH_CHECK();
    dump_slot = ws.dump_slot;
  }
  const int n_tiles = lm_head_tiles<T>(ctx, Tq);
  EpiLMHead el{ws.lm_part, n_tiles, d.vocab, dump_slot, b->logits_dump, b->tokens, ws.row_end,
               relaxed ? ws.want_logit : nullptr, rs_fused};
  {
    ProfScope ps(ctx, st, HSD_PROF_GEMM_LM_HEAD);
    if ((rc = launch_gemm<T>(ctx, st, kSiteLM, Tq, d.vocab, d.d_model, ws.h, ctx->lm_head, el))) return rc;
  }
  hipLaunchKernelGGL(k_lm_reduce, dim3((Tq + 3) / 4), dim3(256), 0, st, Tq, n_tiles, ws.lm_part, b->argmax,
                     b->top2_margin, relaxed ? ws.row_max : nullptr);
  HSD_LAUNCH_CHECK();
  if (relaxed) {
    hipLaunchKernelGGL(k_draft_gap, dim3((Tq + 255) / 256), dim3(256), 0, st, Tq, ws.row_par, ws.want_logit,
                       ws.row_max, b->draft_gap);
    HSD_LAUNCH_CHECK();
  }
  if (tree)
    hipLaunchKernelGGL(k_accept_tree, dim3((b->n_seq + 63) / 64), dim3(64), 0, st, b->n_seq, b->cu_q, b->tokens,
                       b->argmax, ws.row_end, ws.want_logit, relaxed ? b->draft_gap : nullptr, b->log_tau,
                       b->accept_len, b->bonus, b->stop_row);
  else
    hipLaunchKernelGGL(k_accept, dim3((b->n_seq + 3) / 4), dim3(256), 0, st, b->n_seq, b->cu_q, b->tokens, b->argmax,
                       relaxed ? b->draft_gap : nullptr, b->log_tau, b->accept_len, b->bonus);
  HSD_LAUNCH_CHECK();
  return HSD_OK;
}

int verify_common(hsd_ctx *ctx, void *stream, const hsd_kv_pool *pool, const hsd_batch *b, void *ws, size_t ws_bytes,
                  bool page_mode, bool prefill) {
  if (ctx == nullptr || ws == nullptr) return HSD_EINVAL;
  int rc = hsd_validate_batch(&ctx->desc, pool, b, ws_bytes);
  if (rc != HSD_OK) return rc;
  if (pool == nullptr) return HSD_EINVAL;
  if (!prefill && (b->argmax == nullptr || b->accept_len == nullptr || b->bonus == nullptr)) return HSD_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool with_head = !prefill;
  if (ctx->desc.dtype == HSD_BF16)
    rc = forward<bf16>(ctx, st, pool, b, ws, page_mode, with_head);
  else
    rc = forward<float>(ctx, st, pool, b, ws, page_mode, with_head);
  if (rc != HSD_OK) return rc;
  if (prefill) {
    hipLaunchKernelGGL(k_kv_commit, dim3(1), dim3(1024), 0, st, b->n_seq, b->cu_q, b->seq_slot, b->n_slots,
                       b->seq_len, b->block_table, b->max_blocks_per_seq, pool->n_blocks, pool->free_list,
                       pool->free_count, static_cast<const int32_t *>(nullptr), static_cast<const int32_t *>(nullptr),
                       static_cast<int32_t *>(nullptr), 1);
    HSD_LAUNCH_CHECK();
  }
  return HSD_OK;
}

}  // namespace

extern "C" {

const char *hsd_status_string(int status) {
  switch (status) {
    case HSD_OK: return "ok";
    case HSD_EINVAL: return "invalid argument";
    case HSD_ENOSPC: return "workspace too small";
    case HSD_ERANGE: return "size out of range";
    case HSD_EARCH: return "device is not gfx950";
    case HSD_ENODEV: return "no HIP device";
    case HSD_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int hsd_validate_model(const hsd_model_desc *d) {
  if (d == nullptr) return HSD_EINVAL;
  if (d->n_layers < 1 || d->d_model < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->d_ffn < 1 || d->vocab < 1)
    return HSD_EINVAL;
  if (d->head_dim != HSD_HEAD_DIM || d->kv_block_tokens != HSD_KV_BLOCK_TOKENS) return HSD_EINVAL;
  if (d->dtype != HSD_BF16 && d->dtype != HSD_FP32) return HSD_EINVAL;
  if (d->n_q_heads % d->n_kv_heads != 0) return HSD_EINVAL;
  if (d->d_model % 128 != 0 || d->d_ffn % 128 != 0 || d->vocab % 128 != 0) return HSD_EINVAL;
  if (!(d->rms_eps > 0.f) || !(d->rope_theta > 1.f)) return HSD_EINVAL;
  if (d->attn_key_chunk < 0 || d->attn_key_chunk % 128 != 0) return HSD_EINVAL;
  if (d->n_layers > 1024 || d->n_q_heads > 1024) return HSD_ERANGE;
  return HSD_OK;
}

size_t hsd_workspace_bytes(const hsd_model_desc *desc, int32_t max_total_q, int32_t max_n_seq) {
  if (hsd_validate_model(desc) != HSD_OK || max_total_q < 1 || max_n_seq < 1) return 0;
  return carve(*desc, max_total_q, max_n_seq, nullptr).total;
}

int hsd_validate_batch(const hsd_model_desc *desc, const hsd_kv_pool *pool, const hsd_batch *b, size_t ws_bytes) {
  int rc = hsd_validate_model(desc);
  if (rc != HSD_OK) return rc;
  if (b == nullptr) return HSD_EINVAL;
  if (b->n_seq < 1 || b->total_q < b->n_seq || b->max_blocks_per_seq < 1) return HSD_EINVAL;
  if (b->n_slots < 1 || (b->seq_slot == nullptr && b->n_slots < b->n_seq)) return HSD_EINVAL;
  if (b->n_seq > HSD_MAX_SEQ) return HSD_ERANGE;
  if (static_cast<int64_t>(b->total_q) * desc->vocab / 64 > (int64_t{1} << 40)) return HSD_ERANGE;
  if (b->cu_q == nullptr || b->tokens == nullptr || b->seq_len == nullptr || b->block_table == nullptr ||
      b->status == nullptr)
    return HSD_EINVAL;
  if (b->n_dump < 0 || (b->n_dump > 0 && (b->logits_dump == nullptr || b->dump_rows == nullptr))) return HSD_EINVAL;
  // log_tau is log(tau) of a threshold in (0, 1]: finite and <= 0 (the comparison also rejects NaN); the relaxed
  // rule needs somewhere to put the per-row gaps
  if (!(b->log_tau <= 0.f) || std::isinf(b->log_tau)) return HSD_EINVAL;
  if (b->log_tau < 0.f && b->argmax != nullptr && b->draft_gap == nullptr) return HSD_EINVAL;
  if (b->tree_end != nullptr && (b->tree_depth == nullptr || (b->argmax != nullptr && b->stop_row == nullptr)))
    return HSD_EINVAL;
  if (pool != nullptr) {
    if (pool->k_pool == nullptr || pool->v_pool == nullptr || pool->free_list == nullptr ||
        pool->free_count == nullptr || pool->n_blocks < 1)
      return HSD_EINVAL;
  }
  if (ws_bytes < hsd_workspace_bytes(desc, b->total_q, b->n_seq)) return HSD_ENOSPC;
  return HSD_OK;
}

int hsd_create(const hsd_model_desc *desc, const hsd_weights *w, hsd_ctx **out) {
  if (out == nullptr) return HSD_EINVAL;
  *out = nullptr;
  int rc = hsd_validate_model(desc);
  if (rc != HSD_OK) return rc;
  if (w == nullptr || w->tok_embed == nullptr || w->final_norm == nullptr || w->lm_head == nullptr ||
      w->attn_norm == nullptr || w->wqkv == nullptr || w->wo == nullptr || w->ffn_norm == nullptr ||
      w->w_gate_up == nullptr || w->w_down == nullptr)
    return HSD_EINVAL;
  for (int l = 0; l < desc->n_layers; ++l)
    if (w->attn_norm[l] == nullptr || w->wqkv[l] == nullptr || w->wo[l] == nullptr || w->ffn_norm[l] == nullptr ||
        w->w_gate_up[l] == nullptr || w->w_down[l] == nullptr)
      return HSD_EINVAL;
  int dev = 0, count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || count < 1) {
    (void)hipGetLastError();
    return HSD_ENODEV;
  }
  if (hipGetDevice(&dev) != hipSuccess) return HSD_ENODEV;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return HSD_EHIP;
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return HSD_EARCH;
  hsd_ctx *c = new (std::nothrow) hsd_ctx();
  if (c == nullptr) return HSD_EHIP;
  c->desc = *desc;
  c->tok_embed = w->tok_embed;
  c->final_norm = w->final_norm;
  c->lm_head = w->lm_head;
  c->attn_norm.assign(w->attn_norm, w->attn_norm + desc->n_layers);
  c->ffn_norm.assign(w->ffn_norm, w->ffn_norm + desc->n_layers);
  c->wqkv.assign(w->wqkv, w->wqkv + desc->n_layers);
  c->wo.assign(w->wo, w->wo + desc->n_layers);
  c->w_gate_up.assign(w->w_gate_up, w->w_gate_up + desc->n_layers);
  c->w_down.assign(w->w_down, w->w_down + desc->n_layers);
  c->n_cu = prop.multiProcessorCount;
  // the context belongs to the current device: resolve that device's copy of the static scratch array once
  if (hipGetSymbolAddress(&c->static_ws, HIP_SYMBOL(g_static_ws)) != hipSuccess || c->static_ws == nullptr) {
    (void)hipGetLastError();
    delete c;
    return HSD_EHIP;
  }
  c->force_simple = false;
  // 256x256 8-wave tiles for the wide projections (gate/up, LM head), 64x128 tiles for QKV, O and down (more
  // workgroups)
  const int defaults[5] = {5, 2, 8, 2, 8};
  for (int i = 0; i < 5; ++i) c->gemm_cfg[i] = defaults[i];
  *out = c;
  return HSD_OK;
}

int hsd_debug_set(hsd_ctx *c, int knob, int64_t value) {
  if (c == nullptr) return HSD_EINVAL;
  switch (knob) {
    case HSD_DEBUG_SYNC_LAYERS: c->sync_layers = value != 0; return HSD_OK;
    case HSD_DEBUG_FORCE_SIMPLE: c->force_simple = value != 0; return HSD_OK;
    case HSD_DEBUG_GEMM_CFG_QKV:
    case HSD_DEBUG_GEMM_CFG_O:
    case HSD_DEBUG_GEMM_CFG_GATE_UP:
    case HSD_DEBUG_GEMM_CFG_DOWN:
    case HSD_DEBUG_GEMM_CFG_LM_HEAD:
      if (value < 0 || value > 13) return HSD_EINVAL;
      c->gemm_cfg[knob - HSD_DEBUG_GEMM_CFG_QKV] = static_cast<int>(value);
      c->gemm_cfg_forced = true;
      return HSD_OK;
    default: return HSD_EINVAL;
  }
}

int hsd_probe_launch(void *stream, int kind, int n_workgroups, int iters, int arg, void *scratch, size_t scratch_bytes) {
  if (n_workgroups < 1 || n_workgroups > (1 << 20) || iters < 1 || scratch == nullptr || scratch_bytes < 4) return HSD_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float *sink = static_cast<float *>(scratch);
  switch (kind) {
    case HSD_PROBE_MFMA:
      hipLaunchKernelGGL(k_probe_mfma, dim3(n_workgroups), dim3(256), 0, st, iters, sink);
      break;
    case HSD_PROBE_LOAD_REG:
    case HSD_PROBE_LOAD_LDS: {
      const size_t region = scratch_bytes / 8;
      if (region < 32768 || region % 32768 != 0 || region >= (size_t{1} << 31)) return HSD_EINVAL;
      if (kind == HSD_PROBE_LOAD_REG)
        hipLaunchKernelGGL(k_probe_load<false>, dim3(n_workgroups), dim3(256), 32768, st,
                           static_cast<const unsigned char *>(scratch), static_cast<int>(region), iters, sink);
      else
        hipLaunchKernelGGL(k_probe_load<true>, dim3(n_workgroups), dim3(256), 32768, st,
                           static_cast<const unsigned char *>(scratch), static_cast<int>(region), iters, sink);
      break;
    }
    case HSD_PROBE_LDS_READ: {
      if (arg < 1 || arg > 16) return HSD_EINVAL;
      // more than half of a compute unit's LDS: one workgroup per unit
      constexpr int smem = 96 * 1024;
      static const hipError_t attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(k_probe_lds),
                                                            hipFuncAttributeMaxDynamicSharedMemorySize, smem);
      if (attr_rc != hipSuccess) return HSD_EHIP;
      hipLaunchKernelGGL(k_probe_lds, dim3(n_workgroups), dim3(64 * arg), smem, st, iters, sink);
      break;
    }
    default: return HSD_EINVAL;
  }
  HSD_LAUNCH_CHECK();
  return HSD_OK;
}

void hsd_destroy(hsd_ctx *ctx) {
  if (ctx == nullptr) return;
  for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
  delete ctx;
}

int hsd_profile_enable(hsd_ctx *ctx, int which, int32_t max_launches) {
  if (ctx == nullptr || which < HSD_PROF_NONE || which > HSD_PROF_RMSNORM || max_launches < 0) return HSD_EINVAL;
  if (max_launches > (1 << 20)) return HSD_ERANGE;
  for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
  ctx->prof_events.clear();
  ctx->prof_used = 0;
  ctx->prof_which = which;
  if (which == HSD_PROF_NONE) return HSD_OK;
  ctx->prof_events.resize(2 * static_cast<size_t>(max_launches));
  for (size_t i = 0; i < ctx->prof_events.size(); ++i)
    if (hipEventCreate(&ctx->prof_events[i]) != hipSuccess) {
      ctx->prof_events.resize(i);
      return HSD_EHIP;
    }
  return HSD_OK;
}

int hsd_profile_read(hsd_ctx *ctx, int32_t *n_launches, float *total_ms) {
  if (ctx == nullptr || n_launches == nullptr || total_ms == nullptr) return HSD_EINVAL;
  float sum = 0.f;
  for (int i = 0; i < ctx->prof_used; ++i) {
    float ms = 0.f;
    if (hipEventSynchronize(ctx->prof_events[2 * i + 1]) != hipSuccess) return HSD_EHIP;
    if (hipEventElapsedTime(&ms, ctx->prof_events[2 * i], ctx->prof_events[2 * i + 1]) != hipSuccess) return HSD_EHIP;
    sum += ms;
  }
  *n_launches = ctx->prof_used;
  *total_ms = sum;
  ctx->prof_used = 0;
  return HSD_OK;
}

int hsd_kv_pool_init(void *stream, const hsd_kv_pool *pool) {
  if (pool == nullptr || pool->free_list == nullptr || pool->free_count == nullptr || pool->n_blocks < 1)
    return HSD_EINVAL;
  hipLaunchKernelGGL(k_pool_init, dim3((pool->n_blocks + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                     pool->n_blocks, pool->free_list, pool->free_count);
  HSD_LAUNCH_CHECK();
  return HSD_OK;
}

int hsd_verify_region_batch(hsd_ctx *ctx, void *stream, const hsd_kv_pool *pool, const hsd_batch *batch, void *ws,
                            size_t ws_bytes) {
  return verify_common(ctx, stream, pool, batch, ws, ws_bytes, /*page_mode=*/false, /*prefill=*/false);
}

int hsd_verify_region_batch_noalloc(hsd_ctx *ctx, void *stream, const hsd_kv_pool *pool, const hsd_batch *batch) {
  if (ctx == nullptr || batch == nullptr) return HSD_EINVAL;
  if (batch->total_q < 1 || batch->n_seq < 1) return HSD_EINVAL;
  // the batch must fit the fixed scratch array (nothing is allocated here or anywhere below)
  if (hsd_workspace_bytes(&ctx->desc, batch->total_q, batch->n_seq) > kStaticWsBytes) return HSD_ERANGE;
  return verify_common(ctx, stream, pool, batch, ctx->static_ws, kStaticWsBytes, /*page_mode=*/false, /*prefill=*/false);
}

size_t hsd_noalloc_scratch_bytes(void) { return kStaticWsBytes; }

int hsd_verify_page(hsd_ctx *ctx, void *stream, const hsd_kv_pool *pool, const hsd_batch *batch, void *ws,
                    size_t ws_bytes) {
  return verify_common(ctx, stream, pool, batch, ws, ws_bytes, /*page_mode=*/true, /*prefill=*/false);
}

int hsd_prefill(hsd_ctx *ctx, void *stream, const hsd_kv_pool *pool, const hsd_batch *batch, void *ws,
                size_t ws_bytes) {
  return verify_common(ctx, stream, pool, batch, ws, ws_bytes, /*page_mode=*/true, /*prefill=*/true);
}

int hsd_kv_commit_rollback(hsd_ctx *ctx, void *stream, const hsd_kv_pool *pool, const hsd_batch *b,
                           int32_t *pending_out) {
  if (ctx == nullptr || pool == nullptr) return HSD_EINVAL;
  int rc = hsd_validate_batch(&ctx->desc, pool, b, static_cast<size_t>(-1));
  if (rc != HSD_OK) return rc;
  if (b->accept_len == nullptr || b->bonus == nullptr) return HSD_EINVAL;
  if (b->tree_end != nullptr) {
    // packed prefix tree: move the accepted path's K/V to contiguous slots before the lengths change
    if (b->stop_row == nullptr) return HSD_EINVAL;
    const hsd_model_desc &d = ctx->desc;
    const dim3 grid(b->n_seq, d.n_layers * d.n_kv_heads);
    if (d.dtype == HSD_BF16)
      hipLaunchKernelGGL((k_kv_compact<bf16>), grid, dim3(64), 0, static_cast<hipStream_t>(stream), b->cu_q, b->seq_slot,
                         b->n_slots, b->seq_len, b->block_table, b->max_blocks_per_seq, pool->n_blocks, d.n_kv_heads,
                         b->tree_end, b->accept_len, b->stop_row, static_cast<bf16 *>(pool->k_pool),
                         static_cast<bf16 *>(pool->v_pool));
    else
      hipLaunchKernelGGL((k_kv_compact<float>), grid, dim3(64), 0, static_cast<hipStream_t>(stream), b->cu_q, b->seq_slot,
                         b->n_slots, b->seq_len, b->block_table, b->max_blocks_per_seq, pool->n_blocks, d.n_kv_heads,
                         b->tree_end, b->accept_len, b->stop_row, static_cast<float *>(pool->k_pool),
                         static_cast<float *>(pool->v_pool));
    HSD_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(k_kv_commit, dim3(1), dim3(1024), 0, static_cast<hipStream_t>(stream), b->n_seq, b->cu_q,
                     b->seq_slot, b->n_slots, b->seq_len, b->block_table, b->max_blocks_per_seq, pool->n_blocks, pool->free_list,
                     pool->free_count, b->accept_len, b->bonus, pending_out, 0);
  HSD_LAUNCH_CHECK();
  return HSD_OK;
}

}  // extern "C"
