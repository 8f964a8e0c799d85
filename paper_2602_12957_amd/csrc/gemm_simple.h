// Plain LDS-tiled GEMM with fp32 FMA accumulation: C[m,n] = sum_k A[m,k] * W[n,k].
// This is the fp32 debug path (model dtype fp32) and the cross-check for the bf16 MFMA kernel.
// Tile 64x64x32, 256 threads; thread (ty, tx) owns rows ty*8..ty*8+7 and the column pair (tx, tx+32).
#pragma once

#include "common.h"
#include "epilogues.h"

namespace hsd {

__device__ __forceinline__ void load8(const float *p, float *out) {
  float4 a = reinterpret_cast<const float4 *>(p)[0];
  float4 b = reinterpret_cast<const float4 *>(p)[1];
  out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
  out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16 *p, float *out) {
  uint4 r = reinterpret_cast<const uint4 *>(p)[0];
  uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(w[i] << 16);
    out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}

// grid: (N/64, ceil(M/64)).  Requirements checked by the host: N % 64 == 0, K % 32 == 0.
// For Epi::kDual the second weight block starts N rows after the first (W is [2N, K]: gate | up).
template <typename T, typename Epi>
__global__ void __launch_bounds__(256) k_gemm_simple(int M, int N, int K, const T *__restrict__ A,
                                                     const T *__restrict__ W, Epi epi) {
  constexpr int BK = 32;
  __shared__ float As[64][BK + 1];
  __shared__ float Bs[64][BK + 1];
  __shared__ float Bs2[Epi::kDual ? 64 : 1][BK + 1];
  const int t = threadIdx.x, tx = t & 31, ty = t >> 5;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int lr = t >> 2, lk = (t & 3) * 8;

  float acc[8][2], acc2[8][2];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i][0] = acc[i][1] = acc2[i][0] = acc2[i][1] = 0.f;

  for (int k0 = 0; k0 < K; k0 += BK) {
    float va[8], vb[8], vb2[8];
    if (m0 + lr < M) {
      load8(A + static_cast<size_t>(m0 + lr) * K + k0 + lk, va);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) va[i] = 0.f;
    }
    load8(W + static_cast<size_t>(n0 + lr) * K + k0 + lk, vb);
    if (Epi::kDual) load8(W + static_cast<size_t>(N + n0 + lr) * K + k0 + lk, vb2);
    __syncthreads();  // previous tile fully consumed
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      As[lr][lk + i] = va[i];
      Bs[lr][lk + i] = vb[i];
      if (Epi::kDual) Bs2[lr][lk + i] = vb2[i];
    }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < BK; ++kk) {
      float b0 = Bs[tx][kk], b1 = Bs[tx + 32][kk];
      float c0 = 0.f, c1 = 0.f;
      if (Epi::kDual) {
        c0 = Bs2[tx][kk];
        c1 = Bs2[tx + 32][kk];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float a = As[ty * 8 + i][kk];
        acc[i][0] = fmaf(a, b0, acc[i][0]);
        acc[i][1] = fmaf(a, b1, acc[i][1]);
        if (Epi::kDual) {
          acc2[i][0] = fmaf(a, c0, acc2[i][0]);
          acc2[i][1] = fmaf(a, c1, acc2[i][1]);
        }
      }
    }
  }

  if constexpr (std::is_same<Epi, EpiLMHead>::value) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int m = m0 + ty * 8 + i;
      Top2 tp = top2_init();
      top2_push(tp, acc[i][0], n0 + tx);
      top2_push(tp, acc[i][1], n0 + tx + 32);
      if (m < M) epi.dump(m, n0 + tx, acc[i][0], acc[i][1]);
      if (m < M && epi.want_logit != nullptr) {
        const float v0 = acc[i][0], v1 = acc[i][1];
        epi.capture(m, [&](int want, float &out) {
          if (want == n0 + tx) { out = v0; return true; }
          if (want == n0 + tx + 32) { out = v1; return true; }
          return false;
        });
      }
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) {  // stays inside the 32 lanes that share this row
        Top2 u;
        u.m1 = __shfl_xor(tp.m1, o, kWave);
        u.i1 = __shfl_xor(tp.i1, o, kWave);
        u.m2 = __shfl_xor(tp.m2, o, kWave);
        tp = top2_merge(tp, u);
      }
      if (tx == 0 && m < M) epi.part[static_cast<size_t>(m) * epi.n_tiles + blockIdx.x] = tp;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int m = m0 + ty * 8 + i;
      if (m >= M) continue;
      if constexpr (Epi::kDual) {
        epi.pair2(m, n0 + tx, acc[i][0], acc[i][1], acc2[i][0], acc2[i][1]);
      } else {
        epi.pair(m, n0 + tx, acc[i][0], acc[i][1]);
      }
    }
  }
}

}  // namespace hsd
