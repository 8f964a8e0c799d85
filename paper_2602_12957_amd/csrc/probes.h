// Hardware probes: four small kernels that measure, on the chip the library runs on, the rates the GEMM and attention
// rooflines are judged against -- what the matrix pipes sustain when every compute unit runs them (the clock drops
// under that load), what a compute unit's load path takes in from L2, and what its LDS delivers.  Measurement
// helpers, not a step of the method; the caller times the launch.
#pragma once

#include "gemm_mfma_d.h"

namespace hsd {

// kind 0: every wave issues 16 MFMAs (four independent accumulator chains) per iteration, no memory traffic.
// 32768 flop per MFMA and wave.
__global__ void __launch_bounds__(256) k_probe_mfma(int iters, float *sink) {
  const int lane = threadIdx.x & 63;
  floatx16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  bf16x8 fa, fb;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    fa[e] = static_cast<__bf16>(1.0f + lane * 0.001f);
    fb[e] = static_cast<__bf16>(lane * 0.01f - 0.3f);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[j & 3], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) s += acc[i][0];
  if (s == 12345.678f) sink[0] = s;   // never true: keeps the chains alive
}

// kinds 1 and 2: every workgroup (256 threads) streams the region of its XCD (workgroup b reads region b % 8, small
// enough to stay in L2) with 16-byte loads, 32 KB per iteration -- into registers (kind 1) or straight into LDS
// (kind 2).  region_bytes is a multiple of 32 KB.
template <bool TO_LDS>
__global__ void __launch_bounds__(256) k_probe_load(const unsigned char *src, int region_bytes, int iters, float *sink) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int t = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(src + static_cast<size_t>(blockIdx.x % 8) * region_bytes, region_bytes);
  const LdsBytePtr lds = (LdsBytePtr)smem_raw;
  floatx4 acc = {0.f, 0.f, 0.f, 0.f};
  int off = static_cast<int>((static_cast<size_t>(blockIdx.x >> 3) * 32768) % region_bytes);
  for (int it = 0; it < iters; ++it) {
    if (TO_LDS) {
#pragma unroll
      for (int j = 0; j < 8; ++j) lds_load16(rs, lds + wave * 8192 + j * 1024, off + j * 4096 + t * 16, 0);
    } else {
      floatx4 v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j)
        v[j] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs, off + j * 4096 + t * 16, 0, 0));
#pragma unroll
      for (int j = 0; j < 8; ++j) acc += v[j];
    }
    off += 32768;
    if (off >= region_bytes) off = 0;
  }
  HSD_VMCNT(0);
  if (acc[0] == 12345.678f) sink[0] = acc[1];
}

// kind 3: every wave reads 8 KB of LDS per iteration with conflict-free 128-bit reads.
__global__ void __launch_bounds__(1024) k_probe_lds(int iters, float *sink) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int t = threadIdx.x;
  for (int i = t; i < 16384; i += blockDim.x) reinterpret_cast<float *>(smem_raw)[i] = static_cast<float>(i);
  __syncthreads();
  const unsigned char *p = smem_raw + (t & 63) * 16 + ((t >> 6) & 7) * 8192;
  floatx4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
    floatx4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = *reinterpret_cast<const floatx4 *>(p + j * 1024);
#pragma unroll
    for (int j = 0; j < 8; ++j) asm volatile("" ::"v"(v[j]));
    acc += v[0];
  }
  if (acc[0] == 12345.678f) sink[0] = acc[1];
}

}  // namespace hsd
