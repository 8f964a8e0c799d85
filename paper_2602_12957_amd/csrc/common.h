// Shared device helpers for the HSD verification kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/hsd.h"

namespace hsd {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kHd = HSD_HEAD_DIM;
constexpr int kBlk = HSD_KV_BLOCK_TOKENS;

// native vector types (kept in VGPRs as whole registers; HIP's uint4 / float4 structs are not)
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// bf16 is handled as raw 16-bit patterns; arithmetic is always fp32.
struct bf16 {
  uint16_t v;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

// round-to-nearest-even; inputs on this path are finite
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return bf16_to_f32(x.v); }

template <typename T>
__device__ __forceinline__ T from_f32(float x);
template <>
__device__ __forceinline__ float from_f32<float>(float x) {
  return x;
}
template <>
__device__ __forceinline__ bf16 from_f32<bf16>(float x) {
  bf16 r;
  r.v = f32_to_bf16(x);
  return r;
}

// Consecutive outputs of one row written as one 16-byte piece (dst 16-byte aligned): 4 floats, or 8 values
// converted to bf16 with the hardware round-to-nearest-even conversion (same rounding as f32_to_bf16).
__device__ __forceinline__ void store_row(float *dst, const float (&v)[4]) {
  floatx4 f = {v[0], v[1], v[2], v[3]};
  *reinterpret_cast<floatx4 *>(dst) = f;
}
__device__ __forceinline__ void store_row(bf16 *dst, const float (&v)[8]) {
  floatx8 f = {v[0], v[1], v[2], v[3], v[4], v[5], v[6], v[7]};
  *reinterpret_cast<bf16x8 *>(dst) = __builtin_convertvector(f, bf16x8);
}
__device__ __forceinline__ void store_row(float *dst, const float (&v)[8]) {
  floatx4 f0 = {v[0], v[1], v[2], v[3]}, f1 = {v[4], v[5], v[6], v[7]};
  *reinterpret_cast<floatx4 *>(dst) = f0;
  *reinterpret_cast<floatx4 *>(dst + 4) = f1;
}

// Exchange between the two lane halves (lane l and lane l ^ 32) in one cross-lane instruction, no LDS round trip:
// v_permlane32_swap hands back (x of lane l % 32, x of lane 32 + l % 32) in every lane.
__device__ __forceinline__ float half_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Per-row top-2 record used by the LM-head arg-max: largest value m1 at index i1 (lowest index among
// equal maxima), second largest value m2 (may equal m1 when the maximum occurs twice).
struct Top2 {
  float m1;
  int i1;
  float m2;
};

__device__ __forceinline__ Top2 top2_init() { return Top2{-INFINITY, 0x7fffffff, -INFINITY}; }

__device__ __forceinline__ void top2_push(Top2 &t, float v, int idx) {
  if (v > t.m1 || (v == t.m1 && idx < t.i1)) {
    t.m2 = t.m1;
    t.m1 = v;
    t.i1 = idx;
  } else if (v > t.m2) {
    t.m2 = v;
  }
}

__device__ __forceinline__ Top2 top2_merge(const Top2 &a, const Top2 &b) {
  Top2 r;
  bool a_first = (a.m1 > b.m1) || (a.m1 == b.m1 && a.i1 <= b.i1);
  if (a_first) {
    r.m1 = a.m1;
    r.i1 = a.i1;
    r.m2 = fmaxf(a.m2, b.m1);
  } else {
    r.m1 = b.m1;
    r.i1 = b.i1;
    r.m2 = fmaxf(b.m2, a.m1);
  }
  return r;
}

// State row (seq_len / block_table row) of batch sequence s; out-of-range entries are clamped so that no
// kernel can index outside the state arrays (the reservation kernel reports them in the status word).
__device__ __forceinline__ int slot_of(const int32_t *seq_slot, int s, int n_slots) {
  int sl = seq_slot ? seq_slot[s] : s;
  return sl < 0 ? 0 : (sl >= n_slots ? n_slots - 1 : sl);
}

// Per-row metadata built once per pass.
struct RowMeta {
  const int32_t *row_seq;  // [T] state row (slot) of the row's sequence
  const int32_t *row_pos;  // [T] absolute position of the row in its sequence (what the rotary embedding sees)
  const float2 *rope_cs;   // [T][32] (cos, sin) of pos * theta^(-2i/64)
  const int32_t *row_kv;   // [T] 16 * (block id holding the row's cache slot) + slot % 16, or -1 if no valid block
  const int32_t *row_slot; // [T] cache slot of the row's K/V: committed length + index of the row in its block
  const int32_t *row_base; // [T] packed index of the first row of the row's block
  const int32_t *row_end;  // [T] packed index one past the row's subtree (packed prefix tree), or nullptr: chains
};

// Everything a kernel needs to find a (sequence, position) slot in the paged pools.
struct PagedKV {
  void *k_pool;
  void *v_pool;
  const int32_t *block_table;
  int32_t max_blocks_per_seq;
  int32_t n_blocks;
  int32_t n_kv_heads;
  int32_t layer;
};

// Element offset of the (layer, block, kv head) page in a pool laid out [n_layers][n_blocks][n_kv_heads][1024].
// A K page is [16 tokens][64 dims]; a V page is [64 dims][16 token slots] (see kv_v_slot).
__device__ __forceinline__ size_t kv_block_offset(const PagedKV &kv, int block, int kvh) {
  return ((static_cast<size_t>(kv.layer) * kv.n_blocks + block) * kv.n_kv_heads + kvh) * (kBlk * kHd);
}

// The V pages are stored transposed, [dim][16 token slots], with the tokens of a page in the order
// 0-3, 8-11, 4-7, 12-15: the order in which one lane half of a 32x32 MFMA result holds 16 consecutive keys,
// so that the attention kernel can feed probabilities and V^T to the second product without any shuffle.
__device__ __forceinline__ int kv_v_slot(int tok) { return ((tok >> 2) & 1) * 8 + (tok >> 3) * 4 + (tok & 3); }
// element offset of V(token, dim) inside a (block, kv head) page
__device__ __forceinline__ int kv_v_elem(int tok, int dim) { return dim * kBlk + kv_v_slot(tok); }

// Block id holding position `pos` of sequence s, or -1 if the table has no valid block there.
__device__ __forceinline__ int kv_lookup_block(const PagedKV &kv, int s, int pos) {
  int bi = pos / kBlk;
  if (bi >= kv.max_blocks_per_seq) return -1;
  int b = kv.block_table[static_cast<size_t>(s) * kv.max_blocks_per_seq + bi];
  return (b >= 0 && b < kv.n_blocks) ? b : -1;
}

}  // namespace hsd
