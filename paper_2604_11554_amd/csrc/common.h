// Shared device/host helpers for the rollout kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rlx {

typedef uint16_t bf16_t;  // raw bf16 bit pattern
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int WAVE = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even; inputs here are always finite
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// v ~= hi + lo with both terms bf16: the second term carries the next 8 significand bits
__device__ __forceinline__ void split_bf16(float v, bf16_t& hi, bf16_t& lo) {
  hi = f32_to_bf16(v);
  lo = f32_to_bf16(v - bf16_to_f32(hi));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

// 16-byte global load of eight bf16 as an MFMA operand
__device__ __forceinline__ bf16x8 load_bf16x8(const bf16_t* p) {
  u32x4 v = *reinterpret_cast<const u32x4*>(p);
  return __builtin_bit_cast(bf16x8, v);
}
__device__ __forceinline__ bf16x8 zero_bf16x8() {
  u32x4 v = {0u, 0u, 0u, 0u};
  return __builtin_bit_cast(bf16x8, v);
}

// ---------------------------------------------------------------------------------
// Streaming layouts.  Both operands of the skinny GEMM are kept in the order the
// 32x32x16 MFMA consumes them, so that every wave-wide 16-byte load reads one
// contiguous 1 KB block:
//   fragment = 64 lanes x 8 bf16; lane = (row mod 32) + 32 * ((k mod 16) / 8); element = k mod 8
// Weights  [N, K]: fragment index (n / 32) * (K / 16) + k / 16           (rows padded to 32)
// Activations [T, K] as `planes` bf16 terms: fragment index ((k / 16) * ceil(T / 32) + t / 32) * planes + p
// K must be a multiple of 16.
// ---------------------------------------------------------------------------------
__host__ __device__ __forceinline__ size_t packed_weight_elems(int N, int K) {
  return (size_t)((N + 31) / 32) * (size_t)(K / 16) * 512;
}
__host__ __device__ __forceinline__ size_t packed_weight_offset(int n, int k, int K) {
  return (((size_t)(n >> 5) * (size_t)(K >> 4) + (size_t)(k >> 4)) * 64 + (size_t)((n & 31) + 32 * ((k >> 3) & 1))) * 8 +
         (size_t)(k & 7);
}
__host__ __device__ __forceinline__ size_t frag_act_elems(int T, int K, int planes) {
  return (size_t)(K / 16) * (size_t)((T + 31) / 32) * (size_t)planes * 512;
}
// offset of the 8-element group holding (t, k..k+7), k a multiple of 8, of plane p
__host__ __device__ __forceinline__ size_t frag_act_offset(int t, int k, int p, int mtiles, int planes) {
  return ((((size_t)(k >> 4) * (size_t)mtiles + (size_t)(t >> 5)) * (size_t)planes + (size_t)p) * 64 +
          (size_t)((t & 31) + 32 * ((k >> 3) & 1))) * 8;
}

}  // namespace rlx
