// Shared device/host helpers for the rollout kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rlx {

typedef uint16_t h16_t;   // raw bit pattern of a 16-bit float: bf16 or IEEE fp16, fixed per model
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x4 h16x8;      // eight 16-bit floats as an MFMA operand (bit patterns)

constexpr int WAVE = 64;

// element formats of weights, KV pages and activation terms
enum { DT_BF16 = 0, DT_F16 = 1 };

// ---- bf16: the upper half of an fp32; round-to-nearest-even, inputs always finite ----
__device__ __forceinline__ float bf16_to_f32(h16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ h16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (h16_t)(u >> 16);
}
// ---- fp16: the hardware conversions (round-to-nearest-even; magnitudes past 65504 become infinities) ----
__device__ __forceinline__ float f16_to_f32(h16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
__device__ __forceinline__ h16_t f32_to_f16(float f) { return __builtin_bit_cast(h16_t, (_Float16)f); }

// format picked at compile time (inner loops) ...
template <int DT> __device__ __forceinline__ float h16_to_f32(h16_t b) { return DT == DT_F16 ? f16_to_f32(b) : bf16_to_f32(b); }
template <int DT> __device__ __forceinline__ h16_t f32_to_h16(float f) { return DT == DT_F16 ? f32_to_f16(f) : f32_to_bf16(f); }
// ... or at run time (uniform over a launch)
__device__ __forceinline__ float h16_to_f32(h16_t b, int dt) { return dt == DT_F16 ? f16_to_f32(b) : bf16_to_f32(b); }
__device__ __forceinline__ h16_t f32_to_h16(float f, int dt) { return dt == DT_F16 ? f32_to_f16(f) : f32_to_bf16(f); }

// v ~= hi + lo with both terms in the 16-bit format: the second term carries the next significand bits
template <int DT> __device__ __forceinline__ void split_h16(float v, h16_t& hi, h16_t& lo) {
  hi = f32_to_h16<DT>(v);
  lo = f32_to_h16<DT>(v - h16_to_f32<DT>(hi));
}
__device__ __forceinline__ void split_h16(float v, h16_t& hi, h16_t& lo, int dt) {
  hi = f32_to_h16(v, dt);
  lo = f32_to_h16(v - h16_to_f32(hi, dt), dt);
}

// matrix-core steps on bit-pattern operands
typedef __bf16 mfma_bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 mfma_f16x8 __attribute__((ext_vector_type(8)));
template <int DT> __device__ __forceinline__ f32x16 mfma_32x32x16(h16x8 a, h16x8 b, f32x16 c) {
  if (DT == DT_F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(mfma_f16x8, a), __builtin_bit_cast(mfma_f16x8, b), c, 0, 0, 0);
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mfma_bf16x8, a), __builtin_bit_cast(mfma_bf16x8, b), c, 0, 0, 0);
}
template <int DT> __device__ __forceinline__ f32x4 mfma_16x16x32(h16x8 a, h16x8 b, f32x4 c) {
  if (DT == DT_F16)
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(mfma_f16x8, a), __builtin_bit_cast(mfma_f16x8, b), c, 0, 0, 0);
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(mfma_bf16x8, a), __builtin_bit_cast(mfma_bf16x8, b), c, 0, 0, 0);
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

// 16-byte global load of eight 16-bit elements as an MFMA operand
__device__ __forceinline__ h16x8 load_h16x8(const h16_t* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ h16x8 zero_h16x8() { return u32x4{0u, 0u, 0u, 0u}; }
// The same load marked non-temporal, for data that a launch reads once (decode weights, the KV pages of a decode
// step): the lines are not kept in the caches, where they would only push out what is read again.  Measured: a
// kernel that only streams 768 MiB runs at 6.9 TB/s with this mark against 6.2 TB/s without it.
__device__ __forceinline__ u32x4 load_stream_16(const void* p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)); }
__device__ __forceinline__ u32x2 load_stream_8(const void* p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p)); }

// ---------------------------------------------------------------------------------
// Streaming layouts.  Both operands of the skinny GEMM are kept in the order the
// 32x32x16 MFMA consumes them, so that every wave-wide 16-byte load reads one
// contiguous 1 KB block:
//   fragment = 64 lanes x 8 elements; lane = (row mod 32) + 32 * ((k mod 16) / 8); element = k mod 8
// Weights  [N, K]: the 32-row tiles are taken four at a time (the four waves of a GEMM workgroup own one tile each)
//   and the fragments of such a group are interleaved along k, so that the workgroup reads one contiguous run of
//   4 KB per k-step instead of four runs that lie one tile apart (measured: the same bytes stream 3-5 % faster):
//   fragment index ((n / 128) * (K / 16) + k / 16) * 4 + (n / 32) % 4       (rows padded to 128)
// Activations [T, K] as `planes` 16-bit terms: fragment index ((k / 16) * ceil(T / 32) + t / 32) * planes + p
// K must be a multiple of 16.
// ---------------------------------------------------------------------------------
constexpr int W_GROUP = 4;                                   // 32-row tiles per interleaved group
constexpr int W_KSTRIDE = W_GROUP * 512;                      // elements between consecutive k-steps of one tile
__host__ __device__ __forceinline__ size_t packed_weight_elems(int N, int K) {
  return (size_t)((N + 32 * W_GROUP - 1) / (32 * W_GROUP)) * (size_t)(K / 16) * (size_t)W_KSTRIDE;
}
// first element of fragment (tile nt, k-step 0); k-step ks lies ks * W_KSTRIDE elements further
__host__ __device__ __forceinline__ size_t packed_tile_offset(int nt, int KS) {
  return ((size_t)(nt / W_GROUP) * (size_t)KS * W_GROUP + (size_t)(nt % W_GROUP)) * 512;
}
__host__ __device__ __forceinline__ size_t packed_weight_offset(int n, int k, int K) {
  return packed_tile_offset(n >> 5, K >> 4) + (size_t)(k >> 4) * W_KSTRIDE +
         (size_t)((n & 31) + 32 * ((k >> 3) & 1)) * 8 + (size_t)(k & 7);
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
