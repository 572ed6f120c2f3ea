// Device-side helpers shared by the attention kernels: vector types, wave reductions, the split
// partial format and its merge.
//
// Split partial of one (row, q head, split): 130 floats
//   [0] m   running maximum of the scores, in the log2 domain (score * log2(e))
//   [1] l   sum of 2^(s - m)
//   [2..130) O[128], the un-normalised output sum of 2^(s - m) * V
// Splits over the context are merged by the usual log-sum-exp weighting (flash-decoding style).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vc {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// running maximum before any key was seen: finite, so 2^(s - m) and 2^(m_old - m_new) need no
// special cases (2^(-1e30 - x) is 0, and -inf - (-1e30) is -inf)
constexpr float kNoKeyYet = -1.0e30f;

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }

// float -> bf16 bits, round to nearest even (inputs are finite here)
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ __forceinline__ int ceil_div_dev(int a, int b) { return (a + b - 1) / b; }

// 2^(a - b) that is 0 (not NaN) when a = -inf, whatever b is
__device__ __forceinline__ float exp2_diff(float a, float b) { return (a == -INFINITY) ? 0.f : exp2f(a - b); }

}  // namespace vc
