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

// ---- LDS accesses by raw LDS byte address, and direct HBM -> LDS loads ----
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x4v lds_u32x4v;
typedef __attribute__((address_space(3))) u32x2v lds_u32x2v;
typedef __attribute__((address_space(3))) short4v lds_short4v;
__device__ __forceinline__ u32x4v lds_load_u32x4(uint32_t addr) {   // ds_read_b128
  return *reinterpret_cast<const lds_u32x4v*>(static_cast<size_t>(addr));
}
__device__ __forceinline__ u32x2v lds_load_u32x2(uint32_t addr) {   // ds_read_b64
  return *reinterpret_cast<const lds_u32x2v*>(static_cast<size_t>(addr));
}
__device__ __forceinline__ uint32_t lds_address(const void* shared_ptr) {
  return static_cast<uint32_t>(reinterpret_cast<size_t>((const __attribute__((address_space(3))) char*)shared_ptr));
}

// Direct HBM -> LDS load of 16 bytes per lane: lane i's data lands at lds_addr + 16*i (lds_addr is
// wave-uniform and travels in M0).  Issued as inline assembly so that the compiler's own wait-count
// bookkeeping does not force every later LDS read to wait for all loads in flight; the rings built
// on this wait for exactly the data they are about to read (wait_vm).
// Every KV byte is read once per call, so the loads carry the non-temporal hint: the lines are not
// kept in the caches they pass through.  Measured on the int4 record kernel: 231 -> 203 us (6.6 TB/s),
// past what default-policy loads reach on a plain streaming read (6.2 TB/s).
__device__ __forceinline__ void load_to_lds(const uint16_t* gsrc, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" : : "s"(lds_addr), "v"(gsrc) : "memory");
}
// Same with a wave-uniform 64-bit base plus a 32-bit per-lane byte offset.
__device__ __forceinline__ void load_to_lds(const uint8_t* gbase_uniform, uint32_t lane_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
               : : "s"(lds_addr), "v"(lane_off), "s"(gbase_uniform) : "memory");
}
// Same, four bytes per lane: lane i's word lands at lds_addr + 4*i.  (Default cache policy: the kept-index
// lists it brings in measured 0.4 us per call slower with the non-temporal hint.)
__device__ __forceinline__ void load_to_lds_b32(const int* gsrc, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" : : "s"(lds_addr), "v"(gsrc) : "memory");
}

// Wait until at most N_OUTSTANDING vector-memory operations of this wave are in flight (they
// complete in order, so everything older has landed).  A compiler-level memory barrier as well:
// no LDS read may move above the wait that makes its data valid.
template <int N_OUTSTANDING>
__device__ __forceinline__ void wait_vm() {
  static_assert(N_OUTSTANDING >= 0 && N_OUTSTANDING < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N_OUTSTANDING) : "memory");
}
// every LDS read issued so far has returned (needed before a direct load may overwrite what they read)
__device__ __forceinline__ void wait_lds_reads() { asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory"); }

}  // namespace vc
