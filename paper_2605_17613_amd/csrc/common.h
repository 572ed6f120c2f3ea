// Shared host-side helpers of the library: error reporting and argument checks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/vericache.h"

namespace vc {

constexpr int kHeadDim = 128;
constexpr int kRecordBytes = 5120;
constexpr int kPartialFloats = 130;  // m, l, O[128] of one split of one (row, head)

// Thread-local message of the last failing call.
char* err_buf();
vc_status fail(vc_status st, const char* fmt, ...);
vc_status hip_fail(hipError_t e, const char* what);

#define VC_HIP(call)                                              \
  do {                                                            \
    hipError_t e__ = (call);                                      \
    if (e__ != hipSuccess) return ::vc::hip_fail(e__, #call);     \
  } while (0)

#define VC_REQUIRE(cond, st, ...)                                 \
  do {                                                            \
    if (!(cond)) return ::vc::fail(st, __VA_ARGS__);              \
  } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Streaming accesses: data that a kernel touches exactly once is loaded / stored with the
// non-temporal hint, so that it is not kept in the caches it passes through (measured on this GPU: a
// read-once stream runs 10 - 14 % faster with the hint than with the default policy).
typedef uint32_t stream_u32x4 __attribute__((ext_vector_type(4)));
typedef float stream_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_stream(const uint4* p) {
  const stream_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const stream_u32x4*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ float4 ld_stream(const float4* p) {
  const stream_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const stream_f32x4*>(p));
  return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ float ld_stream(const float* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void st_stream(uint4* p, const uint4& v) {
  stream_u32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<stream_u32x4*>(p));
}

// Launch-shape tunables.  Each is read from the environment variable of its name once, when the
// library first needs one (thread safe), and can be overridden with vc_set_tunable; the hot path
// only reads an atomic integer.  tunable() returns the set value if it lies in [lo, hi], else `dflt`.
enum Tunable {
  kTunDraftBf16Wgs, kTunDraftQuantWgs, kTunDraftMinTok, kTunDraftMinBlk, kTunDraftFlat, kTunDraftRowWaves, kTunDraftFused,
  kTunDraftTailSplit,
  kTunVerifyWgs, kTunVerifyMinTok, kTunVerifyWorklist, kTunVerifyListMin, kTunVerifyTaper, kTunVerifyQueueWgs,
  kTunAcceptFused,
  kNumTunables
};
int tunable(Tunable t, int dflt, int lo, int hi);

// One-time per-device set-up of the kernels that need more than the default dynamic LDS (called by
// vc_create with the device current).
vc_status draft_init_device();
vc_status verify_init_device();

}  // namespace vc

struct vc_ctx {
  int device;
  hipStream_t copy_stream;
  // ring of chunk events; ticket t uses events[t % kRing]
  static constexpr int kRing = 4096;
  hipEvent_t* events;  // created on first use
  int64_t issued;  // next ticket
  // armed by vc_time_main_kernel: events recorded around the main kernel(s) of the next attention call
  hipEvent_t time_begin, time_end;
  int n_cu;                // compute units of the device
  // vc_mark / vc_swap_after: events recorded on compute streams for the copy stream to wait on
  static constexpr int kMarkRing = 1024;
  hipEvent_t mark_events[kMarkRing];
  int64_t marks_issued;
  // vc_accept_len: counters (zero between calls) on which the workgroups of a fused launch count
  // themselves: call i uses slot i % kAcceptCounters = one counter for the launch and one per row,
  // each on a cache line of its own
  static constexpr int kAcceptCounters = 16, kAcceptCounterStride = 16, kAcceptMaxRows = 2048;
  static constexpr int kAcceptSlotWords = (1 + kAcceptMaxRows) * kAcceptCounterStride;
  unsigned int* accept_counters;
  uint64_t accept_calls;
  // vc_draft_attn: the same for the fused finish of small launches: one counter per (sequence, KV head)
  static constexpr int kDraftCounterSets = 16, kDraftMaxLists = 256, kDraftCounterStride = 16;
  unsigned int* draft_counters;
  uint64_t draft_calls;
};

namespace vc {
// Record the armed timing events (if any) on `st`; the end mark disarms.
inline void mark_begin(vc_ctx* c, hipStream_t st) { if (c->time_begin) (void)hipEventRecord(c->time_begin, st); }
inline void mark_end(vc_ctx* c, hipStream_t st) {
  if (c->time_end) (void)hipEventRecord(c->time_end, st);
  c->time_begin = nullptr; c->time_end = nullptr;
}
}  // namespace vc

