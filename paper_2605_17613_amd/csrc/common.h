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

// Integer tunable read once from the environment (sweeps); `dflt` when unset or invalid.
int env_int(const char* name, int dflt, int lo, int hi);

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
};

namespace vc {
// Record the armed timing events (if any) on `st`; the end mark disarms.
inline void mark_begin(vc_ctx* c, hipStream_t st) { if (c->time_begin) (void)hipEventRecord(c->time_begin, st); }
inline void mark_end(vc_ctx* c, hipStream_t st) {
  if (c->time_end) (void)hipEventRecord(c->time_end, st);
  c->time_begin = nullptr; c->time_end = nullptr;
}
}  // namespace vc

