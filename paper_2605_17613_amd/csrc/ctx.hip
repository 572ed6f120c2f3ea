// Context, error reporting and the full-KV reload (swap-in) path.
//
// Swap-in follows the paper's runtime loop (section 5.2 step (i), section 4.2.1): the full KV of
// a request sits in CPU memory and is reloaded asynchronously while other work drafts.  Here each
// chunk is one hipMemcpyAsync on a dedicated copy stream followed by one event; compute streams
// wait on the event of the chunk they need, so the host never blocks.
#include <stdarg.h>
#include <stdlib.h>

#include "common.h"

namespace vc {

char* err_buf() {
  static thread_local char buf[512] = "";
  return buf;
}

vc_status fail(vc_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(err_buf(), 512, fmt, ap);
  va_end(ap);
  return st;
}

vc_status hip_fail(hipError_t e, const char* what) {
  snprintf(err_buf(), 512, "%s: %s", what, hipGetErrorString(e));
  return VC_ERR_HIP;
}

int env_int(const char* name, int dflt, int lo, int hi) {
  const char* s = getenv(name);
  if (!s || !*s) return dflt;
  char* end = nullptr;
  long v = strtol(s, &end, 10);
  if (end == s || v < lo || v > hi) return dflt;
  return static_cast<int>(v);
}

}  // namespace vc

using namespace vc;

extern "C" const char* vc_last_error(void) { return err_buf(); }
extern "C" const char* vc_version(void) { return "0.1"; }

extern "C" vc_status vc_create(int device, vc_ctx** out) {
  VC_REQUIRE(out != nullptr, VC_ERR_INVALID_ARG, "vc_create: out is NULL");
  *out = nullptr;
  int count = 0;
  VC_HIP(hipGetDeviceCount(&count));
  VC_REQUIRE(device >= 0 && device < count, VC_ERR_INVALID_ARG, "vc_create: device %d of %d", device, count);
  VC_HIP(hipSetDevice(device));
  vc_ctx* c = static_cast<vc_ctx*>(calloc(1, sizeof(vc_ctx)));
  VC_REQUIRE(c != nullptr, VC_ERR_INVALID_ARG, "vc_create: out of host memory");
  c->device = device;
  hipError_t e = hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking);
  if (e != hipSuccess) {
    free(c);
    return hip_fail(e, "hipStreamCreateWithFlags");
  }
  c->events = static_cast<hipEvent_t*>(calloc(vc_ctx::kRing, sizeof(hipEvent_t)));
  c->issued = 0;
  *out = c;
  return VC_OK;
}

extern "C" vc_status vc_time_main_kernel(vc_ctx* c, void* begin_event, void* end_event) {
  VC_REQUIRE(c != nullptr, VC_ERR_INVALID_ARG, "vc_time_main_kernel: ctx is NULL");
  VC_REQUIRE((begin_event == nullptr) == (end_event == nullptr), VC_ERR_INVALID_ARG,
             "vc_time_main_kernel: pass both events or neither");
  c->time_begin = static_cast<hipEvent_t>(begin_event);
  c->time_end = static_cast<hipEvent_t>(end_event);
  return VC_OK;
}

extern "C" vc_status vc_destroy(vc_ctx* c) {
  if (!c) return VC_OK;
  (void)hipStreamSynchronize(c->copy_stream);
  for (int i = 0; i < vc_ctx::kRing; ++i)
    if (c->events[i]) (void)hipEventDestroy(c->events[i]);
  (void)hipStreamDestroy(c->copy_stream);
  free(c->events);
  free(c);
  return VC_OK;
}

extern "C" vc_status vc_swap_in(vc_ctx* c, const void* host_src, void* dev_dst, const vc_chunk* chunks,
                                int32_t n_chunks, int64_t* first_ticket) {
  VC_REQUIRE(c && first_ticket, VC_ERR_INVALID_ARG, "vc_swap_in: ctx or first_ticket is NULL");
  VC_REQUIRE(n_chunks >= 0, VC_ERR_INVALID_ARG, "vc_swap_in: n_chunks %d", n_chunks);
  *first_ticket = c->issued;
  if (n_chunks == 0) return VC_OK;
  VC_REQUIRE(host_src && dev_dst && chunks, VC_ERR_INVALID_ARG, "vc_swap_in: NULL pointer");
  hipPointerAttribute_t at;
  hipError_t e = hipPointerGetAttributes(&at, host_src);
  if (e != hipSuccess || at.type != hipMemoryTypeHost) {
    (void)hipGetLastError();  // a pageable pointer leaves an error behind; clear it
    return fail(VC_ERR_INVALID_ARG, "vc_swap_in: host_src is not pinned host memory");
  }
  e = hipPointerGetAttributes(&at, dev_dst);
  if (e != hipSuccess || at.type != hipMemoryTypeDevice) {
    (void)hipGetLastError();
    return fail(VC_ERR_INVALID_ARG, "vc_swap_in: dev_dst is not device memory");
  }
  // outstanding = issued tickets whose event has not completed; the ring slot we are about to
  // reuse must have landed
  VC_REQUIRE(n_chunks <= vc_ctx::kRing, VC_ERR_INVALID_ARG, "vc_swap_in: more than %d chunks", vc_ctx::kRing);
  int64_t oldest_needed = c->issued + n_chunks - vc_ctx::kRing;  // tickets below this get overwritten
  if (oldest_needed > 0) {
    hipEvent_t ev = c->events[(oldest_needed - 1) % vc_ctx::kRing];
    if (ev && hipEventQuery(ev) != hipSuccess) {
      (void)hipGetLastError();
      return fail(VC_ERR_INVALID_ARG, "vc_swap_in: more than %d tickets outstanding", vc_ctx::kRing);
    }
  }
  VC_HIP(hipSetDevice(c->device));
  for (int i = 0; i < n_chunks; ++i) {
    const vc_chunk& ch = chunks[i];
    int slot = static_cast<int>(c->issued % vc_ctx::kRing);
    if (!c->events[slot]) VC_HIP(hipEventCreateWithFlags(&c->events[slot], hipEventDisableTiming));
    if (ch.bytes)
      VC_HIP(hipMemcpyAsync(static_cast<char*>(dev_dst) + ch.dst_off, static_cast<const char*>(host_src) + ch.src_off,
                            ch.bytes, hipMemcpyHostToDevice, c->copy_stream));
    VC_HIP(hipEventRecord(c->events[slot], c->copy_stream));
    c->issued++;
  }
  return VC_OK;
}

static vc_status ticket_event(vc_ctx* c, int64_t ticket, hipEvent_t* ev, const char* who) {
  VC_REQUIRE(c != nullptr, VC_ERR_INVALID_ARG, "%s: ctx is NULL", who);
  VC_REQUIRE(ticket >= 0 && ticket < c->issued, VC_ERR_INVALID_ARG, "%s: ticket %lld was never issued", who,
             static_cast<long long>(ticket));
  // a ticket older than one ring has certainly landed (its slot was checked before reuse)
  *ev = (c->issued - ticket > vc_ctx::kRing) ? nullptr : c->events[ticket % vc_ctx::kRing];
  return VC_OK;
}

extern "C" vc_status vc_swap_wait(vc_ctx* c, int64_t ticket, void* stream) {
  hipEvent_t ev;
  vc_status st = ticket_event(c, ticket, &ev, "vc_swap_wait");
  if (st != VC_OK) return st;
  if (ev) VC_HIP(hipStreamWaitEvent(static_cast<hipStream_t>(stream), ev, 0));
  return VC_OK;
}

extern "C" vc_status vc_swap_query(vc_ctx* c, int64_t ticket) {
  hipEvent_t ev;
  vc_status st = ticket_event(c, ticket, &ev, "vc_swap_query");
  if (st != VC_OK) return st;
  if (!ev) return VC_OK;
  hipError_t e = hipEventQuery(ev);
  if (e == hipSuccess) return VC_OK;
  if (e == hipErrorNotReady) {
    (void)hipGetLastError();
    return fail(VC_ERR_NOT_READY, "vc_swap_query: ticket %lld has not landed", static_cast<long long>(ticket));
  }
  return hip_fail(e, "hipEventQuery");
}

extern "C" vc_status vc_swap_sync(vc_ctx* c) {
  VC_REQUIRE(c != nullptr, VC_ERR_INVALID_ARG, "vc_swap_sync: ctx is NULL");
  VC_HIP(hipStreamSynchronize(c->copy_stream));
  return VC_OK;
}
