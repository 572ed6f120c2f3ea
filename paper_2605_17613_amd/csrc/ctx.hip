// Context, error reporting and the full-KV reload (swap-in) path.
//
// Swap-in follows the paper's runtime loop (section 5.2 step (i), section 4.2.1): the full KV of
// a request sits in CPU memory and is reloaded asynchronously while other work drafts.  Here each
// chunk is one hipMemcpyAsync on a dedicated copy stream followed by one event; compute streams
// wait on the event of the chunk they need, so the host never blocks.
#include <limits.h>
#include <stdarg.h>
#include <stdlib.h>

#include <atomic>

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

namespace {
const char* const kTunableNames[kNumTunables] = {
    "VC_DRAFT_BF16_WGS", "VC_DRAFT_QUANT_WGS", "VC_DRAFT_MIN_TOK", "VC_DRAFT_MIN_BLK", "VC_DRAFT_FLAT", "VC_DRAFT_ROW_WAVES", "VC_DRAFT_FUSED",
    "VC_DRAFT_TAIL_SPLIT",
    "VC_VERIFY_WGS", "VC_VERIFY_MIN_TOK", "VC_VERIFY_WORKLIST", "VC_VERIFY_LIST_MIN", "VC_VERIFY_TAPER", "VC_VERIFY_QUEUE_WGS",
    "VC_ACCEPT_FUSED"};
constexpr int kUnset = INT_MIN;

struct TunableTable {
  std::atomic<int> value[kNumTunables];
  TunableTable() {
    for (int i = 0; i < kNumTunables; ++i) {
      int v = kUnset;
      const char* s = getenv(kTunableNames[i]);
      if (s && *s) {
        char* end = nullptr;
        const long x = strtol(s, &end, 10);
        if (end != s && x >= 0 && x <= INT_MAX) v = static_cast<int>(x);
      }
      value[i].store(v, std::memory_order_relaxed);
    }
  }
};
TunableTable& tunables() {
  static TunableTable table;    // constructed once, thread safe
  return table;
}
int tunable_index(const char* name) {
  if (!name) return -1;
  for (int i = 0; i < kNumTunables; ++i)
    if (strcmp(name, kTunableNames[i]) == 0) return i;
  return -1;
}
}  // namespace

int tunable(Tunable t, int dflt, int lo, int hi) {
  const int v = tunables().value[t].load(std::memory_order_relaxed);
  return (v == kUnset || v < lo || v > hi) ? dflt : v;
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
  vc_status st = c->events ? VC_OK : fail(VC_ERR_INVALID_ARG, "vc_create: out of host memory");
  // the kernels' LDS attributes are per device: set them here, once per context, so that no attention
  // call ever has to (a first call made under stream capture could not)
  if (st == VC_OK) st = draft_init_device();
  if (st == VC_OK) st = verify_init_device();
  if (st == VC_OK) {
    int cus = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
    if (e != hipSuccess) st = hip_fail(e, "hipDeviceGetAttribute");
    c->n_cu = cus;
  }
  if (st == VC_OK) {
    const size_t bytes = sizeof(unsigned int) * vc_ctx::kAcceptCounters * vc_ctx::kAcceptSlotWords;
    e = hipMalloc(reinterpret_cast<void**>(&c->accept_counters), bytes);
    if (e == hipSuccess) e = hipMemset(c->accept_counters, 0, bytes);   // synchronous: done before any call
    if (e != hipSuccess) st = hip_fail(e, "vc_create: accept counters");
  }
  if (st == VC_OK) {
    const size_t bytes = sizeof(unsigned int) * vc_ctx::kDraftCounterSets * vc_ctx::kDraftMaxLists * vc_ctx::kDraftCounterStride;
    e = hipMalloc(reinterpret_cast<void**>(&c->draft_counters), bytes);
    if (e == hipSuccess) e = hipMemset(c->draft_counters, 0, bytes);
    if (e != hipSuccess) st = hip_fail(e, "vc_create: draft counters");
  }
  if (st != VC_OK) {
    if (c->accept_counters) (void)hipFree(c->accept_counters);
    if (c->draft_counters) (void)hipFree(c->draft_counters);
    (void)hipStreamDestroy(c->copy_stream);
    free(c->events);
    free(c);
    return st;
  }
  c->issued = 0;
  *out = c;
  return VC_OK;
}

extern "C" vc_status vc_set_tunable(const char* name, int32_t value) {
  const int i = tunable_index(name);
  VC_REQUIRE(i >= 0, VC_ERR_INVALID_ARG, "vc_set_tunable: unknown tunable %s", name ? name : "(null)");
  tunables().value[i].store(value < 0 ? kUnset : value, std::memory_order_relaxed);
  return VC_OK;
}

extern "C" vc_status vc_get_tunable(const char* name, int32_t* value, int32_t* is_set) {
  const int i = tunable_index(name);
  VC_REQUIRE(i >= 0 && value && is_set, VC_ERR_INVALID_ARG, "vc_get_tunable: unknown tunable or NULL pointer");
  const int v = tunables().value[i].load(std::memory_order_relaxed);
  *is_set = v != kUnset;
  *value = v == kUnset ? 0 : v;
  return VC_OK;
}

extern "C" vc_status vc_stream_status(vc_ctx* c, void* stream) {
  VC_REQUIRE(c != nullptr, VC_ERR_INVALID_ARG, "vc_stream_status: ctx is NULL");
  const hipError_t e = hipStreamQuery(static_cast<hipStream_t>(stream));
  if (e == hipSuccess) return VC_OK;
  if (e == hipErrorNotReady) {
    (void)hipGetLastError();
    return fail(VC_ERR_NOT_READY, "vc_stream_status: work is still in flight");
  }
  return hip_fail(e, "hipStreamQuery");
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
  for (int i = 0; i < vc_ctx::kMarkRing; ++i)
    if (c->mark_events[i]) (void)hipEventDestroy(c->mark_events[i]);
  (void)hipStreamDestroy(c->copy_stream);
  if (c->accept_counters) (void)hipFree(c->accept_counters);
  if (c->draft_counters) (void)hipFree(c->draft_counters);
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

namespace vc {
// Rows named by index lists move between a pool (row (cu_ctx[b] + t, h)) and a packed buffer
// (row cu_idx[b]*Hkv + h*n_b + i, list after list); every 16 lanes move one 256-byte row of K and
// of V.  SCATTER: packed -> pool (reload of the dropped rows), else pool -> packed.
struct MoveRowsParams {
  uint16_t* pool_k;
  uint16_t* pool_v;
  uint16_t* packed_k;
  uint16_t* packed_v;
  const int* idx;
  const int* cu_idx;
  const int* cu_ctx;
  int n_kv_heads, seq0;
  long long packed_row0;   // packed row that sits at packed_k / packed_v (staging holds one sequence)
};

constexpr int kMoveRowsUnroll = 4;

template <bool SCATTER>
__global__ __launch_bounds__(256) void move_rows_kernel(MoveRowsParams p) {
  const int b = p.seq0 + blockIdx.z, h = blockIdx.y;
  const int n = p.cu_idx[b + 1] - p.cu_idx[b];
  const size_t list0 = static_cast<size_t>(p.cu_idx[b]) * p.n_kv_heads + static_cast<size_t>(h) * n;
  const int* list = p.idx + list0;
  const size_t row0 = static_cast<size_t>(p.cu_ctx[b]);
  const int sub = threadIdx.x & 15, grp = threadIdx.x >> 4;
  constexpr int kRowsPerPass = 16 * kMoveRowsUnroll;
  for (int i0 = blockIdx.x * kRowsPerPass; i0 < n; i0 += gridDim.x * kRowsPerPass) {
    size_t pool_off[kMoveRowsUnroll], pack_off[kMoveRowsUnroll];
    bool ok[kMoveRowsUnroll];
    uint4 kr[kMoveRowsUnroll], vr[kMoveRowsUnroll];
#pragma unroll
    for (int u = 0; u < kMoveRowsUnroll; ++u) {
      const int i = i0 + grp + 16 * u;
      ok[u] = i < n;
      const int t = ok[u] ? list[i] : 0;
      pool_off[u] = ((row0 + t) * p.n_kv_heads + h) * kHeadDim + 8 * sub;
      pack_off[u] = (list0 + (ok[u] ? i : 0) - static_cast<size_t>(p.packed_row0)) * kHeadDim + 8 * sub;
    }
#pragma unroll
    for (int u = 0; u < kMoveRowsUnroll; ++u) {
      if (ok[u]) {
        kr[u] = ld_stream(reinterpret_cast<const uint4*>((SCATTER ? p.packed_k + pack_off[u] : p.pool_k + pool_off[u])));
        vr[u] = ld_stream(reinterpret_cast<const uint4*>((SCATTER ? p.packed_v + pack_off[u] : p.pool_v + pool_off[u])));
      }
    }
#pragma unroll
    for (int u = 0; u < kMoveRowsUnroll; ++u) {
      if (ok[u]) {
        *reinterpret_cast<uint4*>((SCATTER ? p.pool_k + pool_off[u] : p.packed_k + pack_off[u])) = kr[u];
        *reinterpret_cast<uint4*>((SCATTER ? p.pool_v + pool_off[u] : p.packed_v + pack_off[u])) = vr[u];
      }
    }
  }
}
}  // namespace vc

static vc_status require_kind(const void* ptr, hipMemoryType kind, const char* who, const char* what) {
  hipPointerAttribute_t at;
  hipError_t e = hipPointerGetAttributes(&at, ptr);
  if (e != hipSuccess || at.type != kind) {
    (void)hipGetLastError();
    return fail(VC_ERR_INVALID_ARG, "%s: %s", who, what);
  }
  return VC_OK;
}

extern "C" vc_status vc_pack_rows(vc_ctx* c, const void* k, const void* v, const int32_t* idx, const int32_t* cu_idx,
                                  const int32_t* cu_ctx, int32_t n_seqs, int32_t n_kv_heads, int32_t max_idx,
                                  void* packed_k, void* packed_v, void* stream) {
  VC_REQUIRE(c != nullptr, VC_ERR_INVALID_ARG, "vc_pack_rows: ctx is NULL");
  VC_REQUIRE(n_seqs >= 0 && n_seqs <= 65535 && n_kv_heads > 0 && n_kv_heads <= 65535 && max_idx >= 0, VC_ERR_INVALID_ARG,
             "vc_pack_rows: n_seqs %d n_kv_heads %d max_idx %d", n_seqs, n_kv_heads, max_idx);
  if (n_seqs == 0 || max_idx == 0) return VC_OK;
  VC_REQUIRE(k && v && idx && cu_idx && cu_ctx && packed_k && packed_v, VC_ERR_INVALID_ARG, "vc_pack_rows: NULL pointer");
  VC_REQUIRE(aligned16(k) && aligned16(v) && aligned16(packed_k) && aligned16(packed_v), VC_ERR_INVALID_ARG,
             "vc_pack_rows: pools must be 16-byte aligned");
  vc::MoveRowsParams p{};
  p.pool_k = static_cast<uint16_t*>(const_cast<void*>(k));
  p.pool_v = static_cast<uint16_t*>(const_cast<void*>(v));
  p.packed_k = static_cast<uint16_t*>(packed_k);
  p.packed_v = static_cast<uint16_t*>(packed_v);
  p.idx = idx; p.cu_idx = cu_idx; p.cu_ctx = cu_ctx; p.n_kv_heads = n_kv_heads; p.seq0 = 0; p.packed_row0 = 0;
  const int per_list = ceil_div(max_idx, 16 * vc::kMoveRowsUnroll * 8);   // eight passes per workgroup
  hipLaunchKernelGGL(vc::move_rows_kernel<false>, dim3(per_list, n_kv_heads, n_seqs), dim3(256), 0,
                     static_cast<hipStream_t>(stream), p);
  VC_HIP(hipGetLastError());
  return VC_OK;
}

extern "C" vc_status vc_swap_in_rows(vc_ctx* c, const void* host_packed_k, const void* host_packed_v, void* stage_k,
                                     void* stage_v, int64_t stage_rows, void* dev_k, void* dev_v, const int32_t* dropped,
                                     const int32_t* cu_drop, const int32_t* cu_drop_host, const int32_t* cu_ctx,
                                     int32_t n_kv_heads, int32_t seq_begin, int32_t seq_end, int64_t* first_ticket) {
  const char* who = "vc_swap_in_rows";
  VC_REQUIRE(c && first_ticket, VC_ERR_INVALID_ARG, "%s: ctx or first_ticket is NULL", who);
  VC_REQUIRE(n_kv_heads > 0 && n_kv_heads <= 65535 && stage_rows >= 0, VC_ERR_INVALID_ARG, "%s: n_kv_heads %d stage_rows %lld",
             who, n_kv_heads, static_cast<long long>(stage_rows));
  VC_REQUIRE(seq_begin >= 0 && seq_end >= seq_begin, VC_ERR_INVALID_ARG, "%s: sequences [%d, %d)", who, seq_begin, seq_end);
  *first_ticket = c->issued;
  const int nseq = seq_end - seq_begin;
  if (nseq == 0) return VC_OK;
  VC_REQUIRE(host_packed_k && host_packed_v && stage_k && stage_v && dev_k && dev_v && dropped && cu_drop && cu_drop_host &&
                 cu_ctx, VC_ERR_INVALID_ARG, "%s: NULL pointer", who);
  VC_REQUIRE(aligned16(host_packed_k) && aligned16(host_packed_v) && aligned16(stage_k) && aligned16(stage_v) &&
                 aligned16(dev_k) && aligned16(dev_v), VC_ERR_INVALID_ARG, "%s: buffers must be 16-byte aligned", who);
  VC_REQUIRE(nseq <= vc_ctx::kRing, VC_ERR_INVALID_ARG, "%s: more than %d sequences per call", who, vc_ctx::kRing);
  vc_status st = require_kind(host_packed_k, hipMemoryTypeHost, who, "host_packed_k is not pinned host memory");
  if (st == VC_OK) st = require_kind(host_packed_v, hipMemoryTypeHost, who, "host_packed_v is not pinned host memory");
  if (st == VC_OK) st = require_kind(stage_k, hipMemoryTypeDevice, who, "stage_k is not device memory");
  if (st == VC_OK) st = require_kind(stage_v, hipMemoryTypeDevice, who, "stage_v is not device memory");
  if (st == VC_OK) st = require_kind(dev_k, hipMemoryTypeDevice, who, "dev_k is not device memory");
  if (st == VC_OK) st = require_kind(dev_v, hipMemoryTypeDevice, who, "dev_v is not device memory");
  if (st != VC_OK) return st;
  int max_nd = 0;
  for (int b = seq_begin; b < seq_end; ++b) {
    const int nd = cu_drop_host[b + 1] - cu_drop_host[b];
    VC_REQUIRE(nd >= 0, VC_ERR_INVALID_ARG, "%s: cu_drop_host is not ascending at %d", who, b);
    VC_REQUIRE(static_cast<int64_t>(nd) * n_kv_heads <= stage_rows, VC_ERR_INVALID_ARG,
               "%s: sequence %d needs %lld staging rows, stage_rows is %lld", who, b,
               static_cast<long long>(nd) * n_kv_heads, static_cast<long long>(stage_rows));
    max_nd = nd > max_nd ? nd : max_nd;
  }
  int64_t oldest_needed = c->issued + nseq - vc_ctx::kRing;
  if (oldest_needed > 0) {
    hipEvent_t ev = c->events[(oldest_needed - 1) % vc_ctx::kRing];
    if (ev && hipEventQuery(ev) != hipSuccess) {
      (void)hipGetLastError();
      return fail(VC_ERR_INVALID_ARG, "%s: more than %d tickets outstanding", who, vc_ctx::kRing);
    }
  }
  VC_HIP(hipSetDevice(c->device));
  vc::MoveRowsParams p{};
  p.pool_k = static_cast<uint16_t*>(dev_k);
  p.pool_v = static_cast<uint16_t*>(dev_v);
  p.packed_k = static_cast<uint16_t*>(stage_k);
  p.packed_v = static_cast<uint16_t*>(stage_v);
  p.idx = dropped; p.cu_idx = cu_drop; p.cu_ctx = cu_ctx; p.n_kv_heads = n_kv_heads;
  const size_t row_bytes = kHeadDim * 2;
  for (int b = seq_begin; b < seq_end; ++b) {
    int slot = static_cast<int>(c->issued % vc_ctx::kRing);
    if (!c->events[slot]) VC_HIP(hipEventCreateWithFlags(&c->events[slot], hipEventDisableTiming));
    const int nd = cu_drop_host[b + 1] - cu_drop_host[b];
    if (nd > 0) {
      // the copy stream is in order: the staging buffer is free again once the previous
      // sequence's placement kernel has run
      const size_t first_row = static_cast<size_t>(cu_drop_host[b]) * n_kv_heads;
      const size_t bytes = static_cast<size_t>(nd) * n_kv_heads * row_bytes;
      VC_HIP(hipMemcpyAsync(stage_k, static_cast<const char*>(host_packed_k) + first_row * row_bytes, bytes,
                            hipMemcpyHostToDevice, c->copy_stream));
      VC_HIP(hipMemcpyAsync(stage_v, static_cast<const char*>(host_packed_v) + first_row * row_bytes, bytes,
                            hipMemcpyHostToDevice, c->copy_stream));
      p.seq0 = b;
      p.packed_row0 = static_cast<long long>(first_row);
      const int per_list = ceil_div(nd, 16 * vc::kMoveRowsUnroll * 8);
      hipLaunchKernelGGL(vc::move_rows_kernel<true>, dim3(per_list, n_kv_heads, 1), dim3(256), 0, c->copy_stream, p);
      VC_HIP(hipGetLastError());
    }
    VC_HIP(hipEventRecord(c->events[slot], c->copy_stream));
    c->issued++;
  }
  (void)max_nd;
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

extern "C" vc_status vc_mark(vc_ctx* c, void* stream, int64_t* mark) {
  VC_REQUIRE(c != nullptr && mark != nullptr, VC_ERR_INVALID_ARG, "vc_mark: ctx or mark is NULL");
  VC_HIP(hipSetDevice(c->device));
  const int slot = static_cast<int>(c->marks_issued % vc_ctx::kMarkRing);
  if (!c->mark_events[slot]) {
    VC_HIP(hipEventCreateWithFlags(&c->mark_events[slot], hipEventDisableTiming));
  } else if (hipEventQuery(c->mark_events[slot]) != hipSuccess) {
    // the mark issued kMarkRing marks ago is still pending: its event cannot be re-recorded before it
    // has fired, or a wait for the old mark would be satisfied by the wrong work
    (void)hipGetLastError();
    VC_HIP(hipEventSynchronize(c->mark_events[slot]));
  }
  VC_HIP(hipEventRecord(c->mark_events[slot], static_cast<hipStream_t>(stream)));
  *mark = c->marks_issued++;
  return VC_OK;
}

extern "C" vc_status vc_swap_after(vc_ctx* c, int64_t mark) {
  VC_REQUIRE(c != nullptr, VC_ERR_INVALID_ARG, "vc_swap_after: ctx is NULL");
  VC_REQUIRE(mark >= 0 && mark < c->marks_issued, VC_ERR_INVALID_ARG, "vc_swap_after: mark %lld was never issued",
             static_cast<long long>(mark));
  if (c->marks_issued - mark > vc_ctx::kMarkRing) return VC_OK;   // fired before its slot was reused
  VC_HIP(hipStreamWaitEvent(c->copy_stream, c->mark_events[mark % vc_ctx::kMarkRing], 0));
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
