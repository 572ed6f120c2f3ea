// Greedy acceptance (paper section 4.1 step 3) and kept-index lists from dropped-index lists
// (section 6, CompressedKV.dropped_indices).  Integer / compare work only: results are exact.
//
// Arg-max is a streaming scan of the fp32 logits (HBM bound).  A row is cut into segments so that
// few rows still fill the chip; every workgroup reduces its segment to one 64-bit key
//   key = (order-preserving image of the float) << 32 | ~index
// and stores it in the row's slot for that segment; the largest key of a row is the largest value
// and, among equal values, the lowest index.  The finishing kernel takes the maximum over a row's
// segments (a dozen keys) before it compares with the drafted ids.  In a short scan (up to
// kFusedMaxWgs workgroups) the finish runs inside the scan: every workgroup counts itself on a counter of its row (memory the
// context owns) after it has published its key; the one that completes a row takes the row's arg-max
// and counts the row; the one that completes the launch walks the drafted ids of every sequence.
// Counters go back to zero as they complete - one launch, no workspace that must be cleared.  Longer
// scans (and VC_ACCEPT_FUSED 0) take the finish as a second launch.
#include "common.h"

namespace vc {

constexpr int kAcceptThreads = 256;
constexpr int kSegElems = 8192;  // logits per workgroup

// -0 and +0 are equal logits (the lower index must win between them), so -0 is mapped to +0 first.
__device__ __forceinline__ uint32_t float_order(float f) {
  uint32_t u = __float_as_uint(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ unsigned long long make_key(float v, int idx) {
  return (static_cast<unsigned long long>(float_order(v)) << 32) | static_cast<uint32_t>(~static_cast<uint32_t>(idx));
}

constexpr int kFusedMaxRows = vc_ctx::kAcceptMaxRows;
constexpr int kFusedMaxWgs = 2048;
constexpr int kFusedMaxSeqs = 128;

__device__ __forceinline__ int key_index(unsigned long long key) { return static_cast<int>(~static_cast<uint32_t>(key)); }

struct FinishParams {
  unsigned int* counter;   // NULL: the finish is a launch of its own
  const int* cu_rows;
  const int* draft_ids;
  const int* cu_win;
  int* accept_len;
  int* next_token;
  int* argmax_ids;
  int n_seqs, total_rows;
};

// The compare of one sequence (section 4.1 step 3), by one wave: lane j holds drafted id j against
// the arg-max of row j, a ballot finds the first mismatch.  accept_len = drafted ids that equal the
// arg-max of their row, from the first row on; next_token = the arg-max of the first row that
// disagrees (or of the bonus row), -1 when the sequence has no such row.  id_at(r) = arg-max of row r.
template <typename IdAt>
__device__ __forceinline__ void accept_wave(int b, const int* cu_rows, const int* draft_ids, const int* cu_win, IdAt id_at,
                                            int* accept_len, int* next_token) {
  const int lane = threadIdx.x & 63;
  const int r0 = cu_rows[b], r1 = cu_rows[b + 1];
  const int w0 = cu_win[b], w = cu_win[b + 1] - w0;
  int a = w;
  for (int j0 = 0; j0 < w; j0 += 64) {
    const int j = j0 + lane;
    const bool miss = j < w && draft_ids[w0 + j] != id_at(r0 + j);
    const unsigned long long m = __ballot(miss);
    if (m != 0ull) {
      a = j0 + __ffsll(m) - 1;
      break;
    }
  }
  if (lane == 0) {
    accept_len[b] = a;
    next_token[b] = (r0 + a < r1) ? id_at(r0 + a) : -1;
  }
}

__global__ __launch_bounds__(kAcceptThreads) void argmax_segment_kernel(const float* __restrict__ logits, int vocab,
                                                                       unsigned long long* __restrict__ keys,
                                                                       FinishParams fp) {
  const int row = blockIdx.y;
  const int seg0 = blockIdx.x * kSegElems;
  const int seg1 = min(vocab, seg0 + kSegElems);
  const float* base = logits + static_cast<size_t>(row) * vocab;
  float best = -INFINITY;
  int bidx = 0x7fffffff;
  const bool vec_ok = ((reinterpret_cast<uintptr_t>(base + seg0) & 15u) == 0);
  if (vec_ok) {
    const int nvec = (seg1 - seg0) >> 2;
    const float4* b4 = reinterpret_cast<const float4*>(base + seg0);
    // a segment is at most kSegElems / 4 = 8 vectors per thread: all requested before the first compare
    constexpr int kVecPerThread = kSegElems / 4 / kAcceptThreads;
    float4 xs[kVecPerThread];
#pragma unroll
    for (int u = 0; u < kVecPerThread; ++u) {
      const int i = threadIdx.x + u * kAcceptThreads;
      xs[u] = i < nvec ? ld_stream(b4 + i) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    }
#pragma unroll
    for (int u = 0; u < kVecPerThread; ++u) {
      const int i = threadIdx.x + u * kAcceptThreads;
      if (i < nvec) {
        const float4 x = xs[u];
        const int e = seg0 + 4 * i;
        // ascending index order inside a thread, strict '>' keeps the first of equal values
        if (x.x > best || bidx == 0x7fffffff) { best = x.x; bidx = e; }
        if (x.y > best) { best = x.y; bidx = e + 1; }
        if (x.z > best) { best = x.z; bidx = e + 2; }
        if (x.w > best) { best = x.w; bidx = e + 3; }
      }
    }
    for (int e = seg0 + 4 * nvec + threadIdx.x; e < seg1; e += kAcceptThreads) {
      float x = ld_stream(base + e);
      if (x > best || bidx == 0x7fffffff) { best = x; bidx = e; }
    }
  } else {
    for (int e = seg0 + threadIdx.x; e < seg1; e += kAcceptThreads) {
      float x = ld_stream(base + e);
      if (x > best || bidx == 0x7fffffff) { best = x; bidx = e; }
    }
  }
  unsigned long long key = (bidx == 0x7fffffff) ? 0ull : make_key(best, bidx);
  for (int off = 32; off > 0; off >>= 1) {
    unsigned long long o = __shfl_xor(key, off, 64);
    key = o > key ? o : key;
  }
  __shared__ unsigned long long wk[kAcceptThreads / 64];
  __shared__ int last;
  if ((threadIdx.x & 63) == 0) wk[threadIdx.x >> 6] = key;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < kAcceptThreads / 64; ++w) key = wk[w] > key ? wk[w] : key;
    unsigned long long* slot = keys + static_cast<size_t>(row) * gridDim.x + blockIdx.x;
    if (fp.counter == nullptr) {
      *slot = key;   // 0 (below every real key) for an empty segment
    } else {
      // The key is written through to device-coherent memory (the workgroup that reads it may sit on
      // another XCD, behind another L2) and has arrived there before the count is taken.  A release
      // fence would do the same and also write this XCD's whole L2 back, once per workgroup (measured:
      // 368 against 49 us per call at 8448 workgroups); the key is the only store there is to order.
      // Counting is in two levels - the segments of a row on the row's counter, the rows on the
      // launch's - because thousands of atomics on one address serialise (124 us per call).
      __hip_atomic_store(slot, key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      const unsigned int nseg = gridDim.x;
      unsigned int* row_counter = fp.counter + (1 + row) * vc_ctx::kAcceptCounterStride;
      if (__hip_atomic_fetch_add(row_counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == nseg - 1u) {
        // last segment of its row: every key of the row has been published
        __hip_atomic_store(row_counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next call
        const unsigned long long* k = keys + static_cast<size_t>(row) * nseg;
        unsigned long long best = 0ull;
        for (unsigned int sgm = 0; sgm < nseg; ++sgm) {
          const unsigned long long o = __hip_atomic_load(k + sgm, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          best = o > best ? o : best;
        }
        __hip_atomic_store(fp.argmax_ids + row, key_index(best), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        last = __hip_atomic_fetch_add(fp.counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gridDim.y - 1u;
        if (last) __hip_atomic_store(fp.counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } else {
        last = 0;
      }
    }
  }
  if (fp.counter == nullptr) return;
  __syncthreads();
  if (!last) return;
  // ---- the workgroup that arrived last: the arg-max of every row has been published ----
  // all of them are fetched at once (each is a trip to device-coherent memory), then compared from LDS
  __shared__ int ids[kFusedMaxRows];
  for (int r = threadIdx.x; r < fp.total_rows; r += kAcceptThreads)
    ids[r] = __hip_atomic_load(fp.argmax_ids + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  for (int b = threadIdx.x >> 6; b < fp.n_seqs; b += kAcceptThreads / 64)
    accept_wave(b, fp.cu_rows, fp.draft_ids, fp.cu_win, [&](int r) { return ids[r]; }, fp.accept_len, fp.next_token);
}

__device__ __forceinline__ int row_argmax(const unsigned long long* __restrict__ keys, int nseg, int row) {
  const unsigned long long* k = keys + static_cast<size_t>(row) * nseg;
  unsigned long long best = k[0];
  for (int s = 1; s < nseg; ++s) best = k[s] > best ? k[s] : best;
  return key_index(best);
}

// One workgroup per sequence: its threads take the arg-max of the sequence's rows in parallel
// (written to argmax_ids), then one wave compares them with the drafted ids.
__global__ __launch_bounds__(128) void accept_finish_kernel(const unsigned long long* __restrict__ keys, int nseg,
                                                            const int* __restrict__ cu_rows,
                                                            const int* __restrict__ draft_ids,
                                                            const int* __restrict__ cu_win, int* __restrict__ accept_len,
                                                            int* __restrict__ next_token, int* __restrict__ argmax_ids) {
  const int b = blockIdx.x;
  const int r0 = cu_rows[b], r1 = cu_rows[b + 1];
  for (int r = r0 + threadIdx.x; r < r1; r += blockDim.x) argmax_ids[r] = row_argmax(keys, nseg, r);
  __syncthreads();                            // the ids written above are read below by wave 0
  if (threadIdx.x < 64)
    accept_wave(b, cu_rows, draft_ids, cu_win, [&](int r) { return argmax_ids[r]; }, accept_len, next_token);
}

// keep = [0, len) minus dropped.  A workgroup owns kKeepSpan consecutive positions [p0, p1) of one
// list: one binary search finds the first dropped entry >= p0 (every thread walks the same path, so
// the loads are broadcasts); the at most kKeepSpan entries that can fall below p1 are then read
// coalesced and set bits in an LDS bitmap; a position's rank among the kept ones is p0 minus the
// entries below p0, plus the kept positions before it in the span (workgroup prefix sum), so the
// dropped list is streamed once and the kept list is written in order.
constexpr int kKeepPerThread = 16;
constexpr int kKeepSpan = 256 * kKeepPerThread;

__global__ __launch_bounds__(256) void keep_from_dropped_kernel(const int* __restrict__ dropped,
                                                                const int* __restrict__ cu_drop,
                                                                const int* __restrict__ cu_ctx, int n_kv_heads,
                                                                int* __restrict__ keep_idx, int* __restrict__ cu_keep) {
  const int b = blockIdx.z, h = blockIdx.y;
  const int len = cu_ctx[b + 1] - cu_ctx[b];
  const int nd = cu_drop[b + 1] - cu_drop[b];
  const int keep_base = (cu_ctx[b] - cu_ctx[0]) - (cu_drop[b] - cu_drop[0]);  // = cu_keep[b]
  if (blockIdx.x == 0 && h == 0 && threadIdx.x == 0) {
    cu_keep[b] = keep_base;
    if (b == gridDim.z - 1) cu_keep[b + 1] = keep_base + len - nd;
  }
  const int p0 = blockIdx.x * kKeepSpan;
  if (p0 >= len) return;
  const int p1 = min(len, p0 + kKeepSpan);
  const int nk = len - nd;
  const int* dl = dropped + (static_cast<size_t>(cu_drop[b]) * n_kv_heads + static_cast<size_t>(h) * nd);
  int lo = 0, hi = nd;  // lower bound: first entry >= p0
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (dl[mid] < p0) lo = mid + 1; else hi = mid;
  }
  __shared__ uint32_t bits[kKeepSpan / 32];
  __shared__ int wave_total[4];
  if (threadIdx.x < kKeepSpan / 32) bits[threadIdx.x] = 0u;
  __syncthreads();
  for (int i = threadIdx.x; i < kKeepSpan && lo + i < nd; i += 256) {
    const int v = dl[lo + i];
    if (v < p1) atomicOr(&bits[(v - p0) >> 5], 1u << ((v - p0) & 31));
  }
  __syncthreads();
  // thread t owns positions p0 + 16t .. p0 + 16t + 15
  const int q0 = p0 + kKeepPerThread * threadIdx.x;
  uint32_t mask = (bits[threadIdx.x >> 1] >> (16 * (threadIdx.x & 1))) & 0xFFFFu;   // 1 = dropped
  const int valid = min(kKeepPerThread, max(0, p1 - q0));
  uint32_t kept = ~mask & ((1u << valid) - 1u);
  const int cnt = __popc(kept);
  // exclusive prefix sum of cnt over the workgroup
  int incl = cnt;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(incl, off, 64);
    if (lane >= off) incl += o;
  }
  if (lane == 63) wave_total[wave] = incl;
  __syncthreads();
  int before = incl - cnt;
  for (int w = 0; w < wave; ++w) before += wave_total[w];
  int* out = keep_idx + (static_cast<size_t>(keep_base) * n_kv_heads + static_cast<size_t>(h) * nk) + (p0 - lo) + before;
  while (kept) {
    const int e = __ffs(kept) - 1;
    kept &= kept - 1;
    *out++ = q0 + e;
  }
}

}  // namespace vc

using namespace vc;

extern "C" vc_status vc_accept_workspace_bytes(int32_t total_rows, int32_t vocab, size_t* bytes) {
  VC_REQUIRE(bytes != nullptr, VC_ERR_INVALID_ARG, "vc_accept_workspace_bytes: bytes is NULL");
  VC_REQUIRE(total_rows >= 0 && vocab > 0, VC_ERR_INVALID_ARG, "vc_accept_workspace_bytes: rows %d vocab %d",
             total_rows, vocab);
  *bytes = static_cast<size_t>(total_rows > 0 ? total_rows : 1) * ceil_div(vocab, kSegElems) * sizeof(unsigned long long);
  return VC_OK;
}

extern "C" vc_status vc_accept_len(vc_ctx* ctx, const float* logits, int32_t vocab, const int32_t* cu_rows,
                                   int32_t total_rows, const int32_t* draft_ids, const int32_t* cu_win, int32_t n_seqs,
                                   int32_t* accept_len, int32_t* next_token, int32_t* argmax_ids, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  VC_REQUIRE(ctx != nullptr, VC_ERR_INVALID_ARG, "vc_accept_len: ctx is NULL");
  VC_REQUIRE(n_seqs >= 0 && total_rows >= 0 && vocab > 0, VC_ERR_INVALID_ARG, "vc_accept_len: n_seqs %d rows %d vocab %d",
             n_seqs, total_rows, vocab);
  if (n_seqs == 0) return VC_OK;
  VC_REQUIRE(cu_rows && cu_win && accept_len && next_token, VC_ERR_INVALID_ARG, "vc_accept_len: NULL pointer");
  VC_REQUIRE(total_rows == 0 || (logits && argmax_ids), VC_ERR_INVALID_ARG, "vc_accept_len: logits/argmax_ids NULL");
  VC_REQUIRE((reinterpret_cast<uintptr_t>(logits) & 3u) == 0, VC_ERR_INVALID_ARG, "vc_accept_len: logits misaligned");
  size_t need = 0;
  vc_accept_workspace_bytes(total_rows, vocab, &need);
  VC_REQUIRE(workspace != nullptr && workspace_bytes >= need, VC_ERR_WORKSPACE,
             "vc_accept_len: workspace %zu bytes, need %zu", workspace_bytes, need);
  VC_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 7u) == 0, VC_ERR_INVALID_ARG, "vc_accept_len: workspace misaligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned long long* keys = static_cast<unsigned long long*>(workspace);
  const int nseg = ceil_div(vocab, kSegElems);
  FinishParams fp{};
  // One launch while the scan is short (the second launch is then a fifth of the call: 14.8 -> 11.5 us
  // at 36 rows of 128256 logits).  A workgroup of a fused launch ends with two trips to device-coherent
  // memory; with dozens of workgroups per compute unit those add up to more than the launch they save
  // (8448 workgroups: 57.6 against 47.3 us), so larger scans keep the finish as a launch of its own.
  // (the workgroup that finishes compares the sequences four at a time: not for batches of hundreds)
  const bool fused = total_rows > 0 && total_rows <= kFusedMaxRows && n_seqs <= kFusedMaxSeqs &&
                     static_cast<int64_t>(total_rows) * nseg <= kFusedMaxWgs && ctx->accept_counters != nullptr &&
                     tunable(kTunAcceptFused, 1, 0, 1) != 0;
  if (fused) {
    // calls in flight at the same time (other streams, captured graphs) each count on a counter of their own
    fp.counter = ctx->accept_counters + (ctx->accept_calls++ % vc_ctx::kAcceptCounters) * vc_ctx::kAcceptSlotWords;
    fp.cu_rows = cu_rows; fp.draft_ids = draft_ids; fp.cu_win = cu_win;
    fp.accept_len = accept_len; fp.next_token = next_token; fp.argmax_ids = argmax_ids;
    fp.n_seqs = n_seqs; fp.total_rows = total_rows;
  }
  if (total_rows > 0) {
    dim3 grid(nseg, total_rows);
    hipLaunchKernelGGL(argmax_segment_kernel, grid, dim3(kAcceptThreads), 0, st, logits, vocab, keys, fp);
  }
  if (!fused)
    hipLaunchKernelGGL(accept_finish_kernel, dim3(n_seqs), dim3(128), 0, st, keys, nseg, cu_rows, draft_ids, cu_win,
                       accept_len, next_token, argmax_ids);
  VC_HIP(hipGetLastError());
  return VC_OK;
}

extern "C" vc_status vc_keep_from_dropped(vc_ctx* ctx, const int32_t* dropped, const int32_t* cu_drop,
                                          const int32_t* cu_ctx, int32_t n_seqs, int32_t n_kv_heads, int32_t max_ctx,
                                          int32_t* keep_idx, int32_t* cu_keep, void* stream) {
  VC_REQUIRE(ctx != nullptr, VC_ERR_INVALID_ARG, "vc_keep_from_dropped: ctx is NULL");
  VC_REQUIRE(n_seqs >= 0 && n_kv_heads > 0 && max_ctx >= 0, VC_ERR_INVALID_ARG,
             "vc_keep_from_dropped: n_seqs %d n_kv_heads %d max_ctx %d", n_seqs, n_kv_heads, max_ctx);
  if (n_seqs == 0) return VC_OK;
  VC_REQUIRE(cu_drop && cu_ctx && cu_keep, VC_ERR_INVALID_ARG, "vc_keep_from_dropped: NULL cu array");
  VC_REQUIRE(max_ctx == 0 || keep_idx, VC_ERR_INVALID_ARG, "vc_keep_from_dropped: keep_idx is NULL");
  VC_REQUIRE(n_seqs <= 65535 && n_kv_heads <= 65535, VC_ERR_UNSUPPORTED, "vc_keep_from_dropped: grid too large");
  dim3 grid(max_ctx > 0 ? ceil_div(max_ctx, kKeepSpan) : 1, n_kv_heads, n_seqs);
  hipLaunchKernelGGL(keep_from_dropped_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), dropped, cu_drop,
                     cu_ctx, n_kv_heads, keep_idx, cu_keep);
  VC_HIP(hipGetLastError());
  return VC_OK;
}
