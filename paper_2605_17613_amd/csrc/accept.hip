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

// keep = [0, len) minus dropped, streamed: no search, no LDS, no barrier.  The dropped list d[0..nd) is
// ascending, so the kept positions are the gaps between neighbouring entries: the positions strictly between
// d[i-1] and d[i] (with d[-1] = -1 and d[nd] = len) have exactly i entries below them, so position p there is
// kept entry number p - i.  Every lane reads one 16-byte chunk of the list (aligned in the `dropped` array as
// a whole, so a list's first and last chunk may hold a neighbour's entries, which are ignored), gets the entry
// below its chunk from the lane before it, and writes the kept positions between that entry and its last one -
// one run of the kept list, mostly empty at a 10 % budget; runs longer than a few positions (the forced first /
// last positions, lightly pruned lists) are written by the whole wave, 64 positions per store.  The list is
// read once with full-width loads.
// 128 lists of 65536 positions, 90 % dropped: 9.4 us.  Earlier forms: a workgroup per 4096 positions that found
// its entries by binary search and marked them in an LDS bitmap - 16 dependent trips to memory, 28 us; one
// 4-byte load and one bounded loop per gap - 18 us; 2 / 4 / 8 chunks per lane - 10.3 / 11.4 / 14.2 us (the
// chunks of a lane are worked off one after the other, each with its shuffle and its stores, so more, shorter
// waves hide that better).
constexpr int kKeepChunks = 1;    // 16-byte chunks per lane (see above)
constexpr int kKeepShort = 6;     // longer runs go to the wave

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
  const int nk = len - nd;
  if (nk <= 0) return;
  const long long total = static_cast<long long>(cu_drop[gridDim.z]) * n_kv_heads;     // ints in `dropped`
  const long long off = static_cast<long long>(cu_drop[b]) * n_kv_heads + static_cast<long long>(h) * nd;   // the list's first entry
  const long long a0 = off & ~3ll;                           // the aligned chunk that holds it
  const int shift = static_cast<int>(off - a0);              // entry i sits at int a0 + shift + i
  const int nchunk = (shift + nd) / 4 + 1;                   // ... so that the chunk holding index nd (the last gap) is covered
  const int c0 = blockIdx.x * (256 * kKeepChunks);
  if (c0 >= nchunk) return;
  int* out = keep_idx + (static_cast<size_t>(keep_base) * n_kv_heads + static_cast<size_t>(h) * nk);
  const int lane = threadIdx.x & 63;
  const int* chunks = dropped + a0;                          // 16-byte aligned; the list's entry i is chunks[shift + i]
  const long long left = total - a0;
  const int avail = left > 0x7fffffffll ? 0x7fffffff : static_cast<int>(left);   // ints of `dropped` from `chunks` on

  int e[kKeepChunks][4], prev[kKeepChunks];
#pragma unroll
  for (int c = 0; c < kKeepChunks; ++c) {
    const int j = c0 + 256 * c + threadIdx.x;                // this lane's chunk
    const int at = 4 * j;
    // the entry below the chunk's first one comes from the lane before; a wave's first lane reads it itself
    // (requested here with everything else, not when it is needed: that would be a trip to memory per chunk)
    const int ib = 4 * j - shift - 1;
    prev[c] = (lane == 0 && ib >= 0 && ib < nd) ? chunks[shift + ib] : 0;
    if (j < nchunk && at + 3 < avail) {
      const int4 v = *reinterpret_cast<const int4*>(chunks + at);
      e[c][0] = v.x; e[c][1] = v.y; e[c][2] = v.z; e[c][3] = v.w;
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) e[c][k] = (j < nchunk && at + k < avail) ? chunks[at + k] : 0;
    }
  }
  // Entry i of a well-formed list lies in [i, i + nk] (i entries below it, at most nk kept positions below
  // it); clamped into that range, ANY input gives stores that stay inside the list, so nothing below needs
  // bounds of its own.  Slots before the list count as entry i = i (nothing kept below them), slots from index
  // nd on as i + nk = len + (i - nd) (everything kept below them): the runs that end at them come out right or
  // empty.
  auto entry = [&](int v, int i) { return min(max(i < 0 ? i : i < nd ? v : i + nk, i), i + nk); };
#pragma unroll
  for (int c = 0; c < kKeepChunks; ++c) {
    const int j = c0 + 256 * c + threadIdx.x;
    const int i0 = 4 * j - shift;                            // index of this chunk's first entry (negative before the list)
#pragma unroll
    for (int k = 0; k < 4; ++k) e[c][k] = entry(e[c][k], i0 + k);
    int below = __shfl_up(e[c][3], 1, 64);                   // entry i0 - 1
    if (lane == 0) below = entry(prev[c], i0 - 1);
    // The kept positions between entry i0 - 1 and entry i0 + 3 are one run of the kept list: it starts at
    // kept entry number below + 1 - i0 and has t entries; its r-th entry is the r-th position above `below`
    // that is none of e0, e1, e2, and entry k has ck kept positions of the run below it.
    const int t = j < nchunk ? e[c][3] - below - 4 : 0;
    const int ck0 = e[c][0] - below - 1, ck1 = e[c][1] - below - 2, ck2 = e[c][2] - below - 3;
    int* run = out + (below + 1 - i0);
    const int first = below + 1;
    auto position = [&](int r, int f, int a0_, int a1_, int a2_) { return f + r + (r >= a0_) + (r >= a1_) + (r >= a2_); };
    if (t > 0 && t <= kKeepShort)
      for (int r = 0; r < t; ++r) run[r] = position(r, first, ck0, ck1, ck2);
    unsigned long long big = __ballot(t > kKeepShort);
    while (big) {                                            // a long run: the whole wave writes it
      const int src = __ffsll(big) - 1;
      big &= big - 1;
      const int tt = __shfl(t, src, 64), ff = __shfl(first, src, 64);
      const int b0 = __shfl(ck0, src, 64), b1 = __shfl(ck1, src, 64), b2 = __shfl(ck2, src, 64);
      int* rr = out + (ff - __shfl(i0, src, 64));
      for (int r = lane; r < tt; r += 64) rr[r] = position(r, ff, b0, b1, b2);
    }
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
  VC_REQUIRE((reinterpret_cast<uintptr_t>(dropped) & 15u) == 0, VC_ERR_INVALID_ARG, "vc_keep_from_dropped: dropped not 16-byte aligned");
  // a list of at most max_ctx entries spans at most max_ctx / 4 + 2 aligned chunks
  dim3 grid((max_ctx / 4 + 2) / (256 * kKeepChunks) + 1, n_kv_heads, n_seqs);
  hipLaunchKernelGGL(keep_from_dropped_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), dropped, cu_drop,
                     cu_ctx, n_kv_heads, keep_idx, cu_keep);
  VC_HIP(hipGetLastError());
  return VC_OK;
}
