// Sampling-based acceptance: the rejection-sampling extension the paper's section 4.1 mentions in
// a footnote, read as textbook speculative sampling (the drafted token t_j, sampled from the draft
// distribution q_j, is kept with probability min(1, p_j(t_j) / q_j(t_j)); the first rejected
// position is re-drawn from the normalised positive part of p_j - q_j; if nothing is rejected the
// bonus token is drawn from p_w).  The random numbers are inputs.
//
// All probabilities are evaluated in double precision - p(v) = exp((x_v - M) / T) / S with M the
// row maximum and S the row's sum of exponentials - so that the integer results (accept length,
// drawn token) agree with a plain double-precision evaluation except when a draw falls within
// rounding distance (1e-12 relative) of a decision boundary.  The logits are streamed once for
// the row statistics (HBM bound); the few rows that are re-drawn are read twice more.
#include "common.h"

namespace vc {

constexpr int kSampleThreads = 256;
constexpr int kSamplePerThread = 32;
constexpr int kSampleSeg = kSampleThreads * kSamplePerThread;   // logits per workgroup

struct SampleParams {
  const float* target;
  const float* draft;
  const int* cu_rows;
  const int* cu_win;
  const int* draft_ids;
  const float* u_accept;
  const float* u_resample;
  int* accept_len;
  int* next_token;
  double* seg_stats;    // [rows_total][nseg][2]: segment maximum, segment sum of exp((x - max) / T)
  double* row_stats;    // [rows_total][2]: M, S
  double* res_sums;     // [n_seqs][nseg]: segment sums of the weights of the row that is re-drawn
  int* pick;            // [n_seqs][2]: target row and draft row of the re-draw (-1: none)
  int vocab, nseg, total_rows, total_win, n_seqs;
  double inv_t;
};

// deterministic workgroup sum of one double per thread (fixed tree), result in every thread
__device__ __forceinline__ double block_sum(double v, double* sh) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

__device__ __forceinline__ const float* row_ptr(const SampleParams& p, int r) {
  return r < p.total_rows ? p.target + static_cast<size_t>(r) * p.vocab
                          : p.draft + static_cast<size_t>(r - p.total_rows) * p.vocab;
}

// pass 1: per (row, segment) maximum and sum of exponentials (order inside a segment is free here,
// so the segment is read with coalesced 16-byte loads when the row is aligned for them)
__global__ __launch_bounds__(kSampleThreads) void sample_stats_kernel(SampleParams p) {
  __shared__ double sh[4];
  __shared__ float shm[4];
  const int r = blockIdx.y, seg = blockIdx.x;
  const float* row = row_ptr(p, r);
  const int seg0 = seg * kSampleSeg;
  float x[kSamplePerThread];
  const bool vec = (p.vocab & 3) == 0 && (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
  if (vec) {
#pragma unroll
    for (int i = 0; i < kSamplePerThread / 4; ++i) {
      const int e = seg0 + (i * kSampleThreads + threadIdx.x) * 4;
      float4 v = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      if (e < p.vocab) v = ld_stream(reinterpret_cast<const float4*>(row + e));
      x[4 * i] = v.x; x[4 * i + 1] = v.y; x[4 * i + 2] = v.z; x[4 * i + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kSamplePerThread; ++i) {
      const int e = seg0 + i * kSampleThreads + threadIdx.x;
      x[i] = e < p.vocab ? ld_stream(row + e) : -INFINITY;
    }
  }
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < kSamplePerThread; ++i) m = fmaxf(m, x[i]);
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  if ((threadIdx.x & 63) == 0) shm[threadIdx.x >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(shm[0], shm[1]), fmaxf(shm[2], shm[3]));
  double s = 0.0;
  if (m > -INFINITY) {
#pragma unroll
    for (int i = 0; i < kSamplePerThread; ++i)
      if (x[i] > -INFINITY) s += exp((static_cast<double>(x[i]) - static_cast<double>(m)) * p.inv_t);
  }
  s = block_sum(s, sh);
  if (threadIdx.x == 0) {
    double* dst = p.seg_stats + (static_cast<size_t>(r) * p.nseg + seg) * 2;
    dst[0] = m;
    dst[1] = s;
  }
}

// pass 2: row maximum and row sum from the segment statistics, in segment order
__global__ void sample_rows_kernel(SampleParams p) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= p.total_rows + p.total_win) return;
  const double* st = p.seg_stats + static_cast<size_t>(r) * p.nseg * 2;
  double M = -INFINITY;
  for (int s = 0; s < p.nseg; ++s) M = fmax(M, st[2 * s]);
  double S = 0.0;
  for (int s = 0; s < p.nseg; ++s)
    if (st[2 * s] > -INFINITY) S += st[2 * s + 1] * exp((st[2 * s] - M) * p.inv_t);
  p.row_stats[2 * r] = M;
  p.row_stats[2 * r + 1] = S;
}

__device__ __forceinline__ double prob_of(const SampleParams& p, int r, float x) {
  const double M = p.row_stats[2 * r], S = p.row_stats[2 * r + 1];
  return x > -INFINITY ? exp((static_cast<double>(x) - M) * p.inv_t) / S : 0.0;
}

// pass 3: the accept tests of one sequence, in order; picks the row to re-draw from
__global__ void sample_decide_kernel(SampleParams p) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= p.n_seqs) return;
  const int r0 = p.cu_rows[b], r1 = p.cu_rows[b + 1];
  const int w0 = p.cu_win[b], w = p.cu_win[b + 1] - w0;
  int a = w;
  for (int j = 0; j < w; ++j) {
    const int t = p.draft_ids[w0 + j];
    const double pt = prob_of(p, r0 + j, p.target[static_cast<size_t>(r0 + j) * p.vocab + t]);
    const double qt = prob_of(p, p.total_rows + w0 + j, p.draft[static_cast<size_t>(w0 + j) * p.vocab + t]);
    if (!(static_cast<double>(p.u_accept[w0 + j]) * qt < pt)) {
      a = j;
      break;
    }
  }
  p.accept_len[b] = a;
  int tr = -1, dr = -1;
  if (a < w) {
    tr = r0 + a;
    dr = p.total_rows + w0 + a;
  } else if (r0 + w < r1) {
    tr = r0 + w;      // bonus row: drawn from p alone
  }
  p.pick[2 * b] = tr;
  p.pick[2 * b + 1] = dr;
  if (tr < 0) p.next_token[b] = -1;
}

// weight of vocabulary entry v of the row that sequence b re-draws from
__device__ __forceinline__ double redraw_weight(const SampleParams& p, int tr, int dr, int v) {
  const double pv = prob_of(p, tr, p.target[static_cast<size_t>(tr) * p.vocab + v]);
  if (dr < 0) return pv;
  const double qv = prob_of(p, dr, p.draft[static_cast<size_t>(dr - p.total_rows) * p.vocab + v]);
  const double d = pv - qv;
  return d > 0.0 ? d : 0.0;
}

// pass 4: segment sums of the re-draw weights (each thread sums its 32 consecutive entries in order)
__global__ __launch_bounds__(kSampleThreads) void sample_weights_kernel(SampleParams p) {
  __shared__ double sh[4];
  const int b = blockIdx.y, seg = blockIdx.x;
  const int tr = p.pick[2 * b], dr = p.pick[2 * b + 1];
  if (tr < 0) return;
  const int e0 = seg * kSampleSeg + threadIdx.x * kSamplePerThread;
  double s = 0.0;
  for (int i = 0; i < kSamplePerThread; ++i)
    if (e0 + i < p.vocab) s += redraw_weight(p, tr, dr, e0 + i);
  s = block_sum(s, sh);
  if (threadIdx.x == 0) p.res_sums[static_cast<size_t>(b) * p.nseg + seg] = s;
}

// pass 5: inverse CDF - the smallest v whose running sum exceeds u * total
__global__ __launch_bounds__(kSampleThreads) void sample_pick_kernel(SampleParams p) {
  __shared__ double part[kSampleThreads];
  __shared__ double base_sh, thr_sh;
  __shared__ int seg_sh, thread_sh;
  const int b = blockIdx.x;
  const int tr = p.pick[2 * b], dr = p.pick[2 * b + 1];
  if (tr < 0) return;
  if (threadIdx.x == 0) {
    const double* ss = p.res_sums + static_cast<size_t>(b) * p.nseg;
    double total = 0.0;
    for (int s = 0; s < p.nseg; ++s) total += ss[s];
    const double thr = static_cast<double>(p.u_resample[b]) * total;
    double run = 0.0;
    int seg = p.nseg - 1;
    for (int s = 0; s < p.nseg; ++s) {
      if (run + ss[s] > thr) {
        seg = s;
        break;
      }
      run += ss[s];
    }
    if (seg == p.nseg - 1 && !(run + ss[seg] > thr)) {
      // rounding left the threshold above the last running sum: restart the last segment's search
      run = 0.0;
      for (int s = 0; s < seg; ++s) run += ss[s];
    }
    seg_sh = seg;
    base_sh = run;
    thr_sh = thr;
  }
  __syncthreads();
  const int seg = seg_sh;
  const int e0 = seg * kSampleSeg + threadIdx.x * kSamplePerThread;
  double w[kSamplePerThread];
  double s = 0.0;
  for (int i = 0; i < kSamplePerThread; ++i) {
    w[i] = e0 + i < p.vocab ? redraw_weight(p, tr, dr, e0 + i) : 0.0;
    s += w[i];
  }
  part[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    double run = base_sh;
    int th = -1;
    for (int t = 0; t < kSampleThreads; ++t) {
      const double before = run;
      run += part[t];
      part[t] = before;           // exclusive running sum in front of thread t
      if (th < 0 && run > thr_sh) th = t;
    }
    thread_sh = th;
  }
  __syncthreads();
  int th = thread_sh;
  if (th < 0) {
    // no running sum exceeds the threshold (rounding): take the last entry with a positive weight
    if (threadIdx.x == 0) {
      int last = min(p.vocab, (seg + 1) * kSampleSeg) - 1;
      while (last > 0 && !(redraw_weight(p, tr, dr, last) > 0.0)) --last;
      p.next_token[b] = last;
    }
    return;
  }
  if (threadIdx.x == th) {
    double run = part[th];
    int v = min(p.vocab, e0 + kSamplePerThread) - 1;
    for (int i = 0; i < kSamplePerThread; ++i) {
      run += w[i];
      if (run > thr_sh) {
        v = e0 + i;
        break;
      }
    }
    p.next_token[b] = v;
  }
}

static size_t align16(size_t n) { return (n + 15) & ~static_cast<size_t>(15); }

}  // namespace vc

using namespace vc;

extern "C" vc_status vc_accept_sample_workspace_bytes(int32_t total_rows, int32_t total_win, int32_t n_seqs,
                                                      int32_t vocab, size_t* bytes) {
  VC_REQUIRE(bytes != nullptr, VC_ERR_INVALID_ARG, "vc_accept_sample_workspace_bytes: bytes is NULL");
  VC_REQUIRE(total_rows >= 0 && total_win >= 0 && n_seqs >= 0 && vocab > 0, VC_ERR_INVALID_ARG,
             "vc_accept_sample_workspace_bytes: rows %d win %d seqs %d vocab %d", total_rows, total_win, n_seqs, vocab);
  const size_t nseg = static_cast<size_t>(ceil_div(vocab, kSampleSeg));
  const size_t rows = static_cast<size_t>(total_rows) + total_win;
  *bytes = align16(rows * nseg * 2 * sizeof(double)) + align16(rows * 2 * sizeof(double)) +
           align16(static_cast<size_t>(n_seqs) * nseg * sizeof(double)) + align16(static_cast<size_t>(n_seqs) * 2 * sizeof(int)) + 16;
  return VC_OK;
}

extern "C" vc_status vc_accept_sample(vc_ctx* ctx, const float* target_logits, const float* draft_logits, int32_t vocab,
                                      const int32_t* cu_rows, int32_t total_rows, const int32_t* draft_ids,
                                      const int32_t* cu_win, int32_t total_win, int32_t n_seqs, float temperature,
                                      const float* u_accept, const float* u_resample, int32_t* accept_len,
                                      int32_t* next_token, void* workspace, size_t workspace_bytes, void* stream) {
  VC_REQUIRE(ctx != nullptr, VC_ERR_INVALID_ARG, "vc_accept_sample: ctx is NULL");
  VC_REQUIRE(n_seqs >= 0 && total_rows >= 0 && total_win >= 0 && vocab > 0, VC_ERR_INVALID_ARG,
             "vc_accept_sample: n_seqs %d rows %d win %d vocab %d", n_seqs, total_rows, total_win, vocab);
  VC_REQUIRE(temperature > 0.f && temperature < INFINITY, VC_ERR_INVALID_ARG, "vc_accept_sample: temperature %g", temperature);
  VC_REQUIRE(total_rows >= total_win, VC_ERR_INVALID_ARG, "vc_accept_sample: fewer target rows (%d) than drafted positions (%d)",
             total_rows, total_win);
  if (n_seqs == 0) return VC_OK;
  VC_REQUIRE(cu_rows && cu_win && accept_len && next_token && u_resample, VC_ERR_INVALID_ARG, "vc_accept_sample: NULL pointer");
  VC_REQUIRE(total_rows == 0 || target_logits, VC_ERR_INVALID_ARG, "vc_accept_sample: target_logits is NULL");
  VC_REQUIRE(total_win == 0 || (draft_logits && draft_ids && u_accept), VC_ERR_INVALID_ARG,
             "vc_accept_sample: draft_logits / draft_ids / u_accept is NULL");
  VC_REQUIRE(total_rows + total_win <= 65535 && n_seqs <= 65535, VC_ERR_UNSUPPORTED, "vc_accept_sample: too many rows for one launch");
  size_t need = 0;
  vc_accept_sample_workspace_bytes(total_rows, total_win, n_seqs, vocab, &need);
  VC_REQUIRE(workspace != nullptr && workspace_bytes >= need, VC_ERR_WORKSPACE, "vc_accept_sample: workspace %zu bytes, need %zu",
             workspace_bytes, need);
  VC_REQUIRE(aligned16(workspace), VC_ERR_INVALID_ARG, "vc_accept_sample: workspace not 16-byte aligned");

  SampleParams p{};
  p.target = target_logits; p.draft = draft_logits;
  p.cu_rows = cu_rows; p.cu_win = cu_win; p.draft_ids = draft_ids;
  p.u_accept = u_accept; p.u_resample = u_resample;
  p.accept_len = accept_len; p.next_token = next_token;
  p.vocab = vocab; p.nseg = ceil_div(vocab, kSampleSeg);
  p.total_rows = total_rows; p.total_win = total_win; p.n_seqs = n_seqs;
  p.inv_t = 1.0 / static_cast<double>(temperature);
  const size_t rows = static_cast<size_t>(total_rows) + total_win;
  char* w = static_cast<char*>(workspace);
  p.seg_stats = reinterpret_cast<double*>(w); w += align16(rows * p.nseg * 2 * sizeof(double));
  p.row_stats = reinterpret_cast<double*>(w); w += align16(rows * 2 * sizeof(double));
  p.res_sums = reinterpret_cast<double*>(w); w += align16(static_cast<size_t>(n_seqs) * p.nseg * sizeof(double));
  p.pick = reinterpret_cast<int*>(w);

  hipStream_t st = static_cast<hipStream_t>(stream);
  if (rows > 0) {
    hipLaunchKernelGGL(sample_stats_kernel, dim3(p.nseg, static_cast<unsigned>(rows)), dim3(kSampleThreads), 0, st, p);
    hipLaunchKernelGGL(sample_rows_kernel, dim3(ceil_div(static_cast<int>(rows), 256)), dim3(256), 0, st, p);
  }
  hipLaunchKernelGGL(sample_decide_kernel, dim3(ceil_div(n_seqs, 64)), dim3(64), 0, st, p);
  hipLaunchKernelGGL(sample_weights_kernel, dim3(p.nseg, n_seqs), dim3(kSampleThreads), 0, st, p);
  hipLaunchKernelGGL(sample_pick_kernel, dim3(n_seqs), dim3(kSampleThreads), 0, st, p);
  VC_HIP(hipGetLastError());
  return VC_OK;
}
