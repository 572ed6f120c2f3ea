// Optional data-dependent validation of the descriptors' device arrays (the attention calls
// themselves only validate what the host can see in O(1): the paper's interface hands the runtime
// per-request offsets and dropped / kept position lists, section 6, and a wrong list would make a
// kernel read outside its pools).  Asynchronous like every other call: the verdict is written to a
// device report that the caller reads after the stream has reached it.
#include "common.h"

namespace vc {

// report[0] = number of violations, report[1] = smallest violation key, or -1 when there is none
// key = kind << 56 | sequence << 32 | index
__device__ __forceinline__ void violation(unsigned long long* report, int kind, int seq, unsigned index) {
  atomicAdd(report, 1ull);
  atomicMin(report + 1, (static_cast<unsigned long long>(kind) << 56) | (static_cast<unsigned long long>(static_cast<unsigned>(seq)) << 32) | index);
}

__global__ void validate_init_kernel(unsigned long long* report) {
  report[0] = 0ull;
  report[1] = ~0ull;
}

struct ValidateCompParams {
  const int* cu_ctx;
  const int* keep_idx;
  const int* cu_keep;
  const int* cu_blk;
  const int* cu_tail;
  unsigned long long* report;
  int n_kv_heads, max_keep, max_blk, max_tail;
  bool keep_all;   // pool without keep_idx: max_keep bounds the sequence length
};

// Grid (x, KV head, sequence).  Workgroup (0, 0, b) checks the prefix arrays of sequence b; all
// workgroups of (h, b) walk kept-index list (b, h) with a grid-stride loop over its device-side
// length, so a host-side maximum that under-estimates is itself found rather than trusted.
__global__ __launch_bounds__(256) void validate_comp_kernel(ValidateCompParams p) {
  const int b = blockIdx.z, h = blockIdx.y;
  int len = -1;
  if (p.cu_ctx) len = p.cu_ctx[b + 1] - p.cu_ctx[b];
  if (blockIdx.x == 0 && h == 0 && threadIdx.x == 0) {
    if (p.cu_ctx) {
      if (len < 0) violation(p.report, VC_BAD_PREFIX_ORDER, b, 0);
      if (p.keep_all && len > p.max_keep) violation(p.report, VC_BAD_HOST_MAX, b, 0);
    }
    if (p.cu_keep) {
      const int nk = p.cu_keep[b + 1] - p.cu_keep[b];
      if (nk < 0) violation(p.report, VC_BAD_PREFIX_ORDER, b, 1);
      if (nk > p.max_keep) violation(p.report, VC_BAD_HOST_MAX, b, 1);
      if (len >= 0 && nk > len) violation(p.report, VC_BAD_KEEP_COUNT, b, static_cast<unsigned>(nk));
    }
    if (p.cu_blk) {
      const int nb = p.cu_blk[b + 1] - p.cu_blk[b];
      if (nb < 0) violation(p.report, VC_BAD_PREFIX_ORDER, b, 2);
      if (nb > p.max_blk) violation(p.report, VC_BAD_HOST_MAX, b, 2);
    }
    if (p.cu_tail) {
      const int nt = p.cu_tail[b + 1] - p.cu_tail[b];
      if (nt < 0) violation(p.report, VC_BAD_PREFIX_ORDER, b, 3);
      if (nt > p.max_tail) violation(p.report, VC_BAD_HOST_MAX, b, 3);
    }
  }
  if (!p.keep_idx || !p.cu_keep || len < 0) return;
  const int nk = p.cu_keep[b + 1] - p.cu_keep[b];
  if (nk <= 0) return;
  const int* list = p.keep_idx + static_cast<size_t>(p.cu_keep[b]) * p.n_kv_heads + static_cast<size_t>(h) * nk;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < nk; i += gridDim.x * blockDim.x) {
    const int t = list[i];
    if (t < 0 || t >= len) violation(p.report, VC_BAD_KEEP_RANGE, b, static_cast<unsigned>(i));
    if (i > 0 && list[i - 1] >= t) violation(p.report, VC_BAD_KEEP_ORDER, b, static_cast<unsigned>(i));
  }
}

__global__ __launch_bounds__(256) void validate_full_kernel(const int* cu_ctx, const int* cu_win, int n_seqs, int max_ctx, int max_win,
                                                            int total_win, unsigned long long* report) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= n_seqs) return;
  const int len = cu_ctx[b + 1] - cu_ctx[b];
  if (len < 0) violation(report, VC_BAD_PREFIX_ORDER, b, 0);
  if (len > max_ctx) violation(report, VC_BAD_HOST_MAX, b, 0);
  if (cu_win) {
    const int w = cu_win[b + 1] - cu_win[b];
    if (w < 0) violation(report, VC_BAD_PREFIX_ORDER, b, 4);
    if (w > max_win) violation(report, VC_BAD_HOST_MAX, b, 4);
    if (b == n_seqs - 1 && (cu_win[n_seqs] - cu_win[0]) != total_win) violation(report, VC_BAD_HOST_MAX, b, 5);
  }
}

}  // namespace vc

using namespace vc;

extern "C" vc_status vc_validate_comp_kv(vc_ctx* ctx, const vc_comp_kv* kv, int64_t* report, void* stream) {
  VC_REQUIRE(ctx && kv && report, VC_ERR_INVALID_ARG, "vc_validate_comp_kv: NULL pointer");
  VC_REQUIRE((reinterpret_cast<uintptr_t>(report) & 7u) == 0, VC_ERR_INVALID_ARG, "vc_validate_comp_kv: report not 8-byte aligned");
  VC_REQUIRE(kv->n_seqs >= 0 && kv->n_seqs <= 65535 && kv->n_kv_heads > 0 && kv->n_kv_heads <= 65535, VC_ERR_INVALID_ARG,
             "vc_validate_comp_kv: n_seqs %d n_kv_heads %d", kv->n_seqs, kv->n_kv_heads);
  VC_REQUIRE(!kv->keep_idx || (kv->cu_keep && kv->cu_ctx), VC_ERR_INVALID_ARG, "vc_validate_comp_kv: keep_idx needs cu_keep and cu_ctx");
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned long long* rep = reinterpret_cast<unsigned long long*>(report);
  hipLaunchKernelGGL(validate_init_kernel, dim3(1), dim3(1), 0, st, rep);
  if (kv->n_seqs > 0) {
    ValidateCompParams p{};
    p.cu_ctx = kv->pool_k ? kv->cu_ctx : nullptr;
    p.keep_idx = kv->pool_k ? kv->keep_idx : nullptr;
    p.cu_keep = kv->pool_k && kv->keep_idx ? kv->cu_keep : nullptr;
    p.cu_blk = kv->blocks ? kv->cu_blk : nullptr;
    p.cu_tail = kv->tail_k ? kv->cu_tail : nullptr;
    p.report = rep;
    p.n_kv_heads = kv->n_kv_heads;
    p.max_keep = kv->max_keep; p.max_blk = kv->max_blk; p.max_tail = kv->max_tail;
    p.keep_all = kv->pool_k != nullptr && kv->keep_idx == nullptr;
    const int per_list = p.keep_idx ? ceil_div(kv->max_keep > 0 ? kv->max_keep : 1, 256 * 8) : 1;
    hipLaunchKernelGGL(validate_comp_kernel, dim3(per_list, p.keep_idx ? kv->n_kv_heads : 1, kv->n_seqs), dim3(256), 0, st, p);
  }
  VC_HIP(hipGetLastError());
  return VC_OK;
}

extern "C" vc_status vc_validate_full_kv(vc_ctx* ctx, const vc_full_kv* kv, const int32_t* cu_win, int32_t total_win,
                                         int64_t* report, void* stream) {
  VC_REQUIRE(ctx && kv && report, VC_ERR_INVALID_ARG, "vc_validate_full_kv: NULL pointer");
  VC_REQUIRE((reinterpret_cast<uintptr_t>(report) & 7u) == 0, VC_ERR_INVALID_ARG, "vc_validate_full_kv: report not 8-byte aligned");
  VC_REQUIRE(kv->n_seqs >= 0 && kv->cu_ctx != nullptr, VC_ERR_INVALID_ARG, "vc_validate_full_kv: n_seqs %d or cu_ctx NULL", kv->n_seqs);
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned long long* rep = reinterpret_cast<unsigned long long*>(report);
  hipLaunchKernelGGL(validate_init_kernel, dim3(1), dim3(1), 0, st, rep);
  if (kv->n_seqs > 0)
    hipLaunchKernelGGL(validate_full_kernel, dim3(ceil_div(kv->n_seqs, 256)), dim3(256), 0, st, kv->cu_ctx, cu_win, kv->n_seqs,
                       kv->max_ctx, kv->max_win, total_win, rep);
  VC_HIP(hipGetLastError());
  return VC_OK;
}
