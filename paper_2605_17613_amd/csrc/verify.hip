// Verify attention: a window of drafted tokens attends causally to the full bf16 KV plus the
// window itself (paper section 4.1 step 2).  The g query heads of a KV head times the w window
// positions form w*g rows that share every K/V row, so the row dimension is a real MFMA tile and
// every K/V byte is read from HBM exactly once per (sequence, KV head).
//
// Formulation (bf16 MFMA 32x32x16, fp32 accumulation), per 32-token sub-tile of a wave:
//   S^T[token][row]  = K[token][:] . Q[row][:]      A = K from LDS, B = Q^T (registers, loaded once)
//   O^T[d][row]     += V^T[d][token] * P^T[token][row]
// With rows on the lanes, a lane owns the softmax state of one row and the probabilities leave the
// first product in the register layout the second one wants; V^T comes out of LDS through the
// transposing 64-bit LDS read, so V stays token-major in memory.
//
// A workgroup (8 waves, two per SIMD so one wave's softmax overlaps the other's MFMAs) owns one
// chunk of tokens of one (sequence, KV head).  Rows are cut into groups of 32 (one per wave); with
// R <= 64 rows the waves split each 128-token tile four ways, with R <= 128 two ways, above that
// every wave takes its own 32 rows of a 32-token tile.  Tiles are double buffered in LDS: the next
// tile is fetched into registers while the current one is used.
#include <type_traits>

#include "attn_common.h"
#include "common.h"

namespace vc {

struct VerifyParams {
  const uint16_t* qw;
  const uint16_t* kf;
  const uint16_t* vf;
  const uint16_t* kw;
  const uint16_t* vw;
  const int* cu_ctx;
  const int* cu_win;
  float* ws;
  int n_q_heads, n_kv_heads, g;
  int chunk_tok, ns;   // ns = 4 * chunks of the longest sequence
  float scale_log2e;
};

constexpr int kLdsStride = 136;                 // bf16 per LDS row: 128 + 8 pad (272 bytes)
constexpr int kTileBytes = 128 * kLdsStride * 2;  // one 128-token K or V tile
constexpr int kVerifyLds = 4 * kTileBytes;      // K and V, double buffered
constexpr float kVerifyMargin = 4.f;
constexpr float kMinusBig = -1.0e30f;    // "no key seen yet": finite, so 2^(s - m) needs no special cases

typedef short short4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float16v mfma32(bf16x8v a, bf16x8v b, float16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8v load_bf16x8(const uint16_t* p) {
  bf16x8v r;
  const uint4 raw = *reinterpret_cast<const uint4*>(p);
  __builtin_memcpy(&r, &raw, 16);
  return r;
}

// 16-byte LDS accesses through explicit LDS pointers (ds_read_b128 / ds_write_b128)
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x4v lds_u32x4v;
__device__ __forceinline__ bf16x8v lds_load_bf16x8(const uint16_t* p) {
  const u32x4v raw = *(const lds_u32x4v*)(p);
  return __builtin_bit_cast(bf16x8v, raw);
}
__device__ __forceinline__ void lds_store16(uint16_t* p, const uint4& v) {
  const u32x4v raw = {v.x, v.y, v.z, v.w};
  *(lds_u32x4v*)(p) = raw;
}

// Transposing LDS read: the 16 lanes of a block fetch a 4 x 16 patch (lane 4k+c: row k, columns
// 4c..4c+3) and lane i of the block receives column i of the patch (4 rows).
__device__ __forceinline__ short4v lds_read_tr(const uint16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(p));
}

// One wave owns 32 rows (one MFMA row tile) and, of every LDS tile, one 32-token slice.
// NTG = token slices per tile; the 8 waves of a workgroup form NRG = 8/NTG row groups.
template <int NTG>
__device__ __forceinline__ void verify_body(const VerifyParams& p, uint16_t* smem, int kvh, int chunk, int w0, int w,
                                            int c0, int N) {
  constexpr int NRG = 8 / NTG;
  constexpr int TT = 32 * NTG;          // tokens per LDS tile
  constexpr int NLD = NTG;              // 16-byte loads per thread per matrix per tile (512 threads)
  const int R = w * p.g;
  const int total = N + w;
  const int t_begin = chunk * p.chunk_tok;
  const int t_end = min(total, t_begin + p.chunk_tok);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rg = wave % NRG, tg = wave / NRG;
  const int n = lane & 31, hh = lane >> 5;
  const bool wave_rows = rg * 32 < R;

  // smem in 2-byte elements: buffer 0 = [K tile | V tile], buffer 1 = [K tile | V tile]
  uint16_t* Ks[2] = {smem, smem + kTileBytes};
  uint16_t* Vs[2] = {smem + kTileBytes / 2, smem + kTileBytes + kTileBytes / 2};

  const int r = rg * 32 + n;
  const bool row_ok = r < R;
  const int rc = row_ok ? r : R - 1;
  const int iw = rc / p.g, hq = rc % p.g;
  bf16x8v qb[8];
  {
    const uint16_t* qp = p.qw + (static_cast<size_t>(w0 + iw) * p.n_q_heads + kvh * p.g + hq) * kHeadDim + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qb[ks] = load_bf16x8(qp + 16 * ks);
  }

  float m = kMinusBig, l = 0.f;
  float16v oacc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.f;

  const size_t row_stride = static_cast<size_t>(p.n_kv_heads) * kHeadDim;
  const size_t head_off = static_cast<size_t>(kvh) * kHeadDim;

  // Two register sets of in-flight tiles: a tile is requested two iterations before it is used,
  // so two compute phases (not one) cover the HBM latency.
  uint4 kx[2][NLD], vx[2][NLD];
  const size_t thr_off = static_cast<size_t>(tid >> 4) * row_stride + head_off + 8 * (tid & 15);
  const uint16_t* kfast = p.kf + static_cast<size_t>(c0) * row_stride + thr_off;
  const uint16_t* vfast = p.vf + static_cast<size_t>(c0) * row_stride + thr_off;
  auto fetch = [&](auto SET, int t) {
    constexpr int S = decltype(SET)::value;
    if (t + TT <= N) {                      // whole tile inside the full KV: plain strided loads
      const size_t toff = static_cast<size_t>(t) * row_stride;
#pragma unroll
      for (int c = 0; c < NLD; ++c) {
        kx[S][c] = *reinterpret_cast<const uint4*>(kfast + toff + static_cast<size_t>(32 * c) * row_stride);
        vx[S][c] = *reinterpret_cast<const uint4*>(vfast + toff + static_cast<size_t>(32 * c) * row_stride);
      }
    } else {
#pragma unroll
      for (int c = 0; c < NLD; ++c) {
        const int tok = t + 32 * c + (tid >> 4), part = tid & 15;
        kx[S][c] = uint4{0u, 0u, 0u, 0u};
        vx[S][c] = uint4{0u, 0u, 0u, 0u};
        if (tok < N) {
          const size_t off = static_cast<size_t>(c0 + tok) * row_stride + head_off + 8 * part;
          kx[S][c] = *reinterpret_cast<const uint4*>(p.kf + off);
          vx[S][c] = *reinterpret_cast<const uint4*>(p.vf + off);
        } else if (tok < total) {
          const size_t off = static_cast<size_t>(w0 + tok - N) * row_stride + head_off + 8 * part;
          kx[S][c] = *reinterpret_cast<const uint4*>(p.kw + off);
          vx[S][c] = *reinterpret_cast<const uint4*>(p.vw + off);
        }
      }
    }
  };
  auto stash = [&](auto SET, int buf) {
    constexpr int S = decltype(SET)::value;
#pragma unroll
    for (int c = 0; c < NLD; ++c) {
      const int tt = 32 * c + (tid >> 4), part = tid & 15;
      lds_store16(&Ks[buf][tt * kLdsStride + 8 * part], kx[S][c]);
      lds_store16(&Vs[buf][tt * kLdsStride + 8 * part], vx[S][c]);
    }
  };
  using Set0 = std::integral_constant<int, 0>;
  using Set1 = std::integral_constant<int, 1>;

  // transposing-read coordinates of this lane inside a (token, channel) patch
  const int blk16 = lane >> 4;
  const int tr_row = 4 * (blk16 >> 1) + ((lane & 15) >> 2);
  const int tr_col = 16 * (blk16 & 1) + 4 * (lane & 3);

  auto compute = [&](int buf, int t) {
    const int ts = t + 32 * tg;             // first token of this wave's slice
    if (wave_rows && ts < t_end) {
      const uint16_t* Kt = Ks[buf] + (32 * tg) * kLdsStride;
      const uint16_t* Vt = Vs[buf] + (32 * tg) * kLdsStride;
      // ---- S^T = K Q^T ----
      float16v sacc;
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8v a = lds_load_bf16x8(&Kt[n * kLdsStride + 16 * ks + 8 * hh]);
        sacc = mfma32(a, qb[ks], sacc);
      }
      // register i of this lane is token row 8*(i/4) + 4*hh + i%4 of the slice, for row n
      float s[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = sacc[i] * p.scale_log2e;
      if (ts + 32 > min(N, t_end)) {        // slice touches the window or the end of the chunk
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int tok = ts + 8 * (i >> 2) + 4 * hh + (i & 3);
          const bool ok = tok < t_end && (tok < N || tok - N <= iw);
          s[i] = ok ? s[i] : -INFINITY;
        }
      }
      float mt = s[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mt = fmaxf(mt, s[i]);
      if (__any(mt > m + kVerifyMargin)) {
        const float mx = fmaxf(mt, __shfl_xor(mt, 32, 64));
        const float mn = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f(m - mn);
        l *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;
        m = mn;
      }
      bf16x8v pb[2];
      float ps = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pr = __builtin_amdgcn_exp2f(s[i] - m);
        ps += pr;
        pb[i >> 3][i & 7] = (__bf16)pr;
      }
      l += ps;
      // ---- O^T += V^T P^T ; A element e of k-step kk is token row 16kk + 8(e/4) + 4hh + e%4 ----
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const uint16_t* base = Vt + (16 * kk + tr_row) * kLdsStride + 32 * dt + tr_col;
          const short4v lo = lds_read_tr(base);
          const short4v hi = lds_read_tr(base + 8 * kLdsStride);
          bf16x8v av;
          const short sv8[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          __builtin_memcpy(&av, sv8, 16);
          oacc[dt] = mfma32(av, pb[kk], oacc[dt]);
        }
      }
    }
  };

  // tile j lives in register set j%2 and LDS buffer j%2
  fetch(Set0{}, t_begin);
  stash(Set0{}, 0);
  if (t_begin + TT < t_end) fetch(Set1{}, t_begin + TT);
  if (t_begin + 2 * TT < t_end) fetch(Set0{}, t_begin + 2 * TT);
  __syncthreads();
  for (int t = t_begin; t < t_end; t += 2 * TT) {
    compute(0, t);
    if (t + TT < t_end) stash(Set1{}, 1);
    if (t + 3 * TT < t_end) fetch(Set1{}, t + 3 * TT);
    __syncthreads();
    if (t + TT >= t_end) break;
    compute(1, t + TT);
    if (t + 2 * TT < t_end) stash(Set0{}, 0);
    if (t + 4 * TT < t_end) fetch(Set0{}, t + 4 * TT);
    __syncthreads();
  }

  if (!wave_rows) return;
  const float lt = l + __shfl_xor(l, 32, 64);
  if (!row_ok) return;
  const size_t grow = static_cast<size_t>(w0 + iw) * p.n_q_heads + kvh * p.g + hq;
  float* dst = p.ws + (grow * p.ns + chunk * 4 + tg) * kPartialFloats;
  if (hh == 0) {
    dst[0] = m;
    dst[1] = lt;
  }
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) dst[2 + 32 * dt + 8 * (i >> 2) + 4 * hh + (i & 3)] = oacc[dt][i];
}

__device__ __forceinline__ int tokens_split(int rows) { return rows <= 64 ? 4 : rows <= 128 ? 2 : 1; }

__global__ __launch_bounds__(512) void verify_kernel(VerifyParams p) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  const int b = blockIdx.z, kvh = blockIdx.y, chunk = blockIdx.x;
  const int w0 = p.cu_win[b], w = p.cu_win[b + 1] - w0;
  if (w == 0) return;
  const int c0 = p.cu_ctx[b], N = p.cu_ctx[b + 1] - c0;
  if (chunk * p.chunk_tok >= N + w) return;
  const int ntg = tokens_split(w * p.g);
  if (ntg == 4) verify_body<4>(p, smem, kvh, chunk, w0, w, c0, N);
  else if (ntg == 2) verify_body<2>(p, smem, kvh, chunk, w0, w, c0, N);
  else verify_body<1>(p, smem, kvh, chunk, w0, w, c0, N);
}

struct VerifyMergeParams {
  const float* ws;
  uint16_t* out;
  float* lse;
  const int* cu_ctx;
  const int* cu_win;
  int n_seqs, n_q_heads, g, ns, chunk_tok;
};

__global__ __launch_bounds__(128) void verify_merge_kernel(VerifyMergeParams p) {
  const int row = blockIdx.y, h = blockIdx.x, d = threadIdx.x;
  int b = 0;
  while (b + 1 < p.n_seqs && p.cu_win[b + 1] <= row) ++b;
  const int w = p.cu_win[b + 1] - p.cu_win[b];
  const int total = (p.cu_ctx[b + 1] - p.cu_ctx[b]) + w;
  const int nchunk = ceil_div_dev(total, p.chunk_tok);
  const int ntg = tokens_split(w * p.g);
  const float* base = p.ws + (static_cast<size_t>(row) * p.n_q_heads + h) * p.ns * kPartialFloats;
  float mm = -INFINITY;
  for (int c = 0; c < nchunk; ++c)
    for (int t = 0; t < ntg; ++t) mm = fmaxf(mm, base[static_cast<size_t>(4 * c + t) * kPartialFloats]);
  float acc = 0.f, lsum = 0.f;
  for (int c = 0; c < nchunk; ++c) {
    for (int t = 0; t < ntg; ++t) {
      const float* pp = base + static_cast<size_t>(4 * c + t) * kPartialFloats;
      const float a = exp2_diff(pp[0], mm);
      acc = fmaf(a, pp[2 + d], acc);
      lsum = fmaf(a, pp[1], lsum);
    }
  }
  const float o = lsum > 0.f ? acc / lsum : 0.f;
  p.out[(static_cast<size_t>(row) * p.n_q_heads + h) * kHeadDim + d] = static_cast<uint16_t>(float_to_bf16_bits(o));
  if (p.lse && d == 0) p.lse[static_cast<size_t>(row) * p.n_q_heads + h] = lsum > 0.f ? (mm + log2f(lsum)) * kLn2 : -INFINITY;
}

struct VerifyPlan {
  int chunk_tok, nchunk, ns;
};

static VerifyPlan make_verify_plan(const vc_full_kv* kv) {
  VerifyPlan pl{};
  const int lists = kv->n_seqs * kv->n_kv_heads;
  const int total_max = kv->max_ctx + kv->max_win;
  int64_t sum = static_cast<int64_t>(kv->sum_ctx > 0 ? kv->sum_ctx + static_cast<int64_t>(kv->n_seqs) * kv->max_win
                                                      : static_cast<int64_t>(total_max) * kv->n_seqs) * kv->n_kv_heads;
  const int target = env_int("VC_VERIFY_WGS", 512, 1, 1 << 20);
  int64_t per = ceil_div64(sum > 0 ? sum : 1, target);
  const int min_tok = env_int("VC_VERIFY_MIN_TOK", 1024, 128, 1 << 24);
  if (per < min_tok) per = min_tok;
  if (per > total_max) per = total_max > 0 ? total_max : 1;
  per = ceil_div64(per, 128) * 128;
  pl.chunk_tok = static_cast<int>(per);
  pl.nchunk = ceil_div(total_max > 0 ? total_max : 1, pl.chunk_tok);
  pl.ns = 4 * pl.nchunk;
  (void)lists;
  return pl;
}

static vc_status check_full(const vc_full_kv* kv, const char* who) {
  VC_REQUIRE(kv != nullptr, VC_ERR_INVALID_ARG, "%s: kv is NULL", who);
  VC_REQUIRE(kv->head_dim == kHeadDim, VC_ERR_UNSUPPORTED, "%s: head_dim %d (only 128)", who, kv->head_dim);
  VC_REQUIRE(kv->n_seqs >= 0 && kv->n_q_heads > 0 && kv->n_kv_heads > 0, VC_ERR_INVALID_ARG, "%s: bad sizes", who);
  VC_REQUIRE(kv->n_q_heads % kv->n_kv_heads == 0, VC_ERR_INVALID_ARG, "%s: n_q_heads %d not a multiple of n_kv_heads %d",
             who, kv->n_q_heads, kv->n_kv_heads);
  VC_REQUIRE(kv->max_ctx >= 0 && kv->max_win >= 0 && kv->sum_ctx >= 0, VC_ERR_INVALID_ARG, "%s: negative count", who);
  VC_REQUIRE(kv->max_win * (kv->n_q_heads / kv->n_kv_heads) <= 256, VC_ERR_UNSUPPORTED,
             "%s: window %d x GQA ratio %d exceeds 256 rows", who, kv->max_win, kv->n_q_heads / kv->n_kv_heads);
  VC_REQUIRE(kv->n_seqs <= 65535 && kv->n_kv_heads <= 65535 && kv->n_q_heads <= 65535, VC_ERR_UNSUPPORTED,
             "%s: batch too large for one launch", who);
  VC_REQUIRE(kv->cu_ctx != nullptr, VC_ERR_INVALID_ARG, "%s: cu_ctx is NULL", who);
  VC_REQUIRE(kv->max_ctx == 0 || (kv->k && kv->v), VC_ERR_INVALID_ARG, "%s: k or v is NULL", who);
  VC_REQUIRE(aligned16(kv->k) && aligned16(kv->v), VC_ERR_INVALID_ARG, "%s: k/v not 16-byte aligned", who);
  return VC_OK;
}

}  // namespace vc

using namespace vc;

extern "C" vc_status vc_verify_workspace_bytes(const vc_full_kv* kv, int32_t total_win, size_t* bytes) {
  vc_status st = check_full(kv, "vc_verify_workspace_bytes");
  if (st != VC_OK) return st;
  VC_REQUIRE(bytes != nullptr && total_win >= 0, VC_ERR_INVALID_ARG, "vc_verify_workspace_bytes: bad arguments");
  const VerifyPlan pl = make_verify_plan(kv);
  *bytes = static_cast<size_t>(total_win > 0 ? total_win : 1) * kv->n_q_heads * pl.ns * kPartialFloats * sizeof(float);
  return VC_OK;
}

extern "C" vc_status vc_verify_attn(vc_ctx* ctx, const vc_full_kv* kv, const void* q_win, const void* k_win,
                                    const void* v_win, const int32_t* cu_win, int32_t total_win, float softmax_scale,
                                    void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  VC_REQUIRE(ctx != nullptr, VC_ERR_INVALID_ARG, "vc_verify_attn: ctx is NULL");
  vc_status stt = check_full(kv, "vc_verify_attn");
  if (stt != VC_OK) return stt;
  VC_REQUIRE(total_win >= 0, VC_ERR_INVALID_ARG, "vc_verify_attn: total_win %d", total_win);
  if (kv->n_seqs == 0 || total_win == 0 || kv->max_win == 0) return VC_OK;
  VC_REQUIRE(q_win && k_win && v_win && cu_win && out, VC_ERR_INVALID_ARG, "vc_verify_attn: NULL pointer");
  VC_REQUIRE(aligned16(q_win) && aligned16(k_win) && aligned16(v_win) && aligned16(out), VC_ERR_INVALID_ARG,
             "vc_verify_attn: window tensors not 16-byte aligned");
  VC_REQUIRE(total_win <= 65535, VC_ERR_UNSUPPORTED, "vc_verify_attn: more than 65535 window rows");
  size_t need = 0;
  vc_verify_workspace_bytes(kv, total_win, &need);
  VC_REQUIRE(workspace != nullptr && workspace_bytes >= need, VC_ERR_WORKSPACE, "vc_verify_attn: workspace %zu bytes, need %zu",
             workspace_bytes, need);
  VC_REQUIRE(aligned16(workspace), VC_ERR_INVALID_ARG, "vc_verify_attn: workspace not 16-byte aligned");

  static bool lds_attr_set = false;
  if (!lds_attr_set) {
    VC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(verify_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               kVerifyLds));
    lds_attr_set = true;
  }
  const VerifyPlan pl = make_verify_plan(kv);
  hipStream_t st = static_cast<hipStream_t>(stream);
  VerifyParams vp{};
  vp.qw = static_cast<const uint16_t*>(q_win);
  vp.kf = static_cast<const uint16_t*>(kv->k);
  vp.vf = static_cast<const uint16_t*>(kv->v);
  vp.kw = static_cast<const uint16_t*>(k_win);
  vp.vw = static_cast<const uint16_t*>(v_win);
  vp.cu_ctx = kv->cu_ctx;
  vp.cu_win = cu_win;
  vp.ws = static_cast<float*>(workspace);
  vp.n_q_heads = kv->n_q_heads; vp.n_kv_heads = kv->n_kv_heads; vp.g = kv->n_q_heads / kv->n_kv_heads;
  vp.chunk_tok = pl.chunk_tok; vp.ns = pl.ns;
  vp.scale_log2e = softmax_scale * kLog2e;
  dim3 grid(pl.nchunk, kv->n_kv_heads, kv->n_seqs);
  hipLaunchKernelGGL(verify_kernel, grid, dim3(512), kVerifyLds, st, vp);
  VerifyMergeParams mp{};
  mp.ws = vp.ws;
  mp.out = static_cast<uint16_t*>(out);
  mp.lse = lse;
  mp.cu_ctx = kv->cu_ctx;
  mp.cu_win = cu_win;
  mp.n_seqs = kv->n_seqs; mp.n_q_heads = kv->n_q_heads; mp.g = vp.g; mp.ns = pl.ns; mp.chunk_tok = pl.chunk_tok;
  hipLaunchKernelGGL(verify_merge_kernel, dim3(kv->n_q_heads, total_win), dim3(128), 0, st, mp);
  VC_HIP(hipGetLastError());
  return VC_OK;
}
