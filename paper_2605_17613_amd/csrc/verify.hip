// Verify attention: a window of drafted tokens attends causally to the full bf16 KV plus the
// window itself (paper section 4.1 step 2).  The g query heads of a KV head times the w window
// positions form w*g rows that share every K/V row, so the row dimension is a real MFMA tile.
//
// Formulation (per 32-token tile, bf16 MFMA 32x32x16, fp32 accumulation):
//   S^T[token][row]  = K[token][:] . Q[row][:]      A = K tile, B = Q^T (held in registers)
//   O^T[d][row]     += V^T[d][token] * P^T[token][row]
// With rows on the lanes every lane owns the softmax state of one row, and the probabilities
// leave the first product already in the register layout the second product wants.
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
  int split_tok, ns, nrp;
  float scale_log2e;
};

constexpr int kLdsStride = 136;  // bf16 elements per LDS row (128 + 8 pad: conflict-free 16-byte reads)

__device__ __forceinline__ float16v mfma32(bf16x8v a, bf16x8v b, float16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8v load_bf16x8(const uint16_t* p) {
  bf16x8v r;
  const uint4 raw = *reinterpret_cast<const uint4*>(p);
  __builtin_memcpy(&r, &raw, 16);
  return r;
}

template <int NRT>
__global__ __launch_bounds__(64) void verify_kernel(VerifyParams p) {
  constexpr int RW = 32 * NRT;
  const int b = blockIdx.z, kvh = blockIdx.y;
  const int rp = blockIdx.x % p.nrp, sp = blockIdx.x / p.nrp;
  const int w0 = p.cu_win[b], w = p.cu_win[b + 1] - w0;
  const int R = w * p.g;
  if (rp * RW >= R) return;
  const int c0 = p.cu_ctx[b], N = p.cu_ctx[b + 1] - c0;
  const int total = N + w;
  const int t0 = sp * p.split_tok;
  if (t0 >= total) return;
  const int t1 = min(total, t0 + p.split_tok);
  const int lane = threadIdx.x;
  const int n = lane & 31, hh = lane >> 5;

  int iw[NRT], hq[NRT];
  bool row_ok[NRT];
  bf16x8v qb[NRT][8];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    const int r = rp * RW + rt * 32 + n;
    row_ok[rt] = r < R;
    const int rc = row_ok[rt] ? r : R - 1;
    iw[rt] = rc / p.g;
    hq[rt] = rc % p.g;
    const uint16_t* qp = p.qw + (static_cast<size_t>(w0 + iw[rt]) * p.n_q_heads + kvh * p.g + hq[rt]) * kHeadDim + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qb[rt][ks] = load_bf16x8(qp + 16 * ks);
  }

  float m[NRT], l[NRT];
  float16v oacc[NRT][4];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    m[rt] = -INFINITY;
    l[rt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[rt][dt][i] = 0.f;
  }

  __shared__ __attribute__((aligned(16))) uint16_t Ks[32 * kLdsStride];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[32 * kLdsStride];
  const size_t row_stride = static_cast<size_t>(p.n_kv_heads) * kHeadDim;
  const size_t head_off = static_cast<size_t>(kvh) * kHeadDim;

  for (int t = t0; t < t1; t += 32) {
    // stage the tile: 32 tokens x 256 bytes of K and of V, 16 bytes per lane per step
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const int chunk = c * 64 + lane;
      const int tt = chunk >> 4, part = chunk & 15;
      const int tok = t + tt;
      uint4 kx = {0u, 0u, 0u, 0u}, vx = {0u, 0u, 0u, 0u};
      if (tok < N) {
        const size_t off = static_cast<size_t>(c0 + tok) * row_stride + head_off + 8 * part;
        kx = *reinterpret_cast<const uint4*>(p.kf + off);
        vx = *reinterpret_cast<const uint4*>(p.vf + off);
      } else if (tok < total) {
        const size_t off = static_cast<size_t>(w0 + tok - N) * row_stride + head_off + 8 * part;
        kx = *reinterpret_cast<const uint4*>(p.kw + off);
        vx = *reinterpret_cast<const uint4*>(p.vw + off);
      }
      *reinterpret_cast<uint4*>(&Ks[tt * kLdsStride + 8 * part]) = kx;
      *reinterpret_cast<uint4*>(&Vs[tt * kLdsStride + 8 * part]) = vx;
    }
    __syncthreads();

    bf16x8v pb[NRT][2];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      float16v acc;
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8v a = load_bf16x8(&Ks[n * kLdsStride + 16 * ks + 8 * hh]);
        acc = mfma32(a, qb[rt][ks], acc);
      }
      // register i of this lane is token row 8*(i/4) + 4*hh + i%4 of the tile, for row n
      float s[16];
      float mt = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int tok = t + 8 * (i >> 2) + 4 * hh + (i & 3);
        const bool ok = tok < t1 && (tok < N || tok - N <= iw[rt]);
        s[i] = ok ? acc[i] * p.scale_log2e : -INFINITY;
        mt = fmaxf(mt, s[i]);
      }
      mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
      const float mn = fmaxf(m[rt], mt);
      const float alpha = exp2_diff(m[rt], mn);
      float ps = 0.f;
      float pr[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        pr[i] = exp2_diff(s[i], mn);
        ps += pr[i];
      }
      l[rt] = l[rt] * alpha + ps;
      m[rt] = mn;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[rt][dt][i] *= alpha;
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[rt][kk][e] = (__bf16)pr[8 * kk + e];
    }
    // O^T += V^T P^T : A = V^T[d][token], element e of k-step kk is token row 16kk + 8(e/4) + 4hh + e%4
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        bf16x8v av;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int rho = 16 * kk + 8 * (e >> 2) + 4 * hh + (e & 3);
          av[e] = __builtin_bit_cast(__bf16, Vs[rho * kLdsStride + 32 * dt + n]);
        }
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) oacc[rt][dt] = mfma32(av, pb[rt][kk], oacc[rt][dt]);
      }
    }
    __syncthreads();
  }

#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    const float lt = l[rt] + __shfl_xor(l[rt], 32, 64);
    if (!row_ok[rt]) continue;
    const size_t grow = static_cast<size_t>(w0 + iw[rt]) * p.n_q_heads + kvh * p.g + hq[rt];
    float* dst = p.ws + (grow * p.ns + sp) * kPartialFloats;
    if (hh == 0) {
      dst[0] = m[rt];
      dst[1] = lt;
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) dst[2 + 32 * dt + 8 * (i >> 2) + 4 * hh + (i & 3)] = oacc[rt][dt][i];
  }
}

struct VerifyMergeParams {
  const float* ws;
  uint16_t* out;
  float* lse;
  const int* cu_ctx;
  const int* cu_win;
  int n_seqs, n_q_heads, ns, split_tok;
};

__global__ __launch_bounds__(128) void verify_merge_kernel(VerifyMergeParams p) {
  const int row = blockIdx.y, h = blockIdx.x, d = threadIdx.x;
  int b = 0;
  while (b + 1 < p.n_seqs && p.cu_win[b + 1] <= row) ++b;
  const int total = (p.cu_ctx[b + 1] - p.cu_ctx[b]) + (p.cu_win[b + 1] - p.cu_win[b]);
  const int cnt = ceil_div_dev(total, p.split_tok);
  const float* base = p.ws + (static_cast<size_t>(row) * p.n_q_heads + h) * p.ns * kPartialFloats;
  float mm = -INFINITY;
  for (int s = 0; s < cnt; ++s) mm = fmaxf(mm, base[static_cast<size_t>(s) * kPartialFloats]);
  float acc = 0.f, lsum = 0.f;
  for (int s = 0; s < cnt; ++s) {
    const float* pp = base + static_cast<size_t>(s) * kPartialFloats;
    const float a = exp2_diff(pp[0], mm);
    acc = fmaf(a, pp[2 + d], acc);
    lsum = fmaf(a, pp[1], lsum);
  }
  const float o = lsum > 0.f ? acc / lsum : 0.f;
  p.out[(static_cast<size_t>(row) * p.n_q_heads + h) * kHeadDim + d] = static_cast<uint16_t>(float_to_bf16_bits(o));
  if (p.lse && d == 0) p.lse[static_cast<size_t>(row) * p.n_q_heads + h] = lsum > 0.f ? (mm + log2f(lsum)) * kLn2 : -INFINITY;
}

struct VerifyPlan {
  int split_tok, ns, nrp, nrt;
};

static VerifyPlan make_verify_plan(const vc_full_kv* kv) {
  VerifyPlan pl{};
  const int g = kv->n_q_heads / kv->n_kv_heads;
  const int rmax = kv->max_win * g;
  pl.nrt = rmax <= 32 ? 1 : 2;
  pl.nrp = ceil_div(rmax > 0 ? rmax : 1, 32 * pl.nrt);
  const int pairs = kv->n_seqs * kv->n_kv_heads * pl.nrp;
  const int target = env_int("VC_VERIFY_TARGET_WGS", 4096, 1, 1 << 20);
  int splits = ceil_div(target, pairs > 0 ? pairs : 1);
  const int total = kv->max_ctx + kv->max_win;
  int per = ceil_div(total > 0 ? total : 1, splits);
  const int min_tok = env_int("VC_VERIFY_MIN_TOK", 1024, 32, 1 << 24);
  if (per < min_tok) per = min_tok;
  per = ceil_div(per, 32) * 32;
  pl.split_tok = per;
  pl.ns = ceil_div(total > 0 ? total : 1, per);
  return pl;
}

static vc_status check_full(const vc_full_kv* kv, const char* who) {
  VC_REQUIRE(kv != nullptr, VC_ERR_INVALID_ARG, "%s: kv is NULL", who);
  VC_REQUIRE(kv->head_dim == kHeadDim, VC_ERR_UNSUPPORTED, "%s: head_dim %d (only 128)", who, kv->head_dim);
  VC_REQUIRE(kv->n_seqs >= 0 && kv->n_q_heads > 0 && kv->n_kv_heads > 0, VC_ERR_INVALID_ARG, "%s: bad sizes", who);
  VC_REQUIRE(kv->n_q_heads % kv->n_kv_heads == 0, VC_ERR_INVALID_ARG, "%s: n_q_heads %d not a multiple of n_kv_heads %d",
             who, kv->n_q_heads, kv->n_kv_heads);
  VC_REQUIRE(kv->n_q_heads / kv->n_kv_heads <= 16, VC_ERR_UNSUPPORTED, "%s: GQA ratio above 16", who);
  VC_REQUIRE(kv->max_ctx >= 0 && kv->max_win >= 0, VC_ERR_INVALID_ARG, "%s: negative max", who);
  VC_REQUIRE(kv->max_win <= 64, VC_ERR_UNSUPPORTED, "%s: window %d above 64", who, kv->max_win);
  VC_REQUIRE(kv->n_seqs <= 65535 && kv->n_kv_heads <= 65535, VC_ERR_UNSUPPORTED, "%s: batch too large for one launch", who);
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
  vp.split_tok = pl.split_tok; vp.ns = pl.ns; vp.nrp = pl.nrp;
  vp.scale_log2e = softmax_scale * kLog2e;
  dim3 grid(pl.ns * pl.nrp, kv->n_kv_heads, kv->n_seqs);
  if (pl.nrt == 1) hipLaunchKernelGGL(verify_kernel<1>, grid, dim3(64), 0, st, vp);
  else hipLaunchKernelGGL(verify_kernel<2>, grid, dim3(64), 0, st, vp);
  VerifyMergeParams mp{};
  mp.ws = vp.ws;
  mp.out = static_cast<uint16_t*>(out);
  mp.lse = lse;
  mp.cu_ctx = kv->cu_ctx;
  mp.cu_win = cu_win;
  mp.n_seqs = kv->n_seqs; mp.n_q_heads = kv->n_q_heads; mp.ns = pl.ns; mp.split_tok = pl.split_tok;
  hipLaunchKernelGGL(verify_merge_kernel, dim3(kv->n_q_heads, total_win), dim3(128), 0, st, mp);
  VC_HIP(hipGetLastError());
  return VC_OK;
}
