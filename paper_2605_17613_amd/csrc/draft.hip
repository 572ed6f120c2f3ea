// Draft attention: one query token per sequence over the compressed KV cache (paper section 4.1
// step 1; section 4.2.1: the step is bounded by HBM bandwidth, so every kernel here streams its
// source exactly once with 128-bit loads and does the arithmetic in registers).
//
// Three sources (retained bf16 rows, int4/int2 block records, bf16 tail) are each cut into splits
// over their tokens; one workgroup turns one split of one (sequence, KV head) into a partial
// (m, l, O) for the g query heads of that KV head (GQA packing: K/V are read once for all of them)
// and a merge kernel combines the partials of all sources.
#include "attn_common.h"
#include "common.h"

namespace vc {

// --------------------------------------------------------------------------------------------
// bf16 rows (kept-index gather, contiguous pool, or tail)
// --------------------------------------------------------------------------------------------
struct DraftBf16Params {
  const uint16_t* q;
  const uint16_t* pk;
  const uint16_t* pv;
  const int* cu_rows;   // cu_ctx (pool) or cu_tail
  const int* keep_idx;  // GATHER only
  const int* cu_keep;   // GATHER only
  float* ws;
  int n_q_heads, n_kv_heads, g;
  int split_tok, slot0, ns;
  float scale_log2e;
};

// Lane layout: 16 lanes share one token row (lane c holds channels 8c..8c+7), so one wave load
// instruction fetches four 256-byte rows; a wave step covers 16 tokens (4 per 16-lane slot).
template <int GP, bool GATHER>
__global__ __launch_bounds__(256) void draft_bf16_kernel(DraftBf16Params p) {
  const int b = blockIdx.z, kvh = blockIdx.y, sp = blockIdx.x;
  const int row0 = p.cu_rows[b];
  const int count = GATHER ? (p.cu_keep[b + 1] - p.cu_keep[b]) : (p.cu_rows[b + 1] - row0);
  const int start = sp * p.split_tok;
  if (start >= count) return;
  const int end = min(count, start + p.split_tok);
  const int* idx = GATHER ? p.keep_idx + (static_cast<size_t>(p.cu_keep[b]) * p.n_kv_heads + static_cast<size_t>(kvh) * count)
                          : nullptr;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, ts = lane >> 4;

  float qf[GP][8];
#pragma unroll
  for (int hq = 0; hq < GP; ++hq) {
    if (hq < p.g) {
      const uint4 raw = *reinterpret_cast<const uint4*>(
          p.q + (static_cast<size_t>(b) * p.n_q_heads + kvh * p.g + hq) * kHeadDim + 8 * c);
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        qf[hq][2 * i] = bf16_lo(w[i]) * p.scale_log2e;
        qf[hq][2 * i + 1] = bf16_hi(w[i]) * p.scale_log2e;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[hq][e] = 0.f;
    }
  }

  float m[GP], l[GP], o[GP][8];
#pragma unroll
  for (int hq = 0; hq < GP; ++hq) {
    m[hq] = -INFINITY;
    l[hq] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[hq][e] = 0.f;
  }

  const size_t head_off = static_cast<size_t>(kvh) * kHeadDim + 8 * c;
  const size_t row_stride = static_cast<size_t>(p.n_kv_heads) * kHeadDim;

  for (int t0 = start + wave * 16; t0 < end; t0 += 64) {
    uint4 kk[4], vv[4];
    bool valid[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int tok = t0 + u * 4 + ts;
      valid[u] = tok < end;
      const int tokc = valid[u] ? tok : end - 1;
      const int r = GATHER ? idx[tokc] : tokc;
      const size_t off = static_cast<size_t>(row0 + r) * row_stride + head_off;
      kk[u] = *reinterpret_cast<const uint4*>(p.pk + off);
      vv[u] = *reinterpret_cast<const uint4*>(p.pv + off);
    }
    float s[4][GP];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t w[4] = {kk[u].x, kk[u].y, kk[u].z, kk[u].w};
      float kf[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        kf[2 * i] = bf16_lo(w[i]);
        kf[2 * i + 1] = bf16_hi(w[i]);
      }
#pragma unroll
      for (int hq = 0; hq < GP; ++hq) {
        float a = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) a = fmaf(qf[hq][e], kf[e], a);
        a += __shfl_xor(a, 1, 64);
        a += __shfl_xor(a, 2, 64);
        a += __shfl_xor(a, 4, 64);
        a += __shfl_xor(a, 8, 64);
        s[u][hq] = valid[u] ? a : -INFINITY;
      }
    }
    float vf[4][8];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t w[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        vf[u][2 * i] = bf16_lo(w[i]);
        vf[u][2 * i + 1] = bf16_hi(w[i]);
      }
    }
#pragma unroll
    for (int hq = 0; hq < GP; ++hq) {
      const float mn = fmaxf(fmaxf(m[hq], fmaxf(s[0][hq], s[1][hq])), fmaxf(s[2][hq], s[3][hq]));
      const float alpha = exp2_diff(m[hq], mn);
      float pu[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) pu[u] = exp2_diff(s[u][hq], mn);
      l[hq] = l[hq] * alpha + (pu[0] + pu[1]) + (pu[2] + pu[3]);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float acc = o[hq][e] * alpha;
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = fmaf(pu[u], vf[u][e], acc);
        o[hq][e] = acc;
      }
      m[hq] = mn;
    }
  }

  // merge the four 16-lane slots of the wave, then the four waves through LDS
  __shared__ float st[4][GP][kPartialFloats];
#pragma unroll
  for (int hq = 0; hq < GP; ++hq) {
    float mw = fmaxf(m[hq], __shfl_xor(m[hq], 16, 64));
    mw = fmaxf(mw, __shfl_xor(mw, 32, 64));
    const float a = exp2_diff(m[hq], mw);
    float lw = l[hq] * a;
    lw += __shfl_xor(lw, 16, 64);
    lw += __shfl_xor(lw, 32, 64);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x = o[hq][e] * a;
      x += __shfl_xor(x, 16, 64);
      x += __shfl_xor(x, 32, 64);
      if (ts == 0) st[wave][hq][2 + 8 * c + e] = x;
    }
    if (lane == 0) {
      st[wave][hq][0] = mw;
      st[wave][hq][1] = lw;
    }
  }
  __syncthreads();
  const int slot = p.slot0 + sp;
  for (int i = threadIdx.x; i < GP * kHeadDim; i += 256) {
    const int hq = i >> 7, d = i & 127;
    if (hq >= p.g) continue;
    float mm = fmaxf(fmaxf(st[0][hq][0], st[1][hq][0]), fmaxf(st[2][hq][0], st[3][hq][0]));
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float a = exp2_diff(st[w][hq][0], mm);
      acc = fmaf(a, st[w][hq][2 + d], acc);
      lsum = fmaf(a, st[w][hq][1], lsum);
    }
    float* dst = p.ws + ((static_cast<size_t>(b) * p.n_q_heads + kvh * p.g + hq) * p.ns + slot) * kPartialFloats;
    dst[2 + d] = acc;
    if (d == 0) {
      dst[0] = mm;
      dst[1] = lsum;
    }
  }
}

// --------------------------------------------------------------------------------------------
// int4 / int2 block records, dequantisation fused into fp16 MFMA tiles
// --------------------------------------------------------------------------------------------
// Scores:   s[h][t] = sum_d (q[h][d]*sK[d]) * code[t][d]  +  sum_d q[h][d]*zK[d]
//           the key scale is folded into the query once per block (a packed fp16 multiply per two
//           channels), the key zero becomes one extra MFMA per block, and the codes reach the
//           matrix core as exact small integers in fp16.
// Output:   o[h][d] = sum_t (p[h][t]*sV[t][G]) * code[t][d]  +  sum_t p[h][t]*zV[t][G]
//           likewise with the value scale folded into the probabilities per channel group G.
// MFMA 16x16x32 f16: the 16 rows of the query operand are 4 token tiles x 4 query heads, so a
// 64-token iteration produces its 256 scores with lane = token, register = head.
struct DraftQuantParams {
  const uint16_t* q;
  const uint8_t* blocks;
  const int* cu_blk;
  float* ws;
  int n_q_heads, n_kv_heads, g, nquad;
  int bps, slot0, ns;
  float scale_log2e;
};

__device__ __forceinline__ half8v as_half8(const uint32_t (&u)[4]) {
  half8v r;
  __builtin_memcpy(&r, u, 16);
  return r;
}
__device__ __forceinline__ half2v as_half2(uint32_t u) { return __builtin_bit_cast(half2v, u); }
__device__ __forceinline__ uint32_t as_u32(half2v h) { return __builtin_bit_cast(uint32_t, h); }

// One 32-bit word of eight 4-bit codes (element e at bit 16*(e&1) + 4*(e>>1)) -> eight exact fp16
// integers in element order.  0x6400 is fp16 1024: or-ing a code into its mantissa gives 1024+code
// (or 1024+16*code for the upper nibble of a byte).
__device__ __forceinline__ void unpack_i4(uint32_t x, uint32_t (&out)[4]) {
  const uint32_t magic = 0x64006400u;
  const uint32_t y = x >> 8;
  const half2v k1024 = {(_Float16)1024.f, (_Float16)1024.f};
  const half2v k16th = {(_Float16)0.0625f, (_Float16)0.0625f};
  const half2v k64 = {(_Float16)64.f, (_Float16)64.f};
  out[0] = as_u32(as_half2((x & 0x000F000Fu) | magic) - k1024);
  out[1] = as_u32(as_half2((x & 0x00F000F0u) | magic) * k16th - k64);
  out[2] = as_u32(as_half2((y & 0x000F000Fu) | magic) - k1024);
  out[3] = as_u32(as_half2((y & 0x00F000F0u) | magic) * k16th - k64);
}

// One word of sixteen 2-bit codes (element e at bit 16*(e&1) + 2*(e>>1)) -> sixteen fp16 integers.
__device__ __forceinline__ void unpack_i2(uint32_t x, uint32_t (&out)[8]) {
  const uint32_t magic = 0x64006400u;
  const uint32_t y = x >> 8;
  const half2v s0 = {(_Float16)1.f, (_Float16)1.f}, b0 = {(_Float16)1024.f, (_Float16)1024.f};
  const half2v s1 = {(_Float16)0.25f, (_Float16)0.25f}, b1 = {(_Float16)256.f, (_Float16)256.f};
  const half2v s2 = {(_Float16)0.0625f, (_Float16)0.0625f}, b2 = {(_Float16)64.f, (_Float16)64.f};
  const half2v s3 = {(_Float16)0.015625f, (_Float16)0.015625f}, b3 = {(_Float16)16.f, (_Float16)16.f};
  out[0] = as_u32(as_half2((x & 0x00030003u) | magic) * s0 - b0);
  out[1] = as_u32(as_half2((x & 0x000C000Cu) | magic) * s1 - b1);
  out[2] = as_u32(as_half2((x & 0x00300030u) | magic) * s2 - b2);
  out[3] = as_u32(as_half2((x & 0x00C000C0u) | magic) * s3 - b3);
  out[4] = as_u32(as_half2((y & 0x00030003u) | magic) * s0 - b0);
  out[5] = as_u32(as_half2((y & 0x000C000Cu) | magic) * s1 - b1);
  out[6] = as_u32(as_half2((y & 0x00300030u) | magic) * s2 - b2);
  out[7] = as_u32(as_half2((y & 0x00C000C0u) | magic) * s3 - b3);
}

__device__ __forceinline__ float4v mfma16(const uint32_t (&a)[4], const uint32_t (&b)[4], float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(a), as_half8(b), c, 0, 0, 0);
}

__device__ __forceinline__ void u4_to_arr(const uint4& v, uint32_t (&a)[4]) {
  a[0] = v.x; a[1] = v.y; a[2] = v.z; a[3] = v.w;
}

template <int BITS>
__global__ __launch_bounds__(256, 2) void draft_quant_kernel(DraftQuantParams p) {
  constexpr int TB = (BITS == 4) ? 32 : 64;   // tokens per block record
  constexpr int BPI = 64 / TB;                // records per 64-token iteration
  constexpr int NG = kHeadDim / TB;           // value channel groups
  const int b = blockIdx.z, sp = blockIdx.x;
  const int kvh = blockIdx.y / p.nquad, quad = blockIdx.y % p.nquad;
  const int nb = p.cu_blk[b + 1] - p.cu_blk[b];
  const int blk0 = sp * p.bps;
  if (blk0 >= nb) return;
  const int blk1 = min(nb, blk0 + p.bps);
  const uint8_t* rec_base =
      p.blocks + (static_cast<size_t>(p.cu_blk[b]) * p.n_kv_heads + static_cast<size_t>(kvh) * nb) * kRecordBytes;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, j = lane >> 4;
  const int tsel = (lane >> 2) & 3, hq = lane & 3;
  const int hloc = quad * 4 + hq;             // query head inside the GQA group
  const bool head_ok = hloc < p.g;

  // query operand rows: row (tsel, hq) = query head hq, channels 32j .. 32j+31 as natural fp16 pairs
  uint32_t qn[16];
  {
    const uint16_t* qp = p.q + (static_cast<size_t>(b) * p.n_q_heads + kvh * p.g + (head_ok ? hloc : 0)) * kHeadDim + 32 * j;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint4 raw = *reinterpret_cast<const uint4*>(qp + 8 * i);
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        half2v h;
        h[0] = (_Float16)(head_ok ? bf16_lo(w[k]) * p.scale_log2e : 0.f);
        h[1] = (_Float16)(head_ok ? bf16_hi(w[k]) * p.scale_log2e : 0.f);
        qn[4 * i + k] = as_u32(h);
      }
    }
  }

  __shared__ _Float16 p_lds[4][4][72];        // per wave: probabilities [head][token], fp16
  __shared__ float st[4][4][kPartialFloats];  // per wave end state for the cross-wave merge

  float m_run[4], l_part[4];
  float4v oacc[8], zacc;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    m_run[i] = -INFINITY;
    l_part[i] = 0.f;
  }
#pragma unroll
  for (int ct = 0; ct < 8; ++ct) oacc[ct] = float4v{0.f, 0.f, 0.f, 0.f};
  zacc = float4v{0.f, 0.f, 0.f, 0.f};

  for (int it = blk0 + wave * BPI; it < blk1; it += 4 * BPI) {
    const int nvalid = min(BPI, blk1 - it);   // records present in this iteration (1 or 2)
    // ---------------- scores ----------------
    // fold the key scale of this row's block into the query
    const int gsel = (BITS == 4) ? (tsel >> 1) : 0;
    const uint8_t* rec_mine = rec_base + static_cast<size_t>(it + min(gsel, nvalid - 1)) * kRecordBytes;
    uint32_t qf[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint4 sc = *reinterpret_cast<const uint4*>(rec_mine + 4096 + 64 * j + 16 * i);
      const uint32_t w[4] = {sc.x, sc.y, sc.z, sc.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) qf[4 * i + k] = as_u32(as_half2(qn[4 * i + k]) * as_half2(w[k]));
    }
    // key zero term: q . zK, the same for every token of a block
    float4v bias[BPI];
#pragma unroll
    for (int gi = 0; gi < BPI; ++gi) {
      const uint8_t* rec = rec_base + static_cast<size_t>(it + min(gi, nvalid - 1)) * kRecordBytes;
      float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const uint4 z = *reinterpret_cast<const uint4*>(rec + 4096 + 256 + 64 * j + 16 * s);
        uint32_t zb[4];
        u4_to_arr(z, zb);
        const uint32_t a[4] = {qn[4 * s], qn[4 * s + 1], qn[4 * s + 2], qn[4 * s + 3]};
        acc = mfma16(a, zb, acc);
      }
      bias[gi] = acc;
    }
    float4v sacc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int gi = (BITS == 4) ? (t >> 1) : 0;
      const uint8_t* rec = rec_base + static_cast<size_t>(it + min(gi, nvalid - 1)) * kRecordBytes;
      float4v acc = bias[gi];
      if constexpr (BITS == 4) {
        const int tt = 16 * (t & 1) + n;
        const uint4 kw = *reinterpret_cast<const uint4*>(rec + tt * 64 + 16 * j);
        const uint32_t w[4] = {kw.x, kw.y, kw.z, kw.w};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          uint32_t kb[4];
          unpack_i4(w[s], kb);
          const uint32_t a[4] = {qf[4 * s], qf[4 * s + 1], qf[4 * s + 2], qf[4 * s + 3]};
          acc = mfma16(a, kb, acc);
        }
      } else {
        const int tt = 16 * t + n;
        const uint2 kw = *reinterpret_cast<const uint2*>(rec + tt * 32 + 8 * j);
        const uint32_t w[2] = {kw.x, kw.y};
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          uint32_t kb8[8];
          unpack_i2(w[h2], kb8);
#pragma unroll
          for (int a2 = 0; a2 < 2; ++a2) {
            const int s = 2 * h2 + a2;
            const uint32_t kb[4] = {kb8[4 * a2], kb8[4 * a2 + 1], kb8[4 * a2 + 2], kb8[4 * a2 + 3]};
            const uint32_t a[4] = {qf[4 * s], qf[4 * s + 1], qf[4 * s + 2], qf[4 * s + 3]};
            acc = mfma16(a, kb, acc);
          }
        }
      }
      sacc[t] = acc;
    }
    // row (tsel = t, head i) of tile t sits in lanes 16t..16t+15, register i: lane = token
    float sv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float x = (j == 0) ? sacc[0][i] : (j == 1) ? sacc[1][i] : (j == 2) ? sacc[2][i] : sacc[3][i];
      sv[i] = (lane < nvalid * TB) ? x : -INFINITY;
    }
    // ---------------- online softmax (log2 domain) ----------------
    float pr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float mt = wave_max(sv[i]);
      const float mn = fmaxf(m_run[i], mt);
      const float alpha = exp2_diff(m_run[i], mn);
      pr[i] = exp2_diff(sv[i], mn);
      l_part[i] = l_part[i] * alpha + pr[i];
      m_run[i] = mn;
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) oacc[ct][i] *= alpha;
      zacc[i] *= alpha;
      p_lds[wave][i][lane] = (_Float16)pr[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // ---------------- output ----------------
#pragma unroll
    for (int bi = 0; bi < BPI; ++bi) {
      if (bi >= nvalid) break;
      const uint8_t* rec = rec_base + static_cast<size_t>(it + bi) * kRecordBytes;
      if constexpr (BITS == 4) {
        uint32_t pa[4];
        u4_to_arr(*reinterpret_cast<const uint4*>(&p_lds[wave][n & 3][32 * bi + 8 * j]), pa);
        uint32_t pg[NG][4];
#pragma unroll
        for (int G = 0; G < NG; ++G) {
          const uint4 sc = *reinterpret_cast<const uint4*>(rec + 4608 + 64 * G + 16 * j);
          const uint32_t w[4] = {sc.x, sc.y, sc.z, sc.w};
#pragma unroll
          for (int k = 0; k < 4; ++k) pg[G][k] = as_u32(as_half2(pa[k]) * as_half2(w[k]));
        }
        uint32_t zb[4];
        u4_to_arr(*reinterpret_cast<const uint4*>(rec + 4608 + 256 + 64 * (n & 3) + 16 * j), zb);
        zacc = mfma16(pa, zb, zacc);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const uint4 slot = *reinterpret_cast<const uint4*>(rec + 2048 + (64 * c + lane) * 16);
          const uint32_t w[4] = {slot.x, slot.y, slot.z, slot.w};
#pragma unroll
          for (int qq = 0; qq < 4; ++qq) {
            const int ct = 4 * c + qq;
            uint32_t vb[4];
            unpack_i4(w[qq], vb);
            oacc[ct] = mfma16(pg[ct >> 1], vb, oacc[ct]);
          }
        }
      } else {
        uint32_t pa[2][4], pg[NG][2][4];
#pragma unroll
        for (int a2 = 0; a2 < 2; ++a2) {
          u4_to_arr(*reinterpret_cast<const uint4*>(&p_lds[wave][n & 3][16 * j + 8 * a2]), pa[a2]);
#pragma unroll
          for (int G = 0; G < NG; ++G) {
            const uint4 sc = *reinterpret_cast<const uint4*>(rec + 4608 + 128 * G + 32 * j + 16 * a2);
            const uint32_t w[4] = {sc.x, sc.y, sc.z, sc.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) pg[G][a2][k] = as_u32(as_half2(pa[a2][k]) * as_half2(w[k]));
          }
          uint32_t zb[4];
          u4_to_arr(*reinterpret_cast<const uint4*>(rec + 4608 + 256 + 128 * (n & 1) + 32 * j + 16 * a2), zb);
          zacc = mfma16(pa[a2], zb, zacc);
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const uint4 slot = *reinterpret_cast<const uint4*>(rec + 2048 + (64 * c + lane) * 16);
          const uint32_t w[4] = {slot.x, slot.y, slot.z, slot.w};
#pragma unroll
          for (int qq = 0; qq < 4; ++qq) {
            const int ct = 4 * c + qq;
            uint32_t vb8[8];
            unpack_i2(w[qq], vb8);
#pragma unroll
            for (int a2 = 0; a2 < 2; ++a2) {
              const uint32_t vb[4] = {vb8[4 * a2], vb8[4 * a2 + 1], vb8[4 * a2 + 2], vb8[4 * a2 + 3]};
              oacc[ct] = mfma16(pg[ct >> 2][a2], vb, oacc[ct]);
            }
          }
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }

  // ---------------- end of split: wave state -> LDS -> merged partial ----------------
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lsum = wave_sum(l_part[i]);
    if (lane == 0) {
      st[wave][i][0] = m_run[i];
      st[wave][i][1] = lsum;
    }
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) {
      // zero term of (head i, channel group of tile ct) sits in lane G (column G), register i
      const int G = (BITS == 4) ? (ct >> 1) : (ct >> 2);
      const float z = __shfl(zacc[i], G, 64);
      if (j == 0) st[wave][i][2 + 16 * ct + n] = oacc[ct][i] + z;
    }
  }
  __syncthreads();
  const int slot = p.slot0 + sp;
  for (int idx = threadIdx.x; idx < 4 * kHeadDim; idx += 256) {
    const int i = idx >> 7, d = idx & 127;
    const int hl = quad * 4 + i;
    if (hl >= p.g) continue;
    const float mm = fmaxf(fmaxf(st[0][i][0], st[1][i][0]), fmaxf(st[2][i][0], st[3][i][0]));
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float a = exp2_diff(st[w][i][0], mm);
      acc = fmaf(a, st[w][i][2 + d], acc);
      lsum = fmaf(a, st[w][i][1], lsum);
    }
    float* dst = p.ws + ((static_cast<size_t>(b) * p.n_q_heads + kvh * p.g + hl) * p.ns + slot) * kPartialFloats;
    dst[2 + d] = acc;
    if (d == 0) {
      dst[0] = mm;
      dst[1] = lsum;
    }
  }
}

// --------------------------------------------------------------------------------------------
// merge of the split partials of all sources -> bf16 output (+ natural-log LSE)
// --------------------------------------------------------------------------------------------
struct DraftMergeParams {
  const float* ws;
  uint16_t* out;
  float* lse;
  const int* cu_a;      // bf16 source: cu_keep (gather) or cu_ctx (contiguous), or NULL
  const int* cu_blk;    // or NULL
  const int* cu_tail;   // or NULL
  int n_q_heads, ns;
  int split_a, s1, bps, s2, split_t;
};

__global__ __launch_bounds__(128) void draft_merge_kernel(DraftMergeParams p) {
  const int b = blockIdx.y, h = blockIdx.x, d = threadIdx.x;
  const int n1 = p.cu_a ? ceil_div_dev(p.cu_a[b + 1] - p.cu_a[b], p.split_a) : 0;
  const int n2 = p.cu_blk ? ceil_div_dev(p.cu_blk[b + 1] - p.cu_blk[b], p.bps) : 0;
  const int n3 = p.cu_tail ? ceil_div_dev(p.cu_tail[b + 1] - p.cu_tail[b], p.split_t) : 0;
  const float* base = p.ws + (static_cast<size_t>(b) * p.n_q_heads + h) * p.ns * kPartialFloats;
  float mm = -INFINITY;
  for (int s = 0; s < n1; ++s) mm = fmaxf(mm, base[static_cast<size_t>(s) * kPartialFloats]);
  for (int s = 0; s < n2; ++s) mm = fmaxf(mm, base[static_cast<size_t>(p.s1 + s) * kPartialFloats]);
  for (int s = 0; s < n3; ++s) mm = fmaxf(mm, base[static_cast<size_t>(p.s1 + p.s2 + s) * kPartialFloats]);
  float acc = 0.f, lsum = 0.f;
  for (int src = 0; src < 3; ++src) {
    const int cnt = src == 0 ? n1 : src == 1 ? n2 : n3;
    const int off = src == 0 ? 0 : src == 1 ? p.s1 : p.s1 + p.s2;
    for (int s = 0; s < cnt; ++s) {
      const float* pp = base + static_cast<size_t>(off + s) * kPartialFloats;
      const float a = exp2_diff(pp[0], mm);
      acc = fmaf(a, pp[2 + d], acc);
      lsum = fmaf(a, pp[1], lsum);
    }
  }
  const float o = lsum > 0.f ? acc / lsum : 0.f;
  p.out[(static_cast<size_t>(b) * p.n_q_heads + h) * kHeadDim + d] = static_cast<uint16_t>(float_to_bf16_bits(o));
  if (p.lse && d == 0) p.lse[static_cast<size_t>(b) * p.n_q_heads + h] = lsum > 0.f ? (mm + log2f(lsum)) * kLn2 : -INFINITY;
}

// --------------------------------------------------------------------------------------------
// host side
// --------------------------------------------------------------------------------------------
struct DraftPlan {
  int split_a, s1;   // bf16 pool source
  int bps, s2;       // block records
  int split_t, s3;   // tail
  int ns;
};

static int pick_split(int max_count, int pairs, int unit, int min_per_split) {
  if (max_count <= 0) return unit;
  const int target_wgs = env_int("VC_DRAFT_TARGET_WGS", 4096, 1, 1 << 20);
  int splits = ceil_div(target_wgs, pairs > 0 ? pairs : 1);
  if (splits < 1) splits = 1;
  int per = ceil_div(max_count, splits);
  if (per < min_per_split) per = min_per_split;
  per = ceil_div(per, unit) * unit;
  return per;
}

static DraftPlan make_plan(const vc_comp_kv* kv) {
  DraftPlan pl{};
  const int pairs = kv->n_seqs * kv->n_kv_heads;
  const bool has_a = kv->pool_k != nullptr && kv->max_keep > 0;
  const bool has_b = kv->blocks != nullptr && kv->max_blk > 0;
  const bool has_t = kv->tail_k != nullptr && kv->max_tail > 0;
  pl.split_a = pick_split(kv->max_keep, pairs, 64, env_int("VC_DRAFT_MIN_TOK", 256, 64, 1 << 20));
  pl.s1 = has_a ? ceil_div(kv->max_keep, pl.split_a) : 0;
  const int unit = kv->bits == 2 ? 4 : 8;  // one 64-token iteration per wave
  pl.bps = pick_split(kv->max_blk, pairs, unit, env_int("VC_DRAFT_MIN_BLK", 32, 4, 1 << 20));
  pl.s2 = has_b ? ceil_div(kv->max_blk, pl.bps) : 0;
  pl.split_t = pick_split(kv->max_tail, pairs, 64, 256);
  pl.s3 = has_t ? ceil_div(kv->max_tail, pl.split_t) : 0;
  pl.ns = pl.s1 + pl.s2 + pl.s3;
  if (pl.ns == 0) pl.ns = 1;
  return pl;
}

static vc_status check_comp(const vc_comp_kv* kv, const char* who) {
  VC_REQUIRE(kv != nullptr, VC_ERR_INVALID_ARG, "%s: kv is NULL", who);
  VC_REQUIRE(kv->head_dim == kHeadDim, VC_ERR_UNSUPPORTED, "%s: head_dim %d (only 128)", who, kv->head_dim);
  VC_REQUIRE(kv->n_seqs >= 0 && kv->n_q_heads > 0 && kv->n_kv_heads > 0, VC_ERR_INVALID_ARG, "%s: bad sizes", who);
  VC_REQUIRE(kv->n_q_heads % kv->n_kv_heads == 0, VC_ERR_INVALID_ARG, "%s: n_q_heads %d not a multiple of n_kv_heads %d",
             who, kv->n_q_heads, kv->n_kv_heads);
  VC_REQUIRE(kv->n_q_heads / kv->n_kv_heads <= 16, VC_ERR_UNSUPPORTED, "%s: GQA ratio above 16", who);
  VC_REQUIRE(kv->n_seqs <= 65535 && kv->n_kv_heads * 4 <= 65535, VC_ERR_UNSUPPORTED, "%s: batch too large for one launch", who);
  VC_REQUIRE(kv->max_keep >= 0 && kv->max_blk >= 0 && kv->max_tail >= 0, VC_ERR_INVALID_ARG, "%s: negative max", who);
  if (kv->pool_k || kv->pool_v) {
    VC_REQUIRE(kv->pool_k && kv->pool_v && kv->cu_ctx, VC_ERR_INVALID_ARG, "%s: pool needs pool_k, pool_v, cu_ctx", who);
    VC_REQUIRE(aligned16(kv->pool_k) && aligned16(kv->pool_v), VC_ERR_INVALID_ARG, "%s: pool not 16-byte aligned", who);
    VC_REQUIRE(!kv->keep_idx || kv->cu_keep, VC_ERR_INVALID_ARG, "%s: keep_idx needs cu_keep", who);
  }
  if (kv->blocks) {
    VC_REQUIRE(kv->cu_blk != nullptr, VC_ERR_INVALID_ARG, "%s: blocks needs cu_blk", who);
    VC_REQUIRE(aligned16(kv->blocks), VC_ERR_INVALID_ARG, "%s: blocks not 16-byte aligned", who);
    VC_REQUIRE(kv->bits == 4 || kv->bits == 2, VC_ERR_UNSUPPORTED, "%s: bits %d (block records are 4 or 2 bit)", who, kv->bits);
  }
  if (kv->tail_k || kv->tail_v) {
    VC_REQUIRE(kv->tail_k && kv->tail_v && kv->cu_tail, VC_ERR_INVALID_ARG, "%s: tail needs tail_k, tail_v, cu_tail", who);
    VC_REQUIRE(aligned16(kv->tail_k) && aligned16(kv->tail_v), VC_ERR_INVALID_ARG, "%s: tail not 16-byte aligned", who);
  }
  return VC_OK;
}

template <bool GATHER>
static void launch_bf16(int gp, dim3 grid, hipStream_t st, const DraftBf16Params& bp) {
  switch (gp) {
    case 1: hipLaunchKernelGGL((draft_bf16_kernel<1, GATHER>), grid, dim3(256), 0, st, bp); break;
    case 2: hipLaunchKernelGGL((draft_bf16_kernel<2, GATHER>), grid, dim3(256), 0, st, bp); break;
    case 4: hipLaunchKernelGGL((draft_bf16_kernel<4, GATHER>), grid, dim3(256), 0, st, bp); break;
    case 8: hipLaunchKernelGGL((draft_bf16_kernel<8, GATHER>), grid, dim3(256), 0, st, bp); break;
    default: hipLaunchKernelGGL((draft_bf16_kernel<16, GATHER>), grid, dim3(256), 0, st, bp); break;
  }
}

}  // namespace vc

using namespace vc;

extern "C" vc_status vc_draft_workspace_bytes(const vc_comp_kv* kv, size_t* bytes) {
  vc_status st = check_comp(kv, "vc_draft_workspace_bytes");
  if (st != VC_OK) return st;
  VC_REQUIRE(bytes != nullptr, VC_ERR_INVALID_ARG, "vc_draft_workspace_bytes: bytes is NULL");
  const DraftPlan pl = make_plan(kv);
  const size_t rows = static_cast<size_t>(kv->n_seqs > 0 ? kv->n_seqs : 1) * kv->n_q_heads;
  *bytes = rows * pl.ns * kPartialFloats * sizeof(float);
  return VC_OK;
}

extern "C" vc_status vc_draft_attn(vc_ctx* ctx, const vc_comp_kv* kv, const void* q, float softmax_scale, void* out,
                                   float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  VC_REQUIRE(ctx != nullptr, VC_ERR_INVALID_ARG, "vc_draft_attn: ctx is NULL");
  vc_status stt = check_comp(kv, "vc_draft_attn");
  if (stt != VC_OK) return stt;
  if (kv->n_seqs == 0) return VC_OK;
  VC_REQUIRE(q && out, VC_ERR_INVALID_ARG, "vc_draft_attn: q or out is NULL");
  VC_REQUIRE(aligned16(q) && aligned16(out), VC_ERR_INVALID_ARG, "vc_draft_attn: q/out not 16-byte aligned");
  size_t need = 0;
  vc_draft_workspace_bytes(kv, &need);
  VC_REQUIRE(workspace != nullptr && workspace_bytes >= need, VC_ERR_WORKSPACE, "vc_draft_attn: workspace %zu bytes, need %zu",
             workspace_bytes, need);
  VC_REQUIRE(aligned16(workspace), VC_ERR_INVALID_ARG, "vc_draft_attn: workspace not 16-byte aligned");

  const DraftPlan pl = make_plan(kv);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int g = kv->n_q_heads / kv->n_kv_heads;
  int gp = 1;
  while (gp < g) gp <<= 1;
  const float sl2 = softmax_scale * kLog2e;
  float* ws = static_cast<float*>(workspace);

  if (pl.s1 > 0) {
    DraftBf16Params bp{};
    bp.q = static_cast<const uint16_t*>(q);
    bp.pk = static_cast<const uint16_t*>(kv->pool_k);
    bp.pv = static_cast<const uint16_t*>(kv->pool_v);
    bp.cu_rows = kv->cu_ctx;
    bp.keep_idx = kv->keep_idx;
    bp.cu_keep = kv->cu_keep;
    bp.ws = ws;
    bp.n_q_heads = kv->n_q_heads; bp.n_kv_heads = kv->n_kv_heads; bp.g = g;
    bp.split_tok = pl.split_a; bp.slot0 = 0; bp.ns = pl.ns;
    bp.scale_log2e = sl2;
    dim3 grid(pl.s1, kv->n_kv_heads, kv->n_seqs);
    if (kv->keep_idx) launch_bf16<true>(gp, grid, st, bp); else launch_bf16<false>(gp, grid, st, bp);
  }
  if (pl.s2 > 0) {
    DraftQuantParams qp{};
    qp.q = static_cast<const uint16_t*>(q);
    qp.blocks = static_cast<const uint8_t*>(kv->blocks);
    qp.cu_blk = kv->cu_blk;
    qp.ws = ws;
    qp.n_q_heads = kv->n_q_heads; qp.n_kv_heads = kv->n_kv_heads; qp.g = g;
    qp.nquad = ceil_div(g, 4);
    qp.bps = pl.bps; qp.slot0 = pl.s1; qp.ns = pl.ns;
    qp.scale_log2e = sl2;
    dim3 grid(pl.s2, kv->n_kv_heads * qp.nquad, kv->n_seqs);
    if (kv->bits == 4) hipLaunchKernelGGL(draft_quant_kernel<4>, grid, dim3(256), 0, st, qp);
    else hipLaunchKernelGGL(draft_quant_kernel<2>, grid, dim3(256), 0, st, qp);
  }
  if (pl.s3 > 0) {
    DraftBf16Params bp{};
    bp.q = static_cast<const uint16_t*>(q);
    bp.pk = static_cast<const uint16_t*>(kv->tail_k);
    bp.pv = static_cast<const uint16_t*>(kv->tail_v);
    bp.cu_rows = kv->cu_tail;
    bp.ws = ws;
    bp.n_q_heads = kv->n_q_heads; bp.n_kv_heads = kv->n_kv_heads; bp.g = g;
    bp.split_tok = pl.split_t; bp.slot0 = pl.s1 + pl.s2; bp.ns = pl.ns;
    bp.scale_log2e = sl2;
    dim3 grid(pl.s3, kv->n_kv_heads, kv->n_seqs);
    launch_bf16<false>(gp, grid, st, bp);
  }
  DraftMergeParams mp{};
  mp.ws = ws;
  mp.out = static_cast<uint16_t*>(out);
  mp.lse = lse;
  mp.cu_a = pl.s1 > 0 ? (kv->keep_idx ? kv->cu_keep : kv->cu_ctx) : nullptr;
  mp.cu_blk = pl.s2 > 0 ? kv->cu_blk : nullptr;
  mp.cu_tail = pl.s3 > 0 ? kv->cu_tail : nullptr;
  mp.n_q_heads = kv->n_q_heads; mp.ns = pl.ns;
  mp.split_a = pl.split_a; mp.s1 = pl.s1; mp.bps = pl.bps; mp.s2 = pl.s2; mp.split_t = pl.split_t;
  hipLaunchKernelGGL(draft_merge_kernel, dim3(kv->n_q_heads, kv->n_seqs), dim3(128), 0, st, mp);
  VC_HIP(hipGetLastError());
  return VC_OK;
}
