// Compressor-side kernels (paper section 6, Compressor interface): the quantising compress()
// (bf16 K, V -> int4 / int2 block records), its decompress() (records -> bf16 K, V, what a remote
// drafter materialises), and the kept-position lists an online update() derives from scores.
//
// All three are bandwidth work: one wave owns one 5120-byte record (32 or 64 tokens of one KV
// head); rows are fetched with 16 bytes per lane, four token rows per wave load.
#include "attn_common.h"
#include "common.h"

namespace vc {

struct QuantParams {
  const uint16_t* k;      // bf16 [tokens][Hkv][128]  (compress: in, decompress: out)
  const uint16_t* v;
  uint16_t* k_out;
  uint16_t* v_out;
  const uint8_t* blocks;  // decompress: in
  uint8_t* blocks_out;    // compress: out
  const int* cu_ctx;
  const int* cu_blk;
  int n_kv_heads;
};

template <int BITS>
struct QuantGeom {
  static constexpr int TB = BITS == 4 ? 32 : 64;     // tokens per record = channels per value group
  static constexpr int LEVELS = (1 << BITS) - 1;
  static constexpr int E = 32 / BITS;                // codes per 32-bit word
  static constexpr int NL = TB / 4;                  // wave loads per matrix (4 token rows each)
};

// bit position of element e of a code word
template <int BITS>
__device__ __forceinline__ constexpr int field_shift(int e) { return 16 * (e & 1) + BITS * (e >> 1); }

__device__ __forceinline__ void unpack8(const uint4& r, float (&x)[8]) {
  x[0] = bf16_lo(r.x); x[1] = bf16_hi(r.x); x[2] = bf16_lo(r.y); x[3] = bf16_hi(r.y);
  x[4] = bf16_lo(r.z); x[5] = bf16_hi(r.z); x[6] = bf16_lo(r.w); x[7] = bf16_hi(r.w);
}

// fp16 scale and zero point of a group from its minimum and maximum, and the factor the codes are
// computed with: all float32, one rounding per step; code = clamp(rne((x - zero) * inv))
template <int LEVELS>
__device__ __forceinline__ void group_meta(float mn, float mx, _Float16& sh, _Float16& zh, float& zf, float& inv) {
  sh = static_cast<_Float16>(__fdiv_rn(mx - mn, static_cast<float>(LEVELS)));
  zh = static_cast<_Float16>(mn + 0.0f);           // a minimum of -0 is stored as +0
  const float sf = static_cast<float>(sh);
  zf = static_cast<float>(zh);
  inv = sf > 0.f ? __fdiv_rn(1.0f, sf) : 0.f;      // a constant group: every code 0
}

// (the conversion instruction rounds to nearest even and saturates at 0 and 255 by itself, and puts the
// result into a byte of choice of a word: rounding, lower clamp, conversion and packing in one)
template <int LEVELS>
__device__ __forceinline__ uint32_t code_into(float x, float zf, float inv, uint32_t byte, uint32_t word) {
  return __builtin_amdgcn_cvt_pk_u8_f32(fminf((x - zf) * inv, static_cast<float>(LEVELS)), byte, word);
}
template <int LEVELS>
__device__ __forceinline__ uint32_t code_of(float x, float zf, float inv) { return code_into<LEVELS>(x, zf, inv, 0u, 0u); }

// Four 2-bit codes, one per byte of x -> one byte (code of byte k at bits 2k)
__device__ __forceinline__ uint32_t squeeze2(uint32_t x) {
  x |= x >> 6;       // bytes 0 and 2: two codes each
  x |= x >> 12;      // byte 0: four codes
  return x & 0xFFu;
}

// ---------------------------------------------------------------------------------------------
// compress: grid (Hkv, ceil(max_blk / 4), n_seqs), 4 waves, one record per wave.  The KV head is the
// fastest grid dimension: the workgroups that are resident together then read all the heads' 256-byte
// pieces of the same token rows, instead of one head's piece of eight times as many rows.
// ---------------------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(256) void compress_quant_kernel(QuantParams p) {
  using G = QuantGeom<BITS>;
  constexpr int TB = G::TB, LEVELS = G::LEVELS, NL = G::NL;
  static_assert(G::E == NL, "a lane's NL consecutive tokens are exactly the tokens of one value code word");
  __shared__ __attribute__((aligned(16))) uint32_t words_all[4][512];            // value code words, in record order
  __shared__ __attribute__((aligned(16))) uint16_t vmeta_all[4][256];            // value scale[g][t], zero[g][t]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lg = lane >> 4, lc = lane & 15;
  const int b = blockIdx.z, kvh = blockIdx.x, blk = blockIdx.y * 4 + wave;
  const int nb = p.cu_blk[b + 1] - p.cu_blk[b];
  const bool live = blk < nb;                        // the barrier below is reached by every wave
  uint32_t* words = words_all[wave];
  uint16_t* vmeta = vmeta_all[wave];
  const size_t rs = static_cast<size_t>(p.n_kv_heads) * kHeadDim;
  const size_t row0 = (static_cast<size_t>(p.cu_ctx[b]) + static_cast<size_t>(live ? blk : 0) * TB) * rs +
                      static_cast<size_t>(kvh) * kHeadDim + 8 * lc;
  uint8_t* rec = p.blocks_out + (static_cast<size_t>(p.cu_blk[b]) * p.n_kv_heads + static_cast<size_t>(kvh) * nb +
                                 (live ? blk : 0)) * kRecordBytes;
  // Lane (lg, lc) owns channels 8*lc .. +7 of the NL consecutive tokens lg*NL .. lg*NL + NL - 1 (a wave load
  // still fetches four whole rows).  Those tokens are the ones a value code word holds for one channel, so
  // the lane packs its eight value words by itself; nothing is transposed through memory.
  uint4 kraw[NL], vraw[NL];
  if (live) {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      kraw[i] = ld_stream(reinterpret_cast<const uint4*>(p.k + row0 + static_cast<size_t>(lg * NL + i) * rs));
      vraw[i] = ld_stream(reinterpret_cast<const uint4*>(p.v + row0 + static_cast<size_t>(lg * NL + i) * rs));
    }
    // ---- keys: one group per channel over the TB tokens
    float mn[8], mx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { mn[e] = INFINITY; mx[e] = -INFINITY; }
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      float x[8];
      unpack8(kraw[i], x);
#pragma unroll
      for (int e = 0; e < 8; ++e) { mn[e] = fminf(mn[e], x[e]); mx[e] = fmaxf(mx[e], x[e]); }
    }
    float zf[8], inv[8];
    uint32_t sw[4], zw[4];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      mn[e] = fminf(mn[e], __shfl_xor(mn[e], 16, 64)); mx[e] = fmaxf(mx[e], __shfl_xor(mx[e], 16, 64));
      mn[e] = fminf(mn[e], __shfl_xor(mn[e], 32, 64)); mx[e] = fmaxf(mx[e], __shfl_xor(mx[e], 32, 64));
      _Float16 sh, zh;
      group_meta<LEVELS>(mn[e], mx[e], sh, zh, zf[e], inv[e]);
      const uint32_t sb = __builtin_bit_cast(uint16_t, sh), zb = __builtin_bit_cast(uint16_t, zh);
      if (e & 1) { sw[e >> 1] |= sb << 16; zw[e >> 1] |= zb << 16; } else { sw[e >> 1] = sb; zw[e >> 1] = zb; }
    }
    if (lg == 0) {
      *reinterpret_cast<uint4*>(rec + 4096 + 16 * lc) = make_uint4(sw[0], sw[1], sw[2], sw[3]);
      *reinterpret_cast<uint4*>(rec + 4352 + 16 * lc) = make_uint4(zw[0], zw[1], zw[2], zw[3]);
    }
    // Element e of a code word sits at bit 16*(e & 1) + BITS*(e >> 1): the even elements fill the low half
    // of the word, the odd ones the high half.  Codes are converted straight into the bytes of words that
    // collect the even and the odd elements, and squeezed together from there - a few operations per word
    // instead of a shift and an or per code.
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      float x[8];
      unpack8(kraw[i], x);
      const int tk = lg * NL + i;
      uint32_t ev = 0, od = 0;
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        ev = code_into<LEVELS>(x[e], zf[e], inv[e], e >> 1, ev);
        od = code_into<LEVELS>(x[e + 1], zf[e + 1], inv[e + 1], e >> 1, od);
      }
      if (BITS == 4) {
        const uint32_t te = ev | (ev >> 4), to = od | (od >> 4);   // bytes 0 and 2: two codes each
        *reinterpret_cast<uint32_t*>(rec + tk * 64 + 4 * lc) = __builtin_amdgcn_perm(to, te, 0x06040200u);
      } else {
        // 16 channels per word: this lane holds elements 8*(lc & 1) .. +7, its neighbour the rest
        uint32_t w = (squeeze2(ev) | (squeeze2(od) << 16)) << (8 * (lc & 1));
        w |= __shfl_xor(w, 1, 64);
        if ((lc & 1) == 0) *reinterpret_cast<uint32_t*>(rec + tk * 32 + 4 * (lc >> 1)) = w;
      }
    }
    // ---- values: one group per token over TB consecutive channels (TB / 8 lanes); the codes of channel
    // 8*lc + e over this lane's tokens collect in vev / vod [e] (even / odd tokens, four per word)
    uint32_t vev[8][NL / 8], vod[8][NL / 8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
      for (int h = 0; h < NL / 8; ++h) { vev[e][h] = 0; vod[e][h] = 0; }
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      float x[8];
      unpack8(vraw[i], x);
      float lo = x[0], hi = x[0];
#pragma unroll
      for (int e = 1; e < 8; ++e) { lo = fminf(lo, x[e]); hi = fmaxf(hi, x[e]); }
#pragma unroll
      for (int off = 1; off < TB / 8; off <<= 1) {
        lo = fminf(lo, __shfl_xor(lo, off, 64));
        hi = fmaxf(hi, __shfl_xor(hi, off, 64));
      }
      _Float16 sh, zh;
      float zfv, invv;
      group_meta<LEVELS>(lo, hi, sh, zh, zfv, invv);
      const int tk = lg * NL + i;
      const int grp = (8 * lc) / TB;
      if ((8 * lc) % TB == 0) {
        vmeta[grp * TB + tk] = __builtin_bit_cast(uint16_t, sh);
        vmeta[128 + grp * TB + tk] = __builtin_bit_cast(uint16_t, zh);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (i & 1) vod[e][i >> 3] = code_into<LEVELS>(x[e], zfv, invv, (i >> 1) & 3, vod[e][i >> 3]);
        else vev[e][i >> 3] = code_into<LEVELS>(x[e], zfv, invv, (i >> 1) & 3, vev[e][i >> 3]);
      }
    }
    // value code words: word W = 4 * slot + q, slot = 64c + 16j + n, holds channel 64c + 16q + n of the
    // tokens E*j .. E*j + E - 1 - here j = lg
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int ch = 8 * lc + e;
      const int W = 4 * (64 * (ch >> 6) + 16 * lg + (ch & 15)) + ((ch >> 4) & 3);
      uint32_t w;
      if (BITS == 4) {
        const uint32_t te = vev[e][0] | (vev[e][0] >> 4), to = vod[e][0] | (vod[e][0] >> 4);
        w = __builtin_amdgcn_perm(to, te, 0x06040200u);
      } else {
        w = (squeeze2(vev[e][0]) | (squeeze2(vev[e][NL / 8 - 1]) << 8)) |
            ((squeeze2(vod[e][0]) | (squeeze2(vod[e][NL / 8 - 1]) << 8)) << 16);
      }
      words[W] = w;
    }
  }
  __syncthreads();
  if (live) {
    // the 2048 bytes of value code words and the 512 bytes of value scales / zeros leave as 16-byte stores
#pragma unroll
    for (int m = 0; m < 2; ++m)
      *reinterpret_cast<uint4*>(rec + 2048 + 16 * (64 * m + lane)) = *reinterpret_cast<const uint4*>(words + 4 * (64 * m + lane));
    *reinterpret_cast<uint2*>(rec + 4608 + 8 * lane) = *reinterpret_cast<const uint2*>(vmeta + 4 * lane);
  }
}

// ---------------------------------------------------------------------------------------------
// decompress: same geometry; the record is staged in LDS, rows leave as 16-byte stores
// x_hat = fma(scale, code, zero) in float32 (exact whenever scale*code and zero are within 2^9 of
// each other in magnitude, i.e. for any group a min/max quantiser produces), rounded once to bf16
// ---------------------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(256) void decompress_quant_kernel(QuantParams p) {
  using G = QuantGeom<BITS>;
  constexpr int TB = G::TB, E = G::E, NL = G::NL;
  constexpr uint32_t MASK = (1u << BITS) - 1u;
  __shared__ __attribute__((aligned(16))) uint8_t rec_all[4][kRecordBytes];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lg = lane >> 4, lc = lane & 15;
  const int b = blockIdx.z, kvh = blockIdx.x, blk = blockIdx.y * 4 + wave;
  const int nb = p.cu_blk[b + 1] - p.cu_blk[b];
  const bool live = blk < nb;
  uint8_t* rec = rec_all[wave];
  if (live) {
    const uint8_t* src = p.blocks + (static_cast<size_t>(p.cu_blk[b]) * p.n_kv_heads + static_cast<size_t>(kvh) * nb + blk) *
                                        kRecordBytes;
#pragma unroll
    for (int m = 0; m < 5; ++m)
      *reinterpret_cast<uint4*>(rec + 16 * (64 * m + lane)) = ld_stream(reinterpret_cast<const uint4*>(src + 16 * (64 * m + lane)));
  }
  __syncthreads();
  if (!live) return;
  const size_t rs = static_cast<size_t>(p.n_kv_heads) * kHeadDim;
  const size_t row0 = (static_cast<size_t>(p.cu_ctx[b]) + static_cast<size_t>(blk) * TB) * rs +
                      static_cast<size_t>(kvh) * kHeadDim + 8 * lc;
  const _Float16* meta = reinterpret_cast<const _Float16*>(rec + 4096);
  float ks[8], kz[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    ks[e] = static_cast<float>(meta[8 * lc + e]);
    kz[e] = static_cast<float>(meta[128 + 8 * lc + e]);
  }
  const int grp = (8 * lc) / TB;
  // value words of this lane's 8 channels: channel 8*lc + e -> c = lc >> 3, q = (lc >> 1) & 3, n = 8*(lc & 1) + e
  const int vc = lc >> 3, vq = (lc >> 1) & 3, vn0 = 8 * (lc & 1);
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int tk = 4 * i + lg;
    uint32_t kw;
    int ebase;
    if (BITS == 4) { kw = *reinterpret_cast<const uint32_t*>(rec + tk * 64 + 4 * lc); ebase = 0; }
    else { kw = *reinterpret_cast<const uint32_t*>(rec + tk * 32 + 4 * (lc >> 1)); ebase = 8 * (lc & 1); }
    uint32_t ko[4], vo[4];
    const int j = tk / E, ee = tk % E;
    const float vs = static_cast<float>(meta[256 + grp * TB + tk]);
    const float vz = static_cast<float>(meta[384 + grp * TB + tk]);
    const int vshift = 16 * (ee & 1) + BITS * (ee >> 1);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int el = ebase + e;
      const uint32_t kcode = (kw >> (16 * (el & 1) + BITS * (el >> 1))) & MASK;
      const uint32_t kb = float_to_bf16_bits(fmaf(ks[e], static_cast<float>(kcode), kz[e]));
      const uint32_t vword = *reinterpret_cast<const uint32_t*>(rec + 2048 + 16 * (64 * vc + 16 * j + vn0 + e) + 4 * vq);
      const uint32_t vcode = (vword >> vshift) & MASK;
      const uint32_t vb = float_to_bf16_bits(fmaf(vs, static_cast<float>(vcode), vz));
      if (e & 1) { ko[e >> 1] |= kb << 16; vo[e >> 1] |= vb << 16; } else { ko[e >> 1] = kb; vo[e >> 1] = vb; }
    }
    st_stream(reinterpret_cast<uint4*>(p.k_out + row0 + static_cast<size_t>(tk) * rs), make_uint4(ko[0], ko[1], ko[2], ko[3]));
    st_stream(reinterpret_cast<uint4*>(p.v_out + row0 + static_cast<size_t>(tk) * rs), make_uint4(vo[0], vo[1], vo[2], vo[3]));
  }
}

// ---------------------------------------------------------------------------------------------
// kept positions from scores: one workgroup of 1024 threads per (sequence, head) list.
// Radix select (4 passes of 8 bits) finds the score threshold among the free positions; ties at
// the threshold go to the lowest positions; thread i then owns the contiguous run i of positions
// so that the output comes out ascending after one workgroup-wide prefix sum.
// ---------------------------------------------------------------------------------------------
constexpr int kTopkThreads = 1024;

struct TopkParams {
  const float* scores;
  const int* cu_ctx;
  const int* cu_keep;
  const int* forced_first;   // or NULL
  const int* forced_last;    // or NULL
  int* keep_idx;
  int n_kv_heads;
};

// order-preserving key of a float (larger score -> larger key); -0 counts as +0
__device__ __forceinline__ uint32_t score_key(float s) {
  const uint32_t u = __float_as_uint(s + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// number of set bits of `mask` below this lane
__device__ __forceinline__ int lanes_below(unsigned long long mask) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32), __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0));
}

constexpr int kTopkBins = 4096;    // first digit: 12 bits (sign, exponent, 3 mantissa bits), then 10 + 10
constexpr int kTopkCand = 8192;    // keys of the first digit's bucket kept in LDS for the later passes

struct TopkShared {
  int hist[kTopkBins];
  uint32_t cand[kTopkCand];
  int red[kTopkThreads / 64];
  int digit, remaining, bucket, count;
};

// hist[0..nbins) holds digit counts; finds the digit d with  #(digits > d) < remaining <= #(digits >= d).
// Returns d; `remaining` becomes the rank inside that digit's bucket, `bucket` its size.
__device__ __forceinline__ uint32_t select_digit(TopkShared& sh, int nbins, int& remaining, int& bucket) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = nbins / kTopkThreads;            // 4 or 1
  int local[kTopkBins / kTopkThreads];
  int v = 0;
#pragma unroll
  for (int i = 0; i < kTopkBins / kTopkThreads; ++i) {
    local[i] = i < per ? sh.hist[tid * per + i] : 0;
    v += local[i];
  }
  int inc = v;                                     // inclusive suffix sum inside the wave
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_down(inc, off, 64);
    if (lane + off < 64) inc += o;
  }
  if (lane == 0) sh.red[wave] = inc;
  __syncthreads();
  int above = inc - v;
  for (int w = wave + 1; w < kTopkThreads / 64; ++w) above += sh.red[w];
#pragma unroll
  for (int i = kTopkBins / kTopkThreads - 1; i >= 0; --i) {
    if (i < per) {
      const int here = above + local[i];
      if (above < remaining && remaining <= here) {
        sh.digit = tid * per + i;
        sh.remaining = remaining - above;
        sh.bucket = local[i];
      }
      above = here;
    }
  }
  __syncthreads();
  const uint32_t d = static_cast<uint32_t>(sh.digit);
  remaining = sh.remaining;
  bucket = sh.bucket;
  __syncthreads();
  return d;
}

// Visit positions lo + start, lo + start + stride, ... below hi, eight loads in flight per thread:
// fn(t, valid, score) runs for every slot of a batch (valid = false past the end), so that code
// inside may use wave-wide ballots.
constexpr int kTopkBatch = 8;
template <class F>
__device__ __forceinline__ void for_scores(const float* s, int lo, int hi, int start, int stride, F fn) {
  for (int base = lo; base < hi; base += kTopkBatch * stride) {
    float v[kTopkBatch];
#pragma unroll
    for (int u = 0; u < kTopkBatch; ++u) {
      const int t = base + start + u * stride;
      v[u] = t < hi ? s[t] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kTopkBatch; ++u) {
      const int t = base + start + u * stride;
      fn(t, t < hi, v[u]);
    }
  }
}

__global__ __launch_bounds__(kTopkThreads) void topk_keep_kernel(TopkParams p) {
  __shared__ TopkShared sh;
  int* hist = sh.hist;
  const int b = blockIdx.y, h = blockIdx.x, tid = threadIdx.x;
  const int n = p.cu_ctx[b + 1] - p.cu_ctx[b];
  const int span = p.cu_keep[b + 1] - p.cu_keep[b];   // list stride of the sequence, as vc_draft_attn reads the lists
  const int k = min(span, n);
  if (k <= 0) return;
  const int f = min(p.forced_first ? p.forced_first[b] : 0, k);
  const int l = min(p.forced_last ? p.forced_last[b] : 0, k - f);
  const float* s = p.scores + static_cast<size_t>(p.cu_ctx[b]) * p.n_kv_heads + static_cast<size_t>(h) * n;
  int* out = p.keep_idx + static_cast<size_t>(p.cu_keep[b]) * p.n_kv_heads + static_cast<size_t>(h) * span;
  const int free_lo = f, free_hi = n - l;          // free positions: [free_lo, free_hi)
  const int want = k - f - l;                      // how many of them to keep
  // ---- threshold: the want-th largest key among the free positions (radix select, 12 + 10 + 10 bits)
  uint32_t prefix = 0;
  int remaining = want;
  const bool all_free = want >= free_hi - free_lo;
  if (want > 0 && !all_free) {
    for (int i = tid; i < kTopkBins; i += kTopkThreads) hist[i] = 0;
    if (tid == 0) sh.count = 0;
    __syncthreads();
    for_scores(s, free_lo, free_hi, tid, kTopkThreads, [&](int, bool valid, float sc) {
      if (valid) atomicAdd(&hist[score_key(sc) >> 20], 1);
    });
    __syncthreads();
    int bucket;
    prefix = select_digit(sh, kTopkBins, remaining, bucket) << 20;
    const bool in_lds = bucket <= kTopkCand;
    if (in_lds) {
      // gather the bucket's keys (order does not matter for the threshold)
      for_scores(s, free_lo, free_hi, tid, kTopkThreads, [&](int, bool valid, float sc) {
        const uint32_t key = score_key(sc);
        const bool hit = valid && (key & 0xFFF00000u) == prefix;
        const unsigned long long m = __ballot(hit);
        int start = 0;
        if (m != 0 && (tid & 63) == 0) start = atomicAdd(&sh.count, __popcll(m));
        start = __shfl(start, 0, 64);
        if (hit) sh.cand[start + lanes_below(m)] = key;
      });
      __syncthreads();
    }
    uint32_t mask = 0xFFF00000u;
    for (int shift = 10; shift >= 0; shift -= 10) {
      for (int i = tid; i < 1024; i += kTopkThreads) hist[i] = 0;
      __syncthreads();
      if (in_lds) {
        for (int i = tid; i < bucket; i += kTopkThreads) {
          const uint32_t key = sh.cand[i];
          if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 1023u], 1);
        }
      } else {
        for_scores(s, free_lo, free_hi, tid, kTopkThreads, [&](int, bool valid, float sc) {
          const uint32_t key = score_key(sc);
          if (valid && (key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 1023u], 1);
        });
      }
      __syncthreads();
      int dummy;
      prefix |= select_digit(sh, 1024, remaining, dummy) << shift;
      mask |= 1023u << shift;
    }
  }
  // `prefix` is the threshold key, `remaining` how many positions equal to it are kept
  const uint32_t thr = prefix;
  const int need_eq = (want > 0 && !all_free) ? remaining : 0;
  // ---- ordered compaction: wave w owns the contiguous range [wlo, whi) and walks it 64 positions
  // at a time (coalesced); ranks inside a step come from ballots, ranks across waves from LDS
  constexpr int NW = kTopkThreads / 64;
  const int lane = tid & 63, wave = tid >> 6;
  const int per_w = ((n + NW - 1) / NW + 63) / 64 * 64;
  const int wlo = min(wave * per_w, n), whi = min(wlo + per_w, n);
  const bool pick = want > 0 && !all_free;
  int cnt_eq = 0, cnt_sure = 0;
  // class of position t: kept for sure (forced, above the threshold, or everything is kept), or
  // equal to the threshold (kept while the quota lasts)
  auto classify = [&](int t, bool valid, float sc, bool& sure, bool& eq) {
    sure = false; eq = false;
    if (!valid) return;
    if (t < free_lo || t >= free_hi) sure = true;
    else if (want > 0 && all_free) sure = true;
    else if (pick) {
      const uint32_t key = score_key(sc);
      sure = key > thr;
      eq = key == thr;
    }
  };
  for_scores(s, wlo, whi, lane, 64, [&](int t, bool valid, float sc) {
    bool sure, eq;
    classify(t, valid, sc, sure, eq);
    cnt_sure += __popcll(__ballot(sure));
    cnt_eq += __popcll(__ballot(eq));
  });
  if (lane == 0) { hist[wave] = cnt_eq; hist[NW + wave] = cnt_sure; }
  __syncthreads();
  int eq_before = 0, pos = 0;
  for (int w = 0; w < wave; ++w) {
    const int e = hist[w];
    const int take = max(0, min(e, need_eq - eq_before));
    pos += hist[NW + w] + take;
    eq_before += e;
  }
  const int my_eq = max(0, min(cnt_eq, need_eq - eq_before));
  int eq_taken = 0;
  for_scores(s, wlo, whi, lane, 64, [&](int t, bool valid, float sc) {
    bool sure, eq;
    classify(t, valid, sc, sure, eq);
    const unsigned long long eq_mask = __ballot(eq);
    const bool keep = sure || (eq && eq_taken + lanes_below(eq_mask) < my_eq);
    const unsigned long long keep_mask = __ballot(keep);
    if (keep) out[pos + lanes_below(keep_mask)] = t;
    pos += __popcll(keep_mask);
    eq_taken += __popcll(eq_mask);
  });
}

static vc_status check_quant_call(vc_ctx* ctx, const int32_t* cu_ctx, const int32_t* cu_blk, int32_t n_seqs,
                                  int32_t n_kv_heads, int32_t bits, int32_t max_blk, const char* who) {
  VC_REQUIRE(ctx != nullptr, VC_ERR_INVALID_ARG, "%s: ctx is NULL", who);
  VC_REQUIRE(n_seqs >= 0 && n_kv_heads > 0 && max_blk >= 0, VC_ERR_INVALID_ARG, "%s: n_seqs %d n_kv_heads %d max_blk %d",
             who, n_seqs, n_kv_heads, max_blk);
  VC_REQUIRE(bits == 4 || bits == 2, VC_ERR_UNSUPPORTED, "%s: bits %d (block records are 4 or 2 bit)", who, bits);
  VC_REQUIRE(n_seqs <= 65535 && max_blk <= 4 * 65535, VC_ERR_UNSUPPORTED, "%s: grid too large", who);
  if (n_seqs > 0) VC_REQUIRE(cu_ctx && cu_blk, VC_ERR_INVALID_ARG, "%s: NULL cu array", who);
  return VC_OK;
}

}  // namespace vc

using namespace vc;

extern "C" vc_status vc_compress_quant(vc_ctx* ctx, const void* k, const void* v, const int32_t* cu_ctx,
                                       const int32_t* cu_blk, int32_t n_seqs, int32_t n_kv_heads, int32_t bits,
                                       int32_t max_blk, void* blocks, void* stream) {
  vc_status st = check_quant_call(ctx, cu_ctx, cu_blk, n_seqs, n_kv_heads, bits, max_blk, "vc_compress_quant");
  if (st != VC_OK) return st;
  if (n_seqs == 0 || max_blk == 0) return VC_OK;
  VC_REQUIRE(k && v && blocks, VC_ERR_INVALID_ARG, "vc_compress_quant: NULL pointer");
  VC_REQUIRE(aligned16(k) && aligned16(v) && aligned16(blocks), VC_ERR_INVALID_ARG,
             "vc_compress_quant: pointers must be 16-byte aligned");
  QuantParams p{};
  p.k = static_cast<const uint16_t*>(k);
  p.v = static_cast<const uint16_t*>(v);
  p.blocks_out = static_cast<uint8_t*>(blocks);
  p.cu_ctx = cu_ctx; p.cu_blk = cu_blk; p.n_kv_heads = n_kv_heads;
  dim3 grid(n_kv_heads, ceil_div(max_blk, 4), n_seqs);
  if (bits == 4) hipLaunchKernelGGL(compress_quant_kernel<4>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), p);
  else hipLaunchKernelGGL(compress_quant_kernel<2>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), p);
  VC_HIP(hipGetLastError());
  return VC_OK;
}

extern "C" vc_status vc_decompress_quant(vc_ctx* ctx, const void* blocks, const int32_t* cu_blk, const int32_t* cu_ctx,
                                         int32_t n_seqs, int32_t n_kv_heads, int32_t bits, int32_t max_blk, void* k_out,
                                         void* v_out, void* stream) {
  vc_status st = check_quant_call(ctx, cu_ctx, cu_blk, n_seqs, n_kv_heads, bits, max_blk, "vc_decompress_quant");
  if (st != VC_OK) return st;
  if (n_seqs == 0 || max_blk == 0) return VC_OK;
  VC_REQUIRE(k_out && v_out && blocks, VC_ERR_INVALID_ARG, "vc_decompress_quant: NULL pointer");
  VC_REQUIRE(aligned16(k_out) && aligned16(v_out) && aligned16(blocks), VC_ERR_INVALID_ARG,
             "vc_decompress_quant: pointers must be 16-byte aligned");
  QuantParams p{};
  p.blocks = static_cast<const uint8_t*>(blocks);
  p.k_out = static_cast<uint16_t*>(k_out);
  p.v_out = static_cast<uint16_t*>(v_out);
  p.cu_ctx = cu_ctx; p.cu_blk = cu_blk; p.n_kv_heads = n_kv_heads;
  dim3 grid(n_kv_heads, ceil_div(max_blk, 4), n_seqs);
  if (bits == 4) hipLaunchKernelGGL(decompress_quant_kernel<4>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), p);
  else hipLaunchKernelGGL(decompress_quant_kernel<2>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), p);
  VC_HIP(hipGetLastError());
  return VC_OK;
}

extern "C" vc_status vc_topk_keep(vc_ctx* ctx, const float* scores, const int32_t* cu_ctx, const int32_t* cu_keep,
                                  const int32_t* forced_first, const int32_t* forced_last, int32_t n_seqs,
                                  int32_t n_kv_heads, int32_t* keep_idx, void* stream) {
  VC_REQUIRE(ctx != nullptr, VC_ERR_INVALID_ARG, "vc_topk_keep: ctx is NULL");
  VC_REQUIRE(n_seqs >= 0 && n_kv_heads > 0, VC_ERR_INVALID_ARG, "vc_topk_keep: n_seqs %d n_kv_heads %d", n_seqs, n_kv_heads);
  if (n_seqs == 0) return VC_OK;
  VC_REQUIRE(scores && cu_ctx && cu_keep && keep_idx, VC_ERR_INVALID_ARG, "vc_topk_keep: NULL pointer");
  VC_REQUIRE(n_seqs <= 65535, VC_ERR_UNSUPPORTED, "vc_topk_keep: grid too large");
  TopkParams p{};
  p.scores = scores; p.cu_ctx = cu_ctx; p.cu_keep = cu_keep;
  p.forced_first = forced_first; p.forced_last = forced_last;
  p.keep_idx = keep_idx; p.n_kv_heads = n_kv_heads;
  hipLaunchKernelGGL(topk_keep_kernel, dim3(n_kv_heads, n_seqs), dim3(kTopkThreads), 0, static_cast<hipStream_t>(stream), p);
  VC_HIP(hipGetLastError());
  return VC_OK;
}
