// Draft attention: one query token per sequence over the compressed KV cache (paper section 4.1
// step 1; section 4.2.1: the step is bounded by HBM bandwidth, so every kernel here streams its
// source exactly once with 128-bit loads and does the arithmetic in registers).
//
// Two sources (retained bf16 rows, int4/int2 block records) are each cut into splits over their
// tokens; one workgroup turns one split of one (sequence, KV head) into a partial (m, l, O) for the
// g query heads of that KV head (GQA packing: K/V are read once for all of them).  The short bf16
// tail is one more partial, made by extra workgroups of the same launch, and a merge kernel
// combines the partials of all sources.
#include <atomic>

#include "attn_common.h"
#include "common.h"

namespace vc {

// Flat launch (at most 64 sequences): workgroup x of the launch is split x of the list of all the
// splits that exist, sequence after sequence.  Every wave finds its sequence by itself - lane i holds
// the split count of sequence i, a prefix sum over the lanes, one ballot - so a ragged batch launches
// no workgroup per (sequence, split of the longest sequence) that finds nothing to do.  `cu` holds
// the n_seqs + 1 prefix sums of the units (rows or records), `per` the units per split.  Returns
// false when x is beyond the last split, with `b` = how far beyond (0 for the first such x).
__device__ __forceinline__ bool flat_split(const int* cu, int n_seqs, int per, int x, int& b, int& sp) {
  const int lane = threadIdx.x & 63;
  int cnt = 0;
  if (lane < n_seqs) {
    const int s = cu[lane], e = cu[lane + 1];
    cnt = e > s ? (e - s + per - 1) / per : 0;
  }
  int scan = cnt;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(scan, d);
    if (lane >= d) scan += t;
  }
  const unsigned long long hit = __ballot(scan > x);
  if (hit == 0ull) {
    b = x - __builtin_amdgcn_readfirstlane(__shfl(scan, 63));
    return false;
  }
  const int l = __ffsll(hit) - 1;
  b = __builtin_amdgcn_readfirstlane(l);
  sp = __builtin_amdgcn_readfirstlane(x - (__shfl(scan, l) - __shfl(cnt, l)));
  return true;
}

struct DraftMergeParams {
  const float* ws;
  const uint16_t* q;
  uint16_t* out;
  float* lse;
  const int* cu_a;      // bf16 source: cu_keep (gather) or cu_ctx (contiguous), or NULL
  const int* cu_blk;    // or NULL
  const uint16_t* tail_k;  // or NULL
  const uint16_t* tail_v;
  const int* cu_tail;
  int n_q_heads, n_kv_heads, g, ns;
  int split_a, s1, bps;
  int tail_slot;        // >= 0: the tail's partial sits in this slot (tail_partial, run by workgroups of the split launch)
  float scale_log2e;
};

// The merge of one (sequence, query head) by 128 threads (defined with the merge kernels below).  The split
// kernels call it too: in a small launch the workgroup that delivers the last partial of a (sequence, KV
// head) finishes its heads on the spot (see finish_if_last).
template <bool COHERENT, int CHUNK>
__device__ __forceinline__ void merge_head(const DraftMergeParams& p, int b, int h, int d, float* probs);

// Fused finish of small launches.  Every workgroup of a split kernel has written its partials through to
// device-coherent memory (the reader may sit on another XCD, behind another L2) and waited for those stores;
// one thread then counts the workgroup on the counter of its (sequence, KV head).  The workgroup that
// brings the count to `expected` finds every partial of the pair complete: it puts the counter back to
// zero for the next call and merges the pair's g heads, 128 threads each, reading the
// partials with device-coherent loads, all of a head's at once.  No fence: a release fence would write the
// whole L2 back once per workgroup.  `lds` is the workgroup's ring, idle by now.
struct DraftFuse {
  unsigned int* counters;   // one per (sequence, KV head) of the launch, zero between calls; NULL: the merge is a launch of its own
  int expected_mul;         // workgroups per split (passes of the record kernel)
};
__device__ __forceinline__ void st_partial(float* p, float v, bool coherent) {
  if (coherent) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = v;
}
__device__ __forceinline__ void finish_if_last(const DraftFuse& f, const DraftMergeParams& mp, int b, int kvh, int nsplits,
                                               char* lds) {
  __shared__ int last;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();                              // every thread's partial stores have arrived; the ring is no longer read
  if (threadIdx.x == 0) {
    unsigned int* c = f.counters + (static_cast<size_t>(b) * mp.n_kv_heads + kvh) * vc_ctx::kDraftCounterStride;
    const unsigned int expected = static_cast<unsigned int>(nsplits) * f.expected_mul;
    last = expected <= 1u || __hip_atomic_fetch_add(c, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == expected - 1u;
    if (last && expected > 1u) __hip_atomic_store(c, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (!last) return;
  float* probs = reinterpret_cast<float*>(lds) + (threadIdx.x >> 6) * 64;   // a strip of 64 floats per wave
  const int per_pass = blockDim.x >> 7;          // heads merged at a time
  for (int hp = 0; hp < mp.g; hp += per_pass) {
    const int hl = hp + (threadIdx.x >> 7);
    if (hl < mp.g) merge_head<true, 16>(mp, b, kvh * mp.g + hl, threadIdx.x & 127, probs);
  }
}

// The bf16 tail as one more partial.  In launches that keep the merge as a launch of its own, the split
// kernel carries one extra workgroup per (sequence, KV head) that attends the pair's g query heads over the
// tail tokens and writes (m, l, O) into slot `tail_slot`; the merge then only combines partials.  The tail
// work runs beside the splits instead of behind them (a merge that also scores the tail takes 6 us, one that
// does not 4 us).  One wave per head at a time: two lanes per token for the scores (64 channels each, packed
// bf16 dot products against the query row), maximum and exponentials inside the wave, probabilities through
// the wave's own strip of LDS, and every lane accumulates output channels 2*lane and 2*lane + 1.
__device__ __forceinline__ float dot8_bf16(const uint4& a, const uint4& b, float c);
struct TailLane {          // what a lane needs to address the tail of (sequence b, KV head kvh)
  const uint16_t* kcol;    // its 64 channels of the first tail key row
  const uint16_t* vcol;    // its two channels of the first tail value row
  size_t row_stride;
  float* probs;            // the wave's strip of 32 floats in LDS
  int nt, half, tk;
};
struct TailChunk {         // one chunk of 32 tokens as it comes from memory
  uint4 k[8];
  uint32_t v[32];
};
__device__ __forceinline__ TailLane tail_lane(const DraftMergeParams& p, int b, int kvh, float* probs_lds) {
  TailLane g;
  const int lane = threadIdx.x & 63;
  g.half = lane & 1;
  g.tk = lane >> 1;
  g.probs = probs_lds + (threadIdx.x >> 6) * 32;
  const int t0 = p.cu_tail[b];
  g.nt = p.cu_tail[b + 1] - t0;
  g.row_stride = static_cast<size_t>(p.n_kv_heads) * kHeadDim;
  g.kcol = p.tail_k + static_cast<size_t>(t0) * g.row_stride + static_cast<size_t>(kvh) * kHeadDim + 64 * g.half;
  g.vcol = p.tail_v + static_cast<size_t>(t0) * g.row_stride + static_cast<size_t>(kvh) * kHeadDim + 2 * lane;
  return g;
}
__device__ __forceinline__ void tail_request_q(const DraftMergeParams& p, const TailLane& g, int b, int h, uint4 (&q)[8]) {
  const uint16_t* qp = p.q + (static_cast<size_t>(b) * p.n_q_heads + h) * kHeadDim + 64 * g.half;
#pragma unroll
  for (int i = 0; i < 8; ++i) q[i] = *reinterpret_cast<const uint4*>(qp + 8 * i);
}
// everything a chunk needs is requested before anything of it is consumed: one trip to memory per chunk
// (the tails of a speculation horizon are one chunk).  Only called with tokens left (c0 < nt).
__device__ __forceinline__ void tail_request(const TailLane& g, int c0, TailChunk& c) {
  const int cn = min(32, g.nt - c0);
  const uint16_t* kr = g.kcol + static_cast<size_t>(c0 + min(g.tk, cn - 1)) * g.row_stride;
#pragma unroll
  for (int i = 0; i < 8; ++i) c.k[i] = *reinterpret_cast<const uint4*>(kr + 8 * i);
#pragma unroll
  for (int i = 0; i < 32; ++i)
    c.v[i] = *reinterpret_cast<const uint32_t*>(g.vcol + static_cast<size_t>(c0 + min(i, cn - 1)) * g.row_stride);
}
struct TailAcc { float mt, a0, a1, tl; };
__device__ __forceinline__ void tail_consume(const DraftMergeParams& p, const TailLane& g, int c0, const uint4 (&q)[8],
                                             const TailChunk& c, TailAcc& r) {
  const int cn = min(32, g.nt - c0);
  float a = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) a = dot8_bf16(c.k[i], q[i], a);
  a += __shfl_xor(a, 1, 64);
  const float sc = g.tk < cn ? a * p.scale_log2e : -INFINITY;
  const float mn = fmaxf(r.mt, wave_max(sc));
  const float alpha = exp2_diff(r.mt, mn);
  // LDS operations of one wave are carried out in order: the reads below see this write, and the next
  // chunk's write comes after this chunk's reads - the wave is alone on its strip, no barrier
  if (g.half == 0) g.probs[g.tk] = exp2_diff(sc, mn);
  __builtin_amdgcn_wave_barrier();
  r.a0 *= alpha;
  r.a1 *= alpha;
  r.tl *= alpha;
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    const float pv = g.probs[i];               // 0 beyond the chunk's last token
    r.a0 = fmaf(pv, bf16_lo(c.v[i]), r.a0);
    r.a1 = fmaf(pv, bf16_hi(c.v[i]), r.a1);
    r.tl += pv;
  }
  r.mt = mn;
  __builtin_amdgcn_wave_barrier();
}
// chunks from c0 on, then the partial of head h
__device__ __forceinline__ void tail_finish(const DraftMergeParams& p, const TailLane& g, int b, int h, const uint4 (&q)[8],
                                            int c0, TailAcc r) {
  for (; c0 < g.nt; c0 += 32) {
    TailChunk c;
    tail_request(g, c0, c);
    tail_consume(p, g, c0, q, c, r);
  }
  const int lane = threadIdx.x & 63;
  float* dst = const_cast<float*>(p.ws) + ((static_cast<size_t>(b) * p.n_q_heads + h) * p.ns + p.tail_slot) * kPartialFloats;
  *reinterpret_cast<float2*>(dst + 2 + 2 * lane) = make_float2(r.a0, r.a1);
  if (lane == 0) {
    dst[0] = r.mt;
    dst[1] = r.tl;
  }
}
// heads hl0, hl0 + NWAVES, ... of the KV head, one after the other
template <int NWAVES>
__device__ __forceinline__ void tail_heads(const DraftMergeParams& p, const TailLane& g, int b, int kvh, int hl0) {
  for (int hl = hl0; hl < p.g; hl += NWAVES) {
    uint4 q[8];
    if (g.nt > 0) tail_request_q(p, g, b, kvh * p.g + hl, q);
    tail_finish(p, g, b, kvh * p.g + hl, q, 0, TailAcc{-INFINITY, 0.f, 0.f, 0.f});
  }
}
template <int NWAVES>
__device__ __forceinline__ void tail_partial(const DraftMergeParams& p, int b, int kvh, char* lds) {
  const TailLane g = tail_lane(p, b, kvh, reinterpret_cast<float*>(lds));
  tail_heads<NWAVES>(p, g, b, kvh, threadIdx.x >> 6);
}

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
  int n_seqs, flat;     // flat: see flat_split
  int tail;             // the launch carries the tail's workgroups (tail_partial), behind the splits' in launch order
  float scale_log2e;
};

// Formulation (bf16 MFMA 16x16x32, fp32 accumulation), per step of 32 tokens of one wave:
//   S^T[token][head]  = K[token][:] . Q[head][:]          A = K rows from LDS, B = Q^T (registers)
//   O^T[d][head]     += V^T[d][token] * P[token][head]    A = V^T through the transposing LDS read
// The columns are the (up to 16) query heads of the KV head, so GQA packing is the tile's N
// dimension; the D layout of the first product hands every lane 4 tokens of one head per 16-token
// tile, and the 8 tokens a lane gets from the two tiles of a step are taken as its k-slots of the
// second product (token 16*(e/4) + 4*j + e%4 for slot e of lane block j) - the transposing reads
// fetch V in that same order, so probabilities never cross lanes.
//
// Rows travel HBM -> LDS directly: every wave owns a ring of two 32-token stages (K rows, then V
// rows, 256 bytes each) and requests the stage two steps ahead as soon as it has read the current
// one, so there is no barrier and loads stay in flight while the wave computes.  The 16-byte chunk
// c of row r is stored at chunk position c ^ (r & 15): the 16 rows an operand read touches then
// sit in 16 different bank groups.  Kept positions are streamed the same way (a ring of four
// 32-entry index stages per wave), so every load of the loop is accounted for in one wait counter.
constexpr float kLazyMargin = 4.f;  // the running maximum may lag the true one by this much (log2 units)
constexpr int kRowsIdxStage = 256;                              // 64 lanes x 4 bytes (one step's entries, mirrored)
constexpr int rows_wave_lds(int step) { return 2 * step * 512 + 4 * kRowsIdxStage; }   // two stages + index ring
constexpr int rows_lds(int step, int nw) { return nw * rows_wave_lds(step); }

__device__ __forceinline__ float4v mfma16_bf16(bf16x8v a, bf16x8v b, float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ uint32_t rows_lds_off(int row, int chunk) { return row * 256 + ((chunk ^ (row & 15)) << 4); }

__device__ __forceinline__ float4v mfma16_bf16_k16(short4v a, short4v b, float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0);
}

// kRowsStep: tokens per step (32: the second product is one 16x16x32 per output tile; 16: one
// 16x16x16, whose k-slots are exactly the 4 tokens a lane holds); NW: waves per workgroup.
// FUSED: the instantiation for small launches, which carries the merge (finish_if_last); the plain one
// stays free of its registers.
template <bool GATHER, int kRowsStep, int NW, bool FUSED>
__global__ __launch_bounds__(NW * 64, 4 / NW) void draft_bf16_kernel(DraftBf16Params p, DraftMergeParams mp, DraftFuse fz) {
  constexpr int kRowsStage = kRowsStep * 512;                   // K rows then V rows
  constexpr int kRowsWaveLds = rows_wave_lds(kRowsStep);
  constexpr int NT = kRowsStep / 16;                            // 16-token score tiles per step
  constexpr int NLD = kRowsStep / 4;                            // wave loads per matrix per step
  extern __shared__ __attribute__((aligned(1024))) char ring[];
  int b, kvh, sp;
  if (p.flat) {
    kvh = blockIdx.x % p.n_kv_heads;   // heads vary fastest: the workgroups beyond the last split come last
    if (!flat_split(GATHER ? p.cu_keep : p.cu_rows, p.n_seqs, p.split_tok, blockIdx.x / p.n_kv_heads, b, sp)) {
      // the first n_seqs workgroups (per head) beyond the last split take the tails
      if constexpr (!FUSED) {
        if (p.tail && b < p.n_seqs) tail_partial<NW>(mp, b, kvh, ring);
      }
      return;
    }
  } else {
    b = blockIdx.z; kvh = blockIdx.y; sp = blockIdx.x;
    if constexpr (!FUSED) {
      if (b >= p.n_seqs) {
        // the slices behind the last sequence's: one workgroup per (sequence, KV head) for the tails
        b = (b - p.n_seqs) * static_cast<int>(gridDim.x) + sp;
        if (p.tail && b < p.n_seqs) tail_partial<NW>(mp, b, kvh, ring);
        return;
      }
    }
  }
  const int row0 = p.cu_rows[b];
  const int count = GATHER ? (p.cu_keep[b + 1] - p.cu_keep[b]) : (p.cu_rows[b + 1] - row0);
  const int start = sp * p.split_tok;
  constexpr bool fused = FUSED;
  if (start >= count) {
    // fused: the first workgroup of a list without rows still has the list's heads to finish (tail only, or zeros)
    if constexpr (FUSED) {
      if (sp == 0) finish_if_last(fz, mp, b, kvh, 0, ring);
    }
    return;
  }
  const int end = min(count, start + p.split_tok);
  const int* idx = GATHER ? p.keep_idx + (static_cast<size_t>(p.cu_keep[b]) * p.n_kv_heads + static_cast<size_t>(kvh) * count)
                          : nullptr;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, j = lane >> 4;     // n: head column / operand row, j: k-block and D row block
  const int hn = min(n, p.g - 1);             // columns beyond the group replicate its last head (never stored)

  // query as B operand: k-step ks covers channels 32ks .. 32ks+31, this lane holds 32ks + 8j .. +7
  bf16x8v qb[4];
  {
    const uint16_t* qp = p.q + (static_cast<size_t>(b) * p.n_q_heads + kvh * p.g + hn) * kHeadDim + 8 * j;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const uint4 raw = *reinterpret_cast<const uint4*>(qp + 32 * ks);
      qb[ks] = __builtin_bit_cast(bf16x8v, raw);
    }
  }

  // the query loads must have landed before the ring starts (a wait for them inside the loop
  // would also drain the rows in flight).  (Pinning them behind the ring's first requests instead, so that
  // query and first rows are one trip to memory, measured 1.6 us slower per call at 16 x 6554 kept rows; the
  // record kernel, below, gains a little from that order.)
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) asm volatile("" : "+v"(qb[ks]));

  const size_t row_stride = static_cast<size_t>(p.n_kv_heads) * kHeadDim;
  const uint16_t* kbase = p.pk + static_cast<size_t>(row0) * row_stride + static_cast<size_t>(kvh) * kHeadDim;
  const uint16_t* vbase = p.pv + static_cast<size_t>(row0) * row_stride + static_cast<size_t>(kvh) * kHeadDim;

  // steps of this wave: step `it` covers tokens tok0(it) .. tok0(it) + 31 of the list
  auto tok0 = [&](int it) { return start + kRowsStep * (wave + NW * it); };
  const int nst = end > start + kRowsStep * wave ? (end - start - kRowsStep * wave + NW * kRowsStep - 1) / (NW * kRowsStep) : 0;
  const uint32_t wave_lds = lds_address(ring) + wave * kRowsWaveLds;
  const uint32_t idx_lds = wave_lds + 2 * kRowsStage;
  const int ts = lane >> 4, c = lane & 15;    // direct loads: 16 lanes per row, lane c brings one 16-byte chunk

  auto request_idx = [&](int it) {            // kept positions of step `it` -> index stage it % 4 (one load)
    if (it > nst) return;                     // (step nst is still requested: it keeps the wait counts below uniform)
    if constexpr (GATHER) {
      const int t = it < nst ? min(tok0(it) + (lane & (kRowsStep - 1)), end - 1) : end - 1;
      load_to_lds_b32(idx + t, idx_lds + (it & 3) * kRowsIdxStage);
    }
  };
  auto request_rows = [&](int it) {           // rows of step `it` -> stage it % 2 (16 loads); nothing past the last step
    const uint32_t stage = wave_lds + (it & 1) * kRowsStage;
    if (it < nst) {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int r = 4 * i + ts;             // row of the stage
        int row;
        if constexpr (GATHER) {
          row = *reinterpret_cast<const __attribute__((address_space(3))) int*>(
              static_cast<size_t>(idx_lds + (it & 3) * kRowsIdxStage + 4 * r));
        } else {
          row = min(tok0(it) + r, end - 1);
        }
        const size_t off = static_cast<size_t>(row) * row_stride + 8 * (c ^ (r & 15));
        load_to_lds(kbase + off, stage + i * 1024);
        load_to_lds(vbase + off, stage + kRowsStep * 256 + i * 1024);
      }
    }
  };

  // LDS read offsets of this lane inside a stage
  uint32_t kaddr[NT][4];                      // K operand: row 16T + n, chunk 4ks + j
#pragma unroll
  for (int T = 0; T < NT; ++T)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) kaddr[T][ks] = rows_lds_off(16 * T + n, 4 * ks + j);
  // transposing read: lane L of block j addresses row 4j + L/4 (+16), 8 bytes at channel 16dt + 4(L%4)
  uint32_t vaddr[8][NT];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt)
#pragma unroll
    for (int h2 = 0; h2 < NT; ++h2)
      vaddr[dt][h2] = kRowsStep * 256 + rows_lds_off(16 * h2 + 4 * j + (n >> 2), 2 * dt + ((n & 3) >> 1)) + 8 * (n & 1);

  float m_run = kNoKeyYet;                    // running maximum of this column's head (log2 domain)
  float l_part = 0.f;                         // this lane's share of sum 2^(s - m_run)
  float4v oacc[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) oacc[dt] = float4v{0.f, 0.f, 0.f, 0.f};

  // prologue, in the issue order the loop's wait counts assume:
  // idx(0) idx(1) | rows(0) idx(2) | rows(1)
  constexpr int kYounger = 2 * NLD + (GATHER ? 1 : 0);   // loads issued after the rows of a step, before its use
  request_idx(0);
  request_idx(1);
  if constexpr (GATHER) wait_vm<1>();
  request_rows(0);
  request_idx(2);
  if constexpr (GATHER) wait_vm<kYounger>();
  request_rows(1);

  for (int it = 0; it < nst; ++it) {
    // rows(it) have landed once only the younger requests are outstanding: rows(it + 1) and idx(it + 2), which
    // exist together or (in the wave's last step) not at all - no loads are issued just to keep the count, so
    // the last step ends without a trip to memory to wait for
    if (it + 1 < nst) wait_vm<kYounger>();
    else wait_vm<0>();
    const uint32_t stage = wave_lds + (it & 1) * kRowsStage;
    // ---------------- scores ----------------
    float4v sacc[NT];
#pragma unroll
    for (int T = 0; T < NT; ++T) {
      sacc[T] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const bf16x8v a = __builtin_bit_cast(bf16x8v, lds_load_u32x4(stage + kaddr[T][ks]));
        sacc[T] = mfma16_bf16(a, qb[ks], sacc[T]);
      }
    }
    // register i of tile T is token 16T + 4j + i of the step, for head column n
    const int tbase = tok0(it) + 4 * j;
    float smax = -INFINITY;
#pragma unroll
    for (int T = 0; T < NT; ++T)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool valid = tbase + 16 * T + i < end;
        sacc[T][i] = valid ? sacc[T][i] * p.scale_log2e : -INFINITY;
        smax = fmaxf(smax, sacc[T][i]);
      }
    if (__any(smax > m_run + kLazyMargin)) {
      float mx = fmaxf(smax, __shfl_xor(smax, 16, 64));   // the four row blocks of this head
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mn = fmaxf(m_run, mx);
      const float alpha = __builtin_amdgcn_exp2f(m_run - mn);
      l_part *= alpha;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) oacc[dt] *= alpha;
      m_run = mn;
    }
    float pe[4 * NT];
#pragma unroll
    for (int e = 0; e < 4 * NT; ++e) {
      pe[e] = __builtin_amdgcn_exp2f(sacc[e >> 2][e & 3] - m_run);
      l_part += pe[e];
    }
    // ---------------- output ----------------
    if constexpr (NT == 2) {
      bf16x8v pb;
#pragma unroll
      for (int e = 0; e < 8; ++e) pb[e] = (__bf16)pe[e];
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_short4v*>(static_cast<size_t>(stage + vaddr[dt][0])));
        const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_short4v*>(static_cast<size_t>(stage + vaddr[dt][1])));
        const bf16x8v av = __builtin_bit_cast(bf16x8v, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        oacc[dt] = mfma16_bf16(av, pb, oacc[dt]);
      }
    } else {
      typedef __bf16 bf16x4v __attribute__((ext_vector_type(4)));
      bf16x4v pb4;
#pragma unroll
      for (int e = 0; e < 4; ++e) pb4[e] = (__bf16)pe[e];
      const short4v pbs = __builtin_bit_cast(short4v, pb4);
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        const short4v av = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_short4v*>(static_cast<size_t>(stage + vaddr[dt][0])));
        oacc[dt] = mfma16_bf16_k16(av, pbs, oacc[dt]);
      }
    }
    // the stage is free once those reads have returned: request the rows two steps ahead
    wait_lds_reads();
    request_idx(it + 3);
    if (it + 2 < nst) {
      if constexpr (GATHER) wait_vm<kYounger>();   // idx(it + 2) has landed (younger: rows(it + 1), idx(it + 3))
      request_rows(it + 2);
    }
  }
  wait_vm<0>();                               // nothing may land in the ring any more: it is reused below

  // ---------------- end of split: wave state -> LDS -> merged partial ----------------
  float* st = reinterpret_cast<float*>(ring);                 // [wave][head][kPartialFloats], wave-private part first
  constexpr int kWaveFloats = kRowsWaveLds / 4;
  {
    float lsum = l_part + __shfl_xor(l_part, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    if (n < p.g) {
      float* mine = st + wave * kWaveFloats + n * kPartialFloats;
      if (j == 0) {
        mine[0] = m_run;
        mine[1] = lsum;
      }
#pragma unroll
      for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int i = 0; i < 4; ++i) mine[2 + 16 * dt + 4 * j + i] = oacc[dt][i];
    }
  }
  __syncthreads();
  const int slot = p.slot0 + sp;
  for (int i = threadIdx.x; i < p.g * kHeadDim; i += NW * 64) {
    const int hq = i >> 7, d = i & 127;
    const float* s0 = st + hq * kPartialFloats;
    float mm = s0[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) mm = fmaxf(mm, s0[w * kWaveFloats]);
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float a = __builtin_amdgcn_exp2f(s0[w * kWaveFloats] - mm);
      acc = fmaf(a, s0[w * kWaveFloats + 2 + d], acc);
      lsum = fmaf(a, s0[w * kWaveFloats + 1], lsum);
    }
    float* dst = p.ws + ((static_cast<size_t>(b) * p.n_q_heads + kvh * p.g + hq) * p.ns + slot) * kPartialFloats;
    st_partial(dst + 2 + d, acc, fused);
    if (d == 0) {
      st_partial(dst, mm, fused);
      st_partial(dst + 1, lsum, fused);
    }
  }
  if constexpr (FUSED) finish_if_last(fz, mp, b, kvh, ceil_div_dev(count, p.split_tok), ring);
}

// --------------------------------------------------------------------------------------------
// int4 / int2 block records, dequantisation fused into fp16 MFMA tiles
// --------------------------------------------------------------------------------------------
// Everything is laid out so that the matrix core's own register layouts do the data movement and
// the loop needs neither LDS nor cross-lane shuffles (MFMA 16x16x32 f16, D = A*B + C):
//
//   S^T[token][col] = K[token][:] . Q'[col][:]     A = key codes of 16 tokens (exact small integers
//                                                  in fp16), B = the query with the block's key
//                                                  scale folded in; col = (slot, query head)
//   the D layout gives every lane 4 tokens of one column, which is exactly the B layout of
//   O^T[d][col]    += V^T[d][token] * P'[token][col]   A = value codes, B = probabilities times the
//                                                  value scale of channel group `slot`
//   The four column slots carry the four (two for int2) value channel groups, so one pass of the
//   probabilities serves all groups and each output tile picks the slot of its own group.
//   The zero points never touch the codes: the key zero is one extra product whose A operand is
//   the zero points themselves in every row (sum_d zK[d]*q[d], the same for every token of the
//   block), the value zero a product of a constant A operand with p[t]*zV[t].
//   Codes reach the matrix core as the fp16 subnormals 2^-24 * f * code that their masked bit fields
//   already are, one and per two codes (f is 1, 4, 16 or 64 depending on where the field sits in
//   its byte).  1/f is folded into the operand on the other side of the product once, outside the
//   loop; 2^24 is applied to the fp32 results (inside the multiply-add that forms the exponent for
//   the scores, once per split for the outputs).
struct DraftQuantParams {
  const uint16_t* q;
  const uint8_t* blocks;
  const int* cu_blk;
  float* ws;
  int n_q_heads, n_kv_heads, g, npass;
  int bps, slot0, ns;
  int n_seqs, flat;   // flat: see flat_split
  int tail;           // the launch carries the tail's workgroups, as in DraftBf16Params
  float scale_log2e;
};

__device__ __forceinline__ half8v as_half8(const uint32_t (&u)[4]) {
  half8v r;
  __builtin_memcpy(&r, u, 16);
  return r;
}
__device__ __forceinline__ half2v as_half2(uint32_t u) { return __builtin_bit_cast(half2v, u); }
__device__ __forceinline__ uint32_t as_u32(half2v h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ uint32_t pack_half2(float a, float b) {
  half2v h;
  h[0] = (_Float16)a;
  h[1] = (_Float16)b;
  return as_u32(h);
}

// A code field masked out of its word IS an fp16 number: a subnormal (or, from mantissa bit 10 on, nothing
// we use) whose value is 2^-24 * f * code, f = 2^(position of the field in its 16-bit half).  The matrix
// core takes fp16 subnormals exactly (checked on the device: sums of products of such operands come out to
// the last bit), so one v_and_b32 per two codes is the whole dequantisation: f is folded into the operand on
// the other side of the product outside the loop, 2^24 into the fp32 results.
constexpr float kCodeScale = 16777216.f;   // 2^24

// Eight 4-bit codes of one word (element e at bit 16*(e&1) + 4*(e>>1)) -> four fp16 pairs in element
// order holding 2^-24 * code (pairs 0, 2) or 2^-24 * 16 * code (pairs 1, 3).
__device__ __forceinline__ void unpack_i4(uint32_t x, uint32_t (&out)[4]) {
  const uint32_t y = x >> 8;
  out[0] = x & 0x000F000Fu;
  out[1] = x & 0x00F000F0u;
  out[2] = y & 0x000F000Fu;
  out[3] = y & 0x00F000F0u;
}
// Sixteen 2-bit codes (element e at bit 16*(e&1) + 2*(e>>1)) -> eight fp16 pairs holding
// 2^-24 * 4^(r&3) * code for pair r.
__device__ __forceinline__ void unpack_i2(uint32_t x, uint32_t (&out)[8]) {
  const uint32_t y = x >> 8;
  out[0] = x & 0x00030003u;
  out[1] = x & 0x000C000Cu;
  out[2] = x & 0x00300030u;
  out[3] = x & 0x00C000C0u;
  out[4] = y & 0x00030003u;
  out[5] = y & 0x000C000Cu;
  out[6] = y & 0x00300030u;
  out[7] = y & 0x00C000C0u;
}

__device__ __forceinline__ float4v mfma16(const uint32_t (&a)[4], const uint32_t (&b)[4], float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(a), as_half8(b), c, 0, 0, 0);
}

__device__ __forceinline__ void u4_to_arr(const uint4& v, uint32_t (&a)[4]) {
  a[0] = v.x; a[1] = v.y; a[2] = v.z; a[3] = v.w;
}


// Records travel HBM -> LDS directly, into a private ring of kQuantSlots records per wave, two
// records ahead of the one being consumed, so that every wave keeps loads in flight while it
// computes (no barrier: a wave only ever reads what it loaded itself).  The LDS image of a record
// is the record itself except that the 16-byte chunks of the key codes are permuted into the order
// the lanes read them (a direct load writes lane i's chunk at position i, so the permutation is a
// choice of source address and costs nothing):
//   int4: chunk 64*T + lane           <- key bytes of token 8*(n>>2) + 4*T + (n&3), chunk j
//   int2: chunk 32*T + 2*n + m        <- key bytes of token 16*(n>>2) + 4*T + (n&3), chunk m
//         (lane (n, j) then reads the 8 bytes at 512*T + 32*n + 8*j: a linear, conflict-free sweep)
// (three slots at two workgroups per CU measured 2-3 % slower than two slots at three; four slots: int4 203.5 ->
// 206 us and int2 113 -> 125 us at 16 x 65536 tokens, and no gain for one sequence of 131072 tokens at one
// workgroup per CU either - 2048 calls 69 -> 74 ms - so the bytes in flight are not what holds small launches back)
constexpr int kQuantSlots = 2;
constexpr int kQuantRingBytes = 4 * kQuantSlots * kRecordBytes;   // per workgroup of 4 waves

// HPW = query heads per pass (the 16 MFMA columns are HPW heads x 16/HPW slots).  GQA ratios up to 4
// use 4 heads x 4 slots, one slot per value channel group (int2 has two groups: slots repeat);
// ratios of 5 to 8 use 8 heads x 2 slots so that the records are still read once for all heads -
// for int4 a slot then carries two channel groups and scales its probabilities once per group.
// FUSED: as for the row kernel; that instantiation runs two workgroups per CU (it is only used for launches
// that do not fill the GPU anyway).
template <int BITS, int HPW, bool FUSED>
__global__ __launch_bounds__(256, FUSED ? 2 : 3) void draft_quant_kernel(DraftQuantParams p, DraftMergeParams mp, DraftFuse fz) {
  constexpr int TB = (BITS == 4) ? 32 : 64;   // tokens per block record
  constexpr int NT = TB / 16;                 // 16-token score tiles per record
  constexpr int NKS = TB / 32;                // 32-token k-steps of the output product per record
  constexpr int NSLOT = 16 / HPW;             // column slots per head
  constexpr int NG = 128 / TB;                // value channel groups (4 for int4, 2 for int2)
  constexpr int GPS = NG > NSLOT ? NG / NSLOT : 1;   // channel groups a slot carries
  constexpr int TPG = 8 / NG;                 // 16-channel output tiles per channel group
  extern __shared__ __attribute__((aligned(1024))) char ring[];
  int b, sp, yy;
  if (p.flat) {
    // heads vary fastest, so the workgroups beyond the last split are the last ones dispatched
    const int ny = p.n_kv_heads * p.npass;
    yy = blockIdx.x % ny;
    if (!flat_split(p.cu_blk, p.n_seqs, p.bps, blockIdx.x / ny, b, sp)) {
      if constexpr (!FUSED) {
        if (p.tail && b < p.n_seqs && yy % p.npass == 0) tail_partial<4>(mp, b, yy / p.npass, ring);
      }
      return;
    }
  } else {
    b = blockIdx.z; sp = blockIdx.x; yy = blockIdx.y;
    if constexpr (!FUSED) {
      if (b >= p.n_seqs) {
        b = (b - p.n_seqs) * static_cast<int>(gridDim.x) + sp;
        if (p.tail && b < p.n_seqs && yy % p.npass == 0) tail_partial<4>(mp, b, yy / p.npass, ring);
        return;
      }
    }
  }
  const int kvh = yy / p.npass, pass = yy % p.npass;
  const int nb = p.cu_blk[b + 1] - p.cu_blk[b];
  const int blk0 = sp * p.bps;
  constexpr bool fused = FUSED;
  if (blk0 >= nb) {
    // fused: the first workgroup of a list without records still has the list's heads to finish
    if constexpr (FUSED) {
      if (sp == 0 && pass == 0) finish_if_last(fz, mp, b, kvh, 0, ring);
    }
    return;
  }
  const int blk1 = min(nb, blk0 + p.bps);
  const uint8_t* rec_base =
      p.blocks + (static_cast<size_t>(p.cu_blk[b]) * p.n_kv_heads + static_cast<size_t>(kvh) * nb) * kRecordBytes;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, j = lane >> 4;     // n: column / operand row, j: k-block and D row block
  const int slot = n / HPW, hq = n % HPW;
  // value channel group gi of this column's slot; the slot that carries group G, and G's index in it
  auto group_of = [&](int gi) { return NG >= NSLOT ? slot * GPS + gi : slot % NG; };
  auto slot_of = [](int G) { return NG >= NSLOT ? G / GPS : G; };
  auto index_in_slot = [](int G) { return NG >= NSLOT ? G % GPS : 0; };

  // ---- the ring: source offsets of this lane's five 16-byte chunks, and the request itself ----
  uint32_t src_key[2];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    if constexpr (BITS == 4) {
      src_key[c] = (8 * (n >> 2) + 4 * c + (n & 3)) * 64 + 16 * j;
    } else {
      const int T = 2 * c + (lane >> 5), nn = (lane & 31) >> 1, mm = lane & 1;
      src_key[c] = (16 * (nn >> 2) + 4 * T + (nn & 3)) * 32 + 16 * mm;
    }
  }
  const uint32_t src_lin = 2048 + 16 * lane;
  const uint32_t ring_base = lds_address(ring) + wave * (kQuantSlots * kRecordBytes);
  // (the waves take the split's records round robin; a contiguous quarter per wave measured slower: 16 x 65536
  // tokens int4 +0.3 us per call, one sequence of 131072 tokens +0.7 us)
  const int nrec = blk1 > blk0 + wave ? (blk1 - blk0 - wave + 3) / 4 : 0;   // records of this wave
  auto request = [&](int i) {                 // record i of this wave -> ring slot i % kQuantSlots
    const size_t off = static_cast<size_t>(blk0 + wave + 4 * i) * kRecordBytes;
    const uint64_t ga = reinterpret_cast<uint64_t>(rec_base) + off;
    // the address is wave-uniform; readfirstlane (which returns a signed int: widen it unsigned)
    // tells the compiler so, and the load can take it from scalar registers
    const uint32_t ga_lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(ga))));
    const uint32_t ga_hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(ga >> 32))));
    const uint8_t* rec = reinterpret_cast<const uint8_t*>((static_cast<uint64_t>(ga_hi) << 32) | static_cast<uint64_t>(ga_lo));
    const uint32_t dst = ring_base + (i % kQuantSlots) * kRecordBytes;
    load_to_lds(rec, src_key[0], dst);
    load_to_lds(rec, src_key[1], dst + 1024);
    load_to_lds(rec, src_lin, dst + 2048);
    load_to_lds(rec + 1024, src_lin, dst + 3072);
    load_to_lds(rec + 2048, src_lin, dst + 4096);
  };
  const int hloc = pass * HPW + hq;
  const bool head_ok = hloc < p.g;

  // the ring's first records are requested before the query is even loaded: the wait for the query (which the
  // conversions below need) then covers them too - one trip to memory before the loop, not two in a row
  // (0.3 - 0.6 us per call at 16 x 65536 tokens)
#pragma unroll
  for (int i = 0; i < kQuantSlots; ++i)
    if (i < nrec) request(i);

  // query as B operand of the score product: channels 32j .. 32j+31 in natural fp16 pairs, with the
  // softmax scale, log2(e) and the 1/f of the code field each channel meets folded in
  uint32_t qn[16];
  {
    const uint16_t* qp = p.q + (static_cast<size_t>(b) * p.n_q_heads + kvh * p.g + (head_ok ? hloc : 0)) * kHeadDim + 32 * j;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint4 raw = *reinterpret_cast<const uint4*>(qp + 8 * i);
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        // pair index 4i+k: int4 words hold 8 channels (pairs k = 0..3 of word i: f = 1,16,1,16);
        // int2 words hold 16 channels (pairs r = 0..7 of word i/2: f = 4^(r&3), r = 4*(i&1) + k)
        const float f = (BITS == 4) ? ((k & 1) ? 0.0625f : 1.f) : (k == 0 ? 1.f : k == 1 ? 0.25f : k == 2 ? 0.0625f : 0.015625f);
        const float sc = head_ok ? p.scale_log2e * f : 0.f;
        qn[4 * i + k] = pack_half2(bf16_lo(w[k]) * sc, bf16_hi(w[k]) * sc);
      }
    }
  }
  // per-pair un-scaling constants for operands that must stay un-scaled (the key-zero product)
  uint32_t finv[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const float f = (BITS == 4) ? ((k & 1) ? 16.f : 1.f) : (k == 0 ? 1.f : k == 1 ? 4.f : k == 2 ? 16.f : 64.f);
    finv[k] = pack_half2(f, f);
  }
  // (finv doubles as an A operand - the field factor of every k-slot pair, the same in every row: pair k of a
  // probability register quadruple meets f = 1, 16, 1, 16 (int4) or 1, 4, 16, 64 (int2))

  // log2 of the field factor f of each probability register (token position inside its word)
  // int4: token e of a word -> pair e/2 -> f = 16 if (e/2) odd;  int2: pair r = e/2, f = 4^(r&3)
  // register index i of score tile T is token 4*T' + i of the word, see below
  float m_run = -INFINITY;                    // running maximum of this column's head (log2 domain)
  float4v lacc = {0.f, 0.f, 0.f, 0.f};        // sum 2^(s - m_run) of this column, in every row of the tile
  float4v oacc[8], ozero[GPS];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) oacc[dt] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int gi = 0; gi < GPS; ++gi) ozero[gi] = float4v{0.f, 0.f, 0.f, 0.f};

  // query with the field factor undone again, for the key-zero product
  uint32_t qnf[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) qnf[i] = as_u32(as_half2(qn[i]) * as_half2(finv[i & 3]));

  // the query must be complete before the loop: a wait for its loads inside the loop would also drain
  // the records in flight at every step
#pragma unroll
  for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(qn[i]));

  for (int it = 0; it < nrec; ++it) {
    // this record has landed once only the younger requests are outstanding
    const int younger = nrec - 1 - it;
    if (younger >= kQuantSlots - 1) wait_vm<5 * (kQuantSlots - 1)>();
    else if (younger == 1) wait_vm<5>();
    else wait_vm<0>();
    const uint32_t rec = ring_base + (it % kQuantSlots) * kRecordBytes;
    // ---------------- this lane's share of the record, LDS -> registers ----------------
    uint32_t kw[NT][BITS == 4 ? 4 : 2];
#pragma unroll
    for (int T = 0; T < NT; ++T) {
      // tile row m = n is token (TB/4)*(m>>2) + 4*T + (m&3) of the block
      if constexpr (BITS == 4) {
        const u32x4v v = lds_load_u32x4(rec + (64 * T + lane) * 16);
        kw[T][0] = v[0]; kw[T][1] = v[1]; kw[T][2] = v[2]; kw[T][3] = v[3];
      } else {
        const u32x2v v = lds_load_u32x2(rec + 512 * T + 32 * n + 8 * j);
        kw[T][0] = v[0]; kw[T][1] = v[1];
      }
    }
    uint32_t ksc[16], kzr[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u32x4v s4 = lds_load_u32x4(rec + 4096 + 64 * j + 16 * i);
      const u32x4v z4 = lds_load_u32x4(rec + 4096 + 256 + 64 * j + 16 * i);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        ksc[4 * i + k] = s4[k];
        kzr[4 * i + k] = z4[k];
      }
    }
    uint32_t vsl[2][4];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const u32x4v v = lds_load_u32x4(rec + 2048 + (64 * c + lane) * 16);
#pragma unroll
      for (int k = 0; k < 4; ++k) vsl[c][k] = v[k];
    }
    uint32_t vsc[NKS][GPS][4], vzr[NKS][GPS][4];
#pragma unroll
    for (int a = 0; a < NKS; ++a)
#pragma unroll
      for (int gi = 0; gi < GPS; ++gi) {
        // value scale / zero of this slot's channel group gi for the 8 tokens (TB/4)*j + 8a .. +7
        const int off = 2 * (group_of(gi) * TB + (TB / 4) * j + 8 * a);
        const u32x4v sv = lds_load_u32x4(rec + 4608 + off);
        const u32x4v zv = lds_load_u32x4(rec + 4608 + 256 + off);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          vsc[a][gi][k] = sv[k];
          vzr[a][gi][k] = zv[k];
        }
      }
    // the slot is free once those reads have returned: request the record kQuantSlots ahead
    wait_lds_reads();
    if (it + kQuantSlots < nrec) request(it + kQuantSlots);

    // ---------------- scores ----------------
    uint32_t qf[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) qf[i] = as_u32(as_half2(qn[i]) * as_half2(ksc[i]));    // q * sK / f
    float4v init = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      // the key zeros are the A operand themselves (every row the same: a lane's k-slots are its channels
      // 32j + 8s .., exactly the ones its query registers cover), so they cost no multiply
      const uint32_t az[4] = {kzr[4 * s], kzr[4 * s + 1], kzr[4 * s + 2], kzr[4 * s + 3]};
      const uint32_t bq[4] = {qnf[4 * s], qnf[4 * s + 1], qnf[4 * s + 2], qnf[4 * s + 3]};
      init = mfma16(az, bq, init);         // sum_d zK[d] q[d]: the zero-point part of every score of the record
    }
    float4v sacc[NT];
#pragma unroll
    for (int T = 0; T < NT; ++T) {
      float4v acc = {0.f, 0.f, 0.f, 0.f};     // 2^-24 * the code part of the scores
      if constexpr (BITS == 4) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          uint32_t ka[4];
          unpack_i4(kw[T][s], ka);
          const uint32_t bf[4] = {qf[4 * s], qf[4 * s + 1], qf[4 * s + 2], qf[4 * s + 3]};
          acc = mfma16(ka, bf, acc);
        }
      } else {
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          uint32_t k8[8];
          unpack_i2(kw[T][h2], k8);
#pragma unroll
          for (int a2 = 0; a2 < 2; ++a2) {
            const int s = 2 * h2 + a2;
            const uint32_t ka[4] = {k8[4 * a2], k8[4 * a2 + 1], k8[4 * a2 + 2], k8[4 * a2 + 3]};
            const uint32_t bf[4] = {qf[4 * s], qf[4 * s + 1], qf[4 * s + 2], qf[4 * s + 3]};
            acc = mfma16(ka, bf, acc);
          }
        }
      }
      sacc[T] = acc;
    }
    // lane (n, j) now holds, for column n, register i of tile T = token (TB/4)*j + 4T + i

    // ---------------- softmax with a lazily updated maximum ----------------
    const float zpart = init[0];              // (every row of the tile holds the same sum)
    float smax = sacc[0][0];
#pragma unroll
    for (int T = 0; T < NT; ++T)
#pragma unroll
      for (int i = 0; i < 4; ++i) smax = fmaxf(smax, sacc[T][i]);
    smax = fmaf(smax, kCodeScale, zpart);      // the largest score of this lane
    if (__any(smax > m_run + kLazyMargin)) {
      // agree on the new maximum among the lanes of this head (all slots, all row blocks)
      float mx = smax;
      if constexpr (HPW == 4) mx = fmaxf(mx, __shfl_xor(mx, 4, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 8, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mn = fmaxf(m_run, mx);
      const float alpha = exp2_diff(m_run, mn);
      lacc *= alpha;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) oacc[dt] *= alpha;
#pragma unroll
      for (int gi = 0; gi < GPS; ++gi) ozero[gi] *= alpha;
      m_run = mn;
    }
    // probabilities, pre-divided by the field factor of the value code they will meet:
    // token e of a value word (e = 4*(T&1) + i for int4, 4*(T&3) + i for int2) sits in pair e/2
    uint32_t pb[NKS][4];
#pragma unroll
    for (int a = 0; a < NKS; ++a) {
      float pe[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int T = 2 * a + (e >> 2), i = e & 3;
        const int r = (BITS == 4) ? (e >> 1) : ((8 * a + e) >> 1);
        const float lf = (BITS == 4) ? ((r & 1) ? 4.f : 0.f) : 2.f * (r & 3);     // log2 f
        pe[e] = __builtin_amdgcn_exp2f(fmaf(sacc[T][i], kCodeScale, zpart - (m_run + lf)));
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) pb[a][k] = pack_half2(pe[2 * k], pe[2 * k + 1]);
    }

    // ---------------- output ----------------
    uint32_t pg[NKS][GPS][4];
#pragma unroll
    for (int a = 0; a < NKS; ++a) {
      // the denominator and the value-zero term need the probabilities with their field factor undone: both are
      // products with a constant A operand that holds the factor of each k-slot (in every row), which sums
      // f * (p / f) [* zV] over the 32 tokens of the k-step for every column - no multiply to undo the factor
      // (8 per lane and record), no multiply-adds for the denominator (16)
      lacc = mfma16(finv, pb[a], lacc);
#pragma unroll
      for (int gi = 0; gi < GPS; ++gi) {
        uint32_t pz[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          pg[a][gi][k] = as_u32(as_half2(pb[a][k]) * as_half2(vsc[a][gi][k]));   // p * sV / f
          pz[k] = as_u32(as_half2(pb[a][k]) * as_half2(vzr[a][gi][k]));          // p * zV / f
        }
        ozero[gi] = mfma16(finv, pz, ozero[gi]);           // sum_t p[t] zV[t][G]
      }
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
#pragma unroll
      for (int qq = 0; qq < 4; ++qq) {
        const int dt = 4 * c + qq;
        const int gi = index_in_slot(dt / TPG);   // which of its groups a column uses for this tile
        if constexpr (BITS == 4) {
          uint32_t va[4];
          unpack_i4(vsl[c][qq], va);
          oacc[dt] = mfma16(va, pg[0][gi], oacc[dt]);
        } else {
          uint32_t v8[8];
          unpack_i2(vsl[c][qq], v8);
#pragma unroll
          for (int a = 0; a < NKS; ++a) {
            const uint32_t va[4] = {v8[4 * a], v8[4 * a + 1], v8[4 * a + 2], v8[4 * a + 3]};
            oacc[dt] = mfma16(va, pg[a][gi], oacc[dt]);
          }
        }
      }
    }
  }

  // ---------------- end of split: wave state -> LDS -> merged partial ----------------
  wait_vm<0>();                               // nothing may land in the ring any more: it is reused below
  constexpr int kWaveFloats = kQuantSlots * kRecordBytes / 4;
  float* st = reinterpret_cast<float*>(ring);                 // [wave][head][kPartialFloats], each wave in its own ring
  {
    float* mine = st + wave * kWaveFloats + hq * kPartialFloats;
    // the lanes of a head agree on m_run; the constant-operand product has summed l over all tokens (slots are replicas)
    const float lsum = lacc[0];
    if (j == 0 && slot == 0) {
      mine[0] = m_run;
      mine[1] = lsum;
    }
    // output tile dt (channels 16dt..16dt+15) is valid in the columns whose slot carries its group
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      const int Gd = dt / TPG;
      if (slot == slot_of(Gd)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) mine[2 + 16 * dt + 4 * j + i] = fmaf(oacc[dt][i], kCodeScale, ozero[index_in_slot(Gd)][i]);
      }
    }
  }
  __syncthreads();
  const int oslot = p.slot0 + sp;
  for (int idx = threadIdx.x; idx < HPW * kHeadDim; idx += 256) {
    const int i = idx >> 7, d = idx & 127;
    const int hl = pass * HPW + i;
    if (hl >= p.g) continue;
    const float* s0 = st + i * kPartialFloats;
    const float mm = fmaxf(fmaxf(s0[0], s0[kWaveFloats]), fmaxf(s0[2 * kWaveFloats], s0[3 * kWaveFloats]));
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float a = exp2_diff(s0[w * kWaveFloats], mm);
      acc = fmaf(a, s0[w * kWaveFloats + 2 + d], acc);
      lsum = fmaf(a, s0[w * kWaveFloats + 1], lsum);
    }
    float* dst = p.ws + ((static_cast<size_t>(b) * p.n_q_heads + kvh * p.g + hl) * p.ns + oslot) * kPartialFloats;
    st_partial(dst + 2 + d, acc, fused);
    if (d == 0) {
      st_partial(dst, mm, fused);
      st_partial(dst + 1, lsum, fused);
    }
  }
  if constexpr (FUSED) finish_if_last(fz, mp, b, kvh, ceil_div_dev(nb, p.bps), ring);
}

// --------------------------------------------------------------------------------------------
// merge of the split partials, fused with the attention over the bf16 tail -> bf16 output (+ LSE)
// --------------------------------------------------------------------------------------------

// One workgroup of 512 threads per (sequence, query head): four groups of 128 threads; thread d of a
// group owns output channel d.  Group k merges the splits k, k+4, ... and accumulates the tail
// tokens k, k+4, ...; the groups are combined through LDS at the end.  The tail holds at most a few
// tens of tokens (this horizon's drafts plus a partial block), so it is attended to here instead of in
// a launch of its own: thread t of group 0 scores token t.  The kernel is pure latency (a few
// kilobytes per workgroup), so everything is requested before anything is consumed - the key row,
// the first value rows, then eight partials at a time - and the work of a head is spread over the
// groups so that even a single-sequence batch, whose heads each own ~100 splits, needs only a few
// memory round trips.
// This grouped form (kMergeGroups = 4) serves batches of few (sequence, head) pairs, where latency is
// everything; batches of hundreds of pairs take draft_merge_one_kernel below (the groups' barriers and idle
// lanes then cost more than they save).
template <int kMergeGroups>
__global__ __launch_bounds__(128 * kMergeGroups) void draft_merge_kernel(DraftMergeParams p) {
  constexpr int kTailPrefetch = 64 / kMergeGroups > 32 ? 32 : 64 / kMergeGroups;   // value rows per group requested up front
  const int b = blockIdx.y, h = blockIdx.x;
  const int d = threadIdx.x & 127, grp = threadIdx.x >> 7;
  const int n1 = p.cu_a ? ceil_div_dev(p.cu_a[b + 1] - p.cu_a[b], p.split_a) : 0;
  const int n2 = p.cu_blk ? ceil_div_dev(p.cu_blk[b + 1] - p.cu_blk[b], p.bps) : 0;
  const int nsl = n1 + n2 + (p.tail_slot >= 0 ? 1 : 0);   // the tail's partial, when the split launch made one, comes last
  int t0 = 0, nt = 0;
  if (p.tail_k && p.tail_slot < 0) {
    t0 = p.cu_tail[b];
    nt = p.cu_tail[b + 1] - t0;
  }
  const int kvh = h / p.g;
  const size_t row_stride = static_cast<size_t>(p.n_kv_heads) * kHeadDim;
  __shared__ float qs[kHeadDim];
  __shared__ float ps[128];
  __shared__ float red[2];
  __shared__ float gm[kMergeGroups], gl[kMergeGroups], gtl[kMergeGroups];
  __shared__ float gacc[kMergeGroups][kHeadDim], gtacc[kMergeGroups][kHeadDim];

  // ---- requests for the tail first (they are consumed last) ----
  uint4 kraw[16];
  uint16_t vpre[kTailPrefetch];
  float qd = 0.f;
  const uint16_t* vcol = p.tail_v + static_cast<size_t>(t0) * row_stride + static_cast<size_t>(kvh) * kHeadDim + d;
  if (nt > 0) {
    if (grp == 0) {
      qd = bf16_bits_to_float(p.q[(static_cast<size_t>(b) * p.n_q_heads + h) * kHeadDim + d]) * p.scale_log2e;
      const int tk = min(d, nt - 1);
      const uint16_t* kr = p.tail_k + static_cast<size_t>(t0 + tk) * row_stride + static_cast<size_t>(kvh) * kHeadDim;
#pragma unroll
      for (int i = 0; i < 16; ++i) kraw[i] = *reinterpret_cast<const uint4*>(kr + 8 * i);
    }
#pragma unroll
    for (int i = 0; i < kTailPrefetch; ++i) vpre[i] = vcol[static_cast<size_t>(min(grp + kMergeGroups * i, nt - 1)) * row_stride];
  }

  // ---- this group's share of the split partials, eight at a time ----
  const float* base = p.ws + (static_cast<size_t>(b) * p.n_q_heads + h) * p.ns * kPartialFloats;
  float mm = -INFINITY, acc = 0.f, lsum = 0.f;
  for (int s0 = grp; s0 < nsl; s0 += 8 * kMergeGroups) {
    float m8[8], l8[8], o8[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int si = s0 + kMergeGroups * i;
      const int s = min(si, nsl - 1);
      const float* pp = base + static_cast<size_t>(s < n1 ? s : s < n1 + n2 ? p.s1 + (s - n1) : p.tail_slot) * kPartialFloats;
      m8[i] = si < nsl ? pp[0] : -INFINITY;
      l8[i] = pp[1];
      o8[i] = pp[2 + d];
    }
    float mn = mm;
#pragma unroll
    for (int i = 0; i < 8; ++i) mn = fmaxf(mn, m8[i]);
    const float alpha = exp2_diff(mm, mn);
    acc *= alpha;
    lsum *= alpha;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float a = exp2_diff(m8[i], mn);
      acc = fmaf(a, o8[i], acc);
      lsum = fmaf(a, l8[i], lsum);
    }
    mm = mn;
  }

  // ---- the tail, 128 tokens at a time: one more partial (mt, tl, tacc) spread over the groups ----
  float mt = -INFINITY, tacc = 0.f, tl = 0.f;
  if (nt > 0) {
    if (grp == 0) qs[d] = qd;
    __syncthreads();
    for (int c0 = 0; c0 < nt; c0 += 128) {
      const int cn = min(128, nt - c0);
      float s = -INFINITY;
      if (grp == 0) {
        const int t = c0 + d;
        if (c0 > 0 && t < nt) {
          const uint16_t* kr = p.tail_k + static_cast<size_t>(t0 + t) * row_stride + static_cast<size_t>(kvh) * kHeadDim;
#pragma unroll
          for (int i = 0; i < 16; ++i) kraw[i] = *reinterpret_cast<const uint4*>(kr + 8 * i);
        }
        if (t < nt) {
          float a = 0.f;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const uint32_t w[4] = {kraw[i].x, kraw[i].y, kraw[i].z, kraw[i].w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              a = fmaf(qs[8 * i + 2 * k], bf16_lo(w[k]), a);
              a = fmaf(qs[8 * i + 2 * k + 1], bf16_hi(w[k]), a);
            }
          }
          s = a;
        }
        const float wm = wave_max(s);
        if ((d & 63) == 0) red[d >> 6] = wm;
      }
      __syncthreads();
      const float mn = fmaxf(mt, fmaxf(red[0], red[1]));
      const float alpha = exp2_diff(mt, mn);
      if (grp == 0) ps[d] = exp2_diff(s, mn);
      __syncthreads();
      tacc *= alpha;
      tl *= alpha;
      // this group's tokens of the chunk: grp, grp + 4, ...
      int i = 0;
      if (c0 == 0) {
#pragma unroll
        for (; i < kTailPrefetch; ++i) {
          const int u = grp + kMergeGroups * i;
          const float pv = u < cn ? ps[min(u, 127)] : 0.f;
          tacc = fmaf(pv, bf16_bits_to_float(vpre[i]), tacc);
          tl += pv;
        }
      }
      for (; grp + kMergeGroups * i < cn; i += 8) {
        uint16_t v8[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int u = min(grp + kMergeGroups * (i + k), cn - 1);
          v8[k] = vcol[static_cast<size_t>(c0 + u) * row_stride];
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int u = grp + kMergeGroups * (i + k);
          const float pv = u < cn ? ps[min(u, 127)] : 0.f;
          tacc = fmaf(pv, bf16_bits_to_float(v8[k]), tacc);
          tl += pv;
        }
      }
      mt = mn;
      __syncthreads();
    }
  }

  // ---- combine the groups ----
  gacc[grp][d] = acc;
  gtacc[grp][d] = tacc;
  if (d == 0) {
    gm[grp] = mm;
    gl[grp] = lsum;
    gtl[grp] = tl;
  }
  __syncthreads();
  if (grp == 0) {
    float M = mt;
#pragma unroll
    for (int k = 0; k < kMergeGroups; ++k) M = fmaxf(M, gm[k]);
    const float at = exp2_diff(mt, M);
    float num = 0.f, den = 0.f, tnum = 0.f, tden = 0.f;
#pragma unroll
    for (int k = 0; k < kMergeGroups; ++k) {
      const float a = exp2_diff(gm[k], M);
      num = fmaf(a, gacc[k][d], num);
      den = fmaf(a, gl[k], den);
      tnum += gtacc[k][d];
      tden += gtl[k];
    }
    num = fmaf(at, tnum, num);
    den = fmaf(at, tden, den);
    const float o = den > 0.f ? num / den : 0.f;
    p.out[(static_cast<size_t>(b) * p.n_q_heads + h) * kHeadDim + d] = static_cast<uint16_t>(float_to_bf16_bits(o));
    if (p.lse && d == 0) p.lse[static_cast<size_t>(b) * p.n_q_heads + h] = den > 0.f ? (M + log2f(den)) * kLn2 : -INFINITY;
  }
}

// The one-group form (batches of hundreds of heads): 128 threads = two waves per (sequence, query head),
// thread d owns output channel d.  Nothing in it crosses waves, so it has no barrier: every thread merges
// the split partials of the head for its channel, and each wave scores all tail tokens by itself - two
// lanes per token, 64 channels each, packed bf16 dot products against the query row (no conversion, no
// staging of the query in LDS), one shuffle - takes the maximum and the exponentials inside the wave and
// hands the probabilities to its 64 channel threads through a strip of LDS of its own.  (With a barrier
// after each of these phases and one thread per token the tail cost 2.6 us whatever its length: 4.0 us
// for a call without tail tokens against 6.6 us with one.)
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot8_bf16(const uint4& a, const uint4& b, float c) {
  c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2v, a.x), __builtin_bit_cast(bf16x2v, b.x), c, false);
  c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2v, a.y), __builtin_bit_cast(bf16x2v, b.y), c, false);
  c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2v, a.z), __builtin_bit_cast(bf16x2v, b.z), c, false);
  c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2v, a.w), __builtin_bit_cast(bf16x2v, b.w), c, false);
  return c;
}

// COHERENT: the partials were written by other workgroups of the launch that is still running (fused
// finish): read them with device-coherent loads.  CHUNK: partials requested at once.  `probs`: the calling
// wave's strip of 64 floats in LDS.
template <bool COHERENT, int CHUNK>
__device__ __forceinline__ void merge_head(const DraftMergeParams& p, int b, int h, int d, float* probs) {
  constexpr int kPre = 32;                       // value rows requested up front
  const int lane = threadIdx.x & 63;
  const int half = lane & 1, tk = lane >> 1;     // this lane scores channels 64*half .. +63 of tokens tk and 32 + tk of a chunk
  const int n1 = p.cu_a ? ceil_div_dev(p.cu_a[b + 1] - p.cu_a[b], p.split_a) : 0;
  const int n2 = p.cu_blk ? ceil_div_dev(p.cu_blk[b + 1] - p.cu_blk[b], p.bps) : 0;
  const int nsl = n1 + n2 + (p.tail_slot >= 0 ? 1 : 0);   // the tail's partial, when the split launch made one, comes last
  int t0 = 0, nt = 0;
  if (p.tail_k && p.tail_slot < 0) {
    t0 = p.cu_tail[b];
    nt = p.cu_tail[b + 1] - t0;
  }
  const int kvh = h / p.g;
  const size_t row_stride = static_cast<size_t>(p.n_kv_heads) * kHeadDim;

  // ---- requests for the tail first (they are consumed last) ----
  uint4 qraw[8], kraw[2][8];
  uint16_t vpre[kPre];
  const uint16_t* kcol = p.tail_k + static_cast<size_t>(t0) * row_stride + static_cast<size_t>(kvh) * kHeadDim + 64 * half;
  const uint16_t* vcol = p.tail_v + static_cast<size_t>(t0) * row_stride + static_cast<size_t>(kvh) * kHeadDim + d;
  if (nt > 0) {
    const uint16_t* qp = p.q + (static_cast<size_t>(b) * p.n_q_heads + h) * kHeadDim + 64 * half;
#pragma unroll
    for (int i = 0; i < 8; ++i) qraw[i] = *reinterpret_cast<const uint4*>(qp + 8 * i);
#pragma unroll
    for (int ps = 0; ps < 2; ++ps) {
      const uint16_t* kr = kcol + static_cast<size_t>(min(32 * ps + tk, nt - 1)) * row_stride;
#pragma unroll
      for (int i = 0; i < 8; ++i) kraw[ps][i] = *reinterpret_cast<const uint4*>(kr + 8 * i);
    }
#pragma unroll
    for (int i = 0; i < kPre; ++i) vpre[i] = vcol[static_cast<size_t>(min(i, nt - 1)) * row_stride];
  }

  // ---- the split partials, CHUNK at a time ----
  const float* base = p.ws + (static_cast<size_t>(b) * p.n_q_heads + h) * p.ns * kPartialFloats;
  auto ld = [](const float* q) {
    return COHERENT ? __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *q;
  };
  float mm = -INFINITY, acc = 0.f, lsum = 0.f;
  for (int s0 = 0; s0 < nsl; s0 += CHUNK) {
    float m8[CHUNK], l8[CHUNK], o8[CHUNK];
#pragma unroll
    for (int i = 0; i < CHUNK; ++i) {
      const int si = s0 + i;
      const int sl = min(si, nsl - 1);
      const float* pp = base + static_cast<size_t>(sl < n1 ? sl : sl < n1 + n2 ? p.s1 + (sl - n1) : p.tail_slot) * kPartialFloats;
      m8[i] = si < nsl ? ld(pp) : -INFINITY;
      l8[i] = ld(pp + 1);
      o8[i] = ld(pp + 2 + d);
    }
    float mn = mm;
#pragma unroll
    for (int i = 0; i < CHUNK; ++i) mn = fmaxf(mn, m8[i]);
    const float alpha = exp2_diff(mm, mn);
    acc *= alpha;
    lsum *= alpha;
#pragma unroll
    for (int i = 0; i < CHUNK; ++i) {
      const float a = exp2_diff(m8[i], mn);
      acc = fmaf(a, o8[i], acc);
      lsum = fmaf(a, l8[i], lsum);
    }
    mm = mn;
  }

  // ---- the tail, 64 tokens at a time, each wave for itself ----
  float mt = -INFINITY, tacc = 0.f, tl = 0.f;
  for (int c0 = 0; c0 < nt; c0 += 64) {
    const int cn = min(64, nt - c0);
    float sc[2];
#pragma unroll
    for (int ps = 0; ps < 2; ++ps) {
      const int t = c0 + 32 * ps + tk;
      if (c0 > 0) {
        const uint16_t* kr = kcol + static_cast<size_t>(min(t, nt - 1)) * row_stride;
#pragma unroll
        for (int i = 0; i < 8; ++i) kraw[ps][i] = *reinterpret_cast<const uint4*>(kr + 8 * i);
      }
      float a = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) a = dot8_bf16(kraw[ps][i], qraw[i], a);
      a += __shfl_xor(a, 1, 64);
      sc[ps] = t < nt ? a * p.scale_log2e : -INFINITY;
    }
    const float mn = fmaxf(mt, wave_max(fmaxf(sc[0], sc[1])));
    const float alpha = exp2_diff(mt, mn);
    // LDS operations of one wave are carried out in order, so the reads below see these writes, and the
    // writes of the next chunk come after this chunk's reads: no barrier, the wave is alone on its strip
    if (half == 0) {
      probs[tk] = exp2_diff(sc[0], mn);
      probs[32 + tk] = exp2_diff(sc[1], mn);
    }
    __builtin_amdgcn_wave_barrier();
    tacc *= alpha;
    tl *= alpha;
    int i = 0;
    if (c0 == 0) {
#pragma unroll
      for (; i < kPre; ++i) {
        const float pv = i < cn ? probs[i] : 0.f;
        tacc = fmaf(pv, bf16_bits_to_float(vpre[i]), tacc);
        tl += pv;
      }
    }
    for (; i < cn; i += 8) {
      uint16_t v8[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v8[k] = vcol[static_cast<size_t>(c0 + min(i + k, cn - 1)) * row_stride];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float pv = i + k < cn ? probs[i + k] : 0.f;
        tacc = fmaf(pv, bf16_bits_to_float(v8[k]), tacc);
        tl += pv;
      }
    }
    mt = mn;
    __builtin_amdgcn_wave_barrier();
  }

  const float M = fmaxf(mm, mt);
  const float am = exp2_diff(mm, M), at = exp2_diff(mt, M);
  const float num = fmaf(at, tacc, am * acc), den = fmaf(at, tl, am * lsum);
  const float o = den > 0.f ? num / den : 0.f;
  p.out[(static_cast<size_t>(b) * p.n_q_heads + h) * kHeadDim + d] = static_cast<uint16_t>(float_to_bf16_bits(o));
  if (p.lse && d == 0) p.lse[static_cast<size_t>(b) * p.n_q_heads + h] = den > 0.f ? (M + log2f(den)) * kLn2 : -INFINITY;
}

// (two heads per workgroup: 0.3 us per call faster than one at 512 heads, four slower again)
__global__ __launch_bounds__(256) void draft_merge_one_kernel(DraftMergeParams p) {
  __shared__ float probs[4][64];
  const int h = 2 * blockIdx.x + (threadIdx.x >> 7);
  if (h >= p.n_q_heads) return;
  // (a head of at most four partials asks for four at once, not eight)
  if (p.ns <= 4) merge_head<false, 4>(p, blockIdx.y, h, threadIdx.x & 127, probs[threadIdx.x >> 6]);
  else merge_head<false, 8>(p, blockIdx.y, h, threadIdx.x & 127, probs[threadIdx.x >> 6]);
}

// --------------------------------------------------------------------------------------------
// host side
// --------------------------------------------------------------------------------------------
struct DraftPlan {
  int split_a, s1;   // bf16 pool source: tokens per split, splits of the longest sequence
  int bps, s2;       // block records: records per split, splits of the longest sequence
  bool flat_a, flat_b;   // launches that hold only the splits that exist (flat_split)
  bool fused;            // the split kernel's last workgroup per (sequence, KV head) merges: no merge launch
  int row_waves;         // waves per workgroup of the row kernel (4, or 2: two workgroups per compute unit)
  bool tail_split;       // the tail is one more partial, made by extra workgroups of a split launch (tail_partial)
  int ns;
};

// Work is cut into equal chunks so that the whole launch is about one resident round of
// workgroups (`target`), never smaller than `min_per` units per chunk.
static int pick_chunk(int64_t sum_units, int max_units, int lists, int unit, int min_per, int target) {
  if (max_units <= 0) return unit;
  if (sum_units <= 0) sum_units = static_cast<int64_t>(max_units) * lists;
  int64_t per = ceil_div64(sum_units, target > 0 ? target : 1);
  if (per < min_per) per = min_per;
  if (per > max_units) per = max_units;
  per = ceil_div64(per, unit) * unit;
  return static_cast<int>(per);
}

// Query heads per pass of the record kernel: int4 takes 4 heads x 4 slots up to a GQA ratio of 4
// (one slot per channel group, three workgroups per CU) and 8 x 2 above; int2 has only two channel
// groups, so 8 x 2 wastes no column and measured 3-4 % faster at every ratio.
static int heads_per_pass(int bits, int g) { return (bits == 2 || g > 4) ? 8 : 4; }

static DraftPlan make_plan(const vc_comp_kv* kv) {
  DraftPlan pl{};
  const int g = kv->n_q_heads / kv->n_kv_heads;
  const int lists = kv->n_seqs * kv->n_kv_heads;
  const bool has_a = kv->pool_k != nullptr && kv->max_keep > 0;
  const bool has_b = kv->blocks != nullptr && kv->max_blk > 0;
  // A uniform batch wants exactly one resident round of equal chunks (1 workgroup per CU for the
  // row kernel, whose ring fills the LDS; 3 for the record kernel); a ragged one leaves
  // remainders and balances better with chunks half as long (config 4: 189 -> 174 us).
  auto uniform = [&](int sum, int mx) {
    return sum <= 0 || static_cast<int64_t>(mx) * kv->n_seqs * 10 <= static_cast<int64_t>(sum) * 11;
  };
  // ragged: workgroups of two waves, two per compute unit - the same rows in flight, but the launch ends
  // in pieces half as long (config 4, 576 pieces over 16 lists of 228 ... 12710 rows: 48.2 -> 39.3 us).
  // A uniform batch gains nothing from that (one piece per compute unit either way: 72.7 / 73.1 us) and
  // loses when its lists are cut finer (78.6 us): fewer, longer row streams suit the memory better.
  const bool ragged_a = !uniform(kv->sum_keep, kv->max_keep);
  pl.row_waves = tunable(kTunDraftRowWaves, ragged_a ? 2 : 4, 2, 4) == 2 ? 2 : 4;
  const int target_a = tunable(kTunDraftBf16Wgs, ragged_a ? 512 : 256, 1, 1 << 20);
  // (a handful of lists - one long sequence - does better with one workgroup per CU: 256 against 768 measured
  // 29.8 against 31.8 us for the record kernel and 5.4 against 7.4 us for the merge at 8 lists of 4096 records)
  const int npass_b = ceil_div(g, heads_per_pass(kv->bits, g));
  const int target_b = tunable(kTunDraftQuantWgs, lists * npass_b < 32 ? 256 : uniform(kv->sum_blk, kv->max_blk) ? 768 : 1536, 1, 1 << 20);
  pl.split_a = pick_chunk(static_cast<int64_t>(kv->sum_keep) * kv->n_kv_heads, kv->max_keep, lists, 128,
                          tunable(kTunDraftMinTok, 256, 128, 1 << 20), target_a);
  pl.s1 = has_a ? ceil_div(kv->max_keep, pl.split_a) : 0;
  const int npass = npass_b;
  pl.bps = pick_chunk(static_cast<int64_t>(kv->sum_blk) * kv->n_kv_heads * npass, kv->max_blk, lists * npass, 4,
                      tunable(kTunDraftMinBlk, 16, 4, 1 << 20), target_b);
  pl.s2 = has_b ? ceil_div(kv->max_blk, pl.bps) : 0;
  // a ragged batch of at most 64 sequences launches only the splits that exist (config 4: 178 -> 165 us
  // with the record kernel launched so)
  const bool flat_ok = tunable(kTunDraftFlat, 1, 0, 1) != 0 && kv->n_seqs <= 64;
  pl.flat_a = flat_ok && has_a && !uniform(kv->sum_keep, kv->max_keep) &&
              static_cast<int64_t>(pl.s1) * lists <= (1ll << 30);
  pl.flat_b = flat_ok && has_b && !uniform(kv->sum_blk, kv->max_blk) &&
              static_cast<int64_t>(pl.s2) * lists * npass <= (1ll << 30);
  // A tiny launch from one source finishes inside its split kernel (finish_if_last): 13.3 -> 11.4 us per call
  // for one sequence of 4096 tokens (16 workgroups).  From a few hundred workgroups on the merge launch is
  // faster: every trip of the finishing workgroup to device-coherent memory (count, partials) takes about as
  // long as a launch, and the pairs all complete at the end of the launch together (256 workgroups: 16.8 ->
  // 17.8 us at 8 sequences x 2048 kept rows, 75.5 -> 89.4 ms for the 2048 calls of a 131072-token horizon;
  // config 2: 3 - 15 us slower per call).
  const int64_t wgs = has_a ? static_cast<int64_t>(pl.s1) * lists : static_cast<int64_t>(pl.s2) * lists * npass;
  pl.fused = has_a != has_b && lists <= vc_ctx::kDraftMaxLists && wgs <= tunable(kTunDraftFused, 64, 0, 1 << 20);
  if (pl.fused) pl.flat_a = pl.flat_b = false;   // every list needs its first workgroup, rows or not
  // With a merge launch of its own, the tail is attended to beside the splits, not in the merge
  // (its workgroups sit in grid slices behind the sequences': the grid's z extent stays below 65536)
  pl.tail_split = !pl.fused && (has_a || has_b) && kv->tail_k != nullptr && kv->max_tail > 0 && kv->n_seqs <= 32767 &&
                  tunable(kTunDraftTailSplit, 1, 0, 1) != 0;
  pl.ns = pl.s1 + pl.s2 + (pl.tail_split ? 1 : 0);
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
  VC_REQUIRE(kv->n_seqs <= 65535 && kv->n_kv_heads * 4 <= 65535 && kv->n_q_heads <= 65535, VC_ERR_UNSUPPORTED,
             "%s: batch too large for one launch", who);
  VC_REQUIRE(kv->max_keep >= 0 && kv->max_blk >= 0 && kv->max_tail >= 0 && kv->sum_keep >= 0 && kv->sum_blk >= 0,
             VC_ERR_INVALID_ARG, "%s: negative count", who);
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

// Scratch of the entry point that allocates nothing (vc_draft_attn_static): the split partials live in
// this file-scope device array instead of a caller workspace.  Every GPU holds its own copy at its
// own address; the address is looked up once per device (draft_init_device, with that device
// current) and host code only ever uses that pointer, never the symbol itself.
constexpr size_t kStaticScratchBytes = static_cast<size_t>(8) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::atomic<void*> scratch_ptr[kMaxDevices];

// the row kernel's ring needs more dynamic LDS than the default limit: a per-device function attribute
// The split kernels exist in two instantiations each: with the fused finish (small launches: fz.counters
// set) and without.
template <bool GATHER, int NW>
static void launch_rows(dim3 grid, hipStream_t st, const DraftBf16Params& bp, const DraftMergeParams& mp, const DraftFuse& fz) {
  if (fz.counters) hipLaunchKernelGGL((draft_bf16_kernel<GATHER, 32, NW, true>), grid, dim3(NW * 64), rows_lds(32, NW), st, bp, mp, fz);
  else hipLaunchKernelGGL((draft_bf16_kernel<GATHER, 32, NW, false>), grid, dim3(NW * 64), rows_lds(32, NW), st, bp, mp, fz);
}
template <int BITS, int HPW>
static void launch_records(dim3 grid, hipStream_t st, const DraftQuantParams& qp, const DraftMergeParams& mp, const DraftFuse& fz) {
  if (fz.counters) hipLaunchKernelGGL((draft_quant_kernel<BITS, HPW, true>), grid, dim3(256), kQuantRingBytes, st, qp, mp, fz);
  else hipLaunchKernelGGL((draft_quant_kernel<BITS, HPW, false>), grid, dim3(256), kQuantRingBytes, st, qp, mp, fz);
}
template <bool GATHER, int NW>
static vc_status rows_attributes() {
  VC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(draft_bf16_kernel<GATHER, 32, NW, false>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, rows_lds(32, NW)));
  VC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(draft_bf16_kernel<GATHER, 32, NW, true>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, rows_lds(32, NW)));
  return VC_OK;
}

vc_status draft_init_device() {
  int dev = -1;
  VC_HIP(hipGetDevice(&dev));
  if (dev >= 0 && dev < kMaxDevices && scratch_ptr[dev].load(std::memory_order_acquire) == nullptr) {
    void* ptr = nullptr;
    VC_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  vc_status st = rows_attributes<true, 4>();
  if (st == VC_OK) st = rows_attributes<false, 4>();
  if (st == VC_OK) st = rows_attributes<true, 2>();
  if (st == VC_OK) st = rows_attributes<false, 2>();
  if (st != VC_OK) return st;
  return VC_OK;
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

// Both draft entry points: `workspace` is the caller's buffer (vc_draft_attn) or this device's
// static scratch (vc_draft_attn_static, whose `who` names it in messages).
static vc_status draft_attn_impl(const char* who, vc_ctx* ctx, const vc_comp_kv* kv, const void* q, float softmax_scale,
                                 void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  VC_REQUIRE(q && out, VC_ERR_INVALID_ARG, "%s: q or out is NULL", who);
  VC_REQUIRE(aligned16(q) && aligned16(out), VC_ERR_INVALID_ARG, "%s: q/out not 16-byte aligned", who);
  size_t need = 0;
  vc_draft_workspace_bytes(kv, &need);
  VC_REQUIRE(workspace != nullptr && workspace_bytes >= need, VC_ERR_WORKSPACE, "%s: workspace %zu bytes, need %zu", who,
             workspace_bytes, need);
  VC_REQUIRE(aligned16(workspace), VC_ERR_INVALID_ARG, "%s: workspace not 16-byte aligned", who);

  const DraftPlan pl = make_plan(kv);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int g = kv->n_q_heads / kv->n_kv_heads;
  const float sl2 = softmax_scale * kLog2e;
  float* ws = static_cast<float*>(workspace);

  DraftMergeParams mp{};
  mp.ws = ws;
  mp.q = static_cast<const uint16_t*>(q);
  mp.out = static_cast<uint16_t*>(out);
  mp.lse = lse;
  mp.cu_a = pl.s1 > 0 ? (kv->keep_idx ? kv->cu_keep : kv->cu_ctx) : nullptr;
  mp.cu_blk = pl.s2 > 0 ? kv->cu_blk : nullptr;
  const bool has_t = kv->tail_k != nullptr && kv->max_tail > 0;
  mp.tail_k = has_t ? static_cast<const uint16_t*>(kv->tail_k) : nullptr;
  mp.tail_v = has_t ? static_cast<const uint16_t*>(kv->tail_v) : nullptr;
  mp.cu_tail = kv->cu_tail;
  mp.n_q_heads = kv->n_q_heads; mp.n_kv_heads = kv->n_kv_heads; mp.g = g; mp.ns = pl.ns;
  mp.split_a = pl.split_a; mp.s1 = pl.s1; mp.bps = pl.bps;
  mp.tail_slot = pl.tail_split ? pl.s1 + pl.s2 : -1;
  mp.scale_log2e = sl2;
  DraftFuse fz{};
  if (pl.fused && ctx->draft_counters != nullptr) {
    // calls in flight at the same time (other streams, captured graphs) count on sets of their own
    fz.counters = ctx->draft_counters + (ctx->draft_calls++ % vc_ctx::kDraftCounterSets) *
                                            (static_cast<size_t>(vc_ctx::kDraftMaxLists) * vc_ctx::kDraftCounterStride);
    fz.expected_mul = 1;
  }

  mark_begin(ctx, st);
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
    bp.n_seqs = kv->n_seqs; bp.flat = pl.flat_a;
    // one more workgroup per (sequence, KV head) for the tails, behind the splits' in launch order.  (Handing a
    // list's tail to the workgroup of its last split instead, requested ahead of that workgroup's ring, was
    // slower: the row loop lost 1.3 us to the registers held across it - 16 x 6554 kept rows, 74.8 against 73.4 us.)
    bp.tail = pl.tail_split && pl.s2 == 0 ? 1 : 0;   // (a record launch of the same call carries them instead: it hides them)
    dim3 grid(pl.s1, kv->n_kv_heads, kv->n_seqs + (bp.tail ? ceil_div(kv->n_seqs, pl.s1) : 0));
    if (pl.flat_a) grid = dim3(static_cast<unsigned>(pl.s1 + bp.tail) * kv->n_seqs * kv->n_kv_heads, 1, 1);
    // 32-token steps (16-token steps with 8 waves measured the same: the gather itself binds); 4 waves
    // per workgroup, or 2 so that two workgroups share a compute unit (pl.row_waves)
    if (pl.row_waves == 2) {
      if (kv->keep_idx) launch_rows<true, 2>(grid, st, bp, mp, fz);
      else launch_rows<false, 2>(grid, st, bp, mp, fz);
    } else {
      if (kv->keep_idx) launch_rows<true, 4>(grid, st, bp, mp, fz);
      else launch_rows<false, 4>(grid, st, bp, mp, fz);
    }
  }
  if (pl.s2 > 0) {
    DraftQuantParams qp{};
    qp.q = static_cast<const uint16_t*>(q);
    qp.blocks = static_cast<const uint8_t*>(kv->blocks);
    qp.cu_blk = kv->cu_blk;
    qp.ws = ws;
    qp.n_q_heads = kv->n_q_heads; qp.n_kv_heads = kv->n_kv_heads; qp.g = g;
    const int hpw = heads_per_pass(kv->bits, g);
    qp.npass = ceil_div(g, hpw);
    qp.bps = pl.bps; qp.slot0 = pl.s1; qp.ns = pl.ns;
    qp.scale_log2e = sl2;
    qp.n_seqs = kv->n_seqs; qp.flat = pl.flat_b;
    // the tail's workgroups travel with the record launch whenever the call has one: three workgroups share a
    // compute unit there and the launch drains over some microseconds, which hides them; the row launch, one
    // resident round of workgroups that fill the LDS, ends 1.6 us later with them
    qp.tail = pl.tail_split ? 1 : 0;
    fz.expected_mul = qp.npass;
    // flat: every sequence has at most s2 splits, all heads of a split are neighbours in the launch
    dim3 grid(pl.s2, kv->n_kv_heads * qp.npass, kv->n_seqs + (qp.tail ? ceil_div(kv->n_seqs, pl.s2) : 0));
    if (pl.flat_b) grid = dim3(static_cast<unsigned>(pl.s2 + qp.tail) * kv->n_seqs * kv->n_kv_heads * qp.npass, 1, 1);
    if (kv->bits == 4 && hpw == 4) launch_records<4, 4>(grid, st, qp, mp, fz);
    else if (kv->bits == 4) launch_records<4, 8>(grid, st, qp, mp, fz);
    else if (hpw == 4) launch_records<2, 4>(grid, st, qp, mp, fz);
    else launch_records<2, 8>(grid, st, qp, mp, fz);
  }
  mark_end(ctx, st);
  if (fz.counters != nullptr) {
    VC_HIP(hipGetLastError());
    return VC_OK;
  }
  if (static_cast<int64_t>(kv->n_seqs) * kv->n_q_heads < 256)
    hipLaunchKernelGGL(draft_merge_kernel<4>, dim3(kv->n_q_heads, kv->n_seqs), dim3(512), 0, st, mp);
  else
    hipLaunchKernelGGL(draft_merge_one_kernel, dim3((kv->n_q_heads + 1) / 2, kv->n_seqs), dim3(256), 0, st, mp);
  VC_HIP(hipGetLastError());
  return VC_OK;
}

extern "C" vc_status vc_draft_attn(vc_ctx* ctx, const vc_comp_kv* kv, const void* q, float softmax_scale, void* out,
                                   float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  VC_REQUIRE(ctx != nullptr, VC_ERR_INVALID_ARG, "vc_draft_attn: ctx is NULL");
  vc_status stt = check_comp(kv, "vc_draft_attn");
  if (stt != VC_OK) return stt;
  if (kv->n_seqs == 0) return VC_OK;
  return draft_attn_impl("vc_draft_attn", ctx, kv, q, softmax_scale, out, lse, workspace, workspace_bytes, stream);
}

extern "C" vc_status vc_draft_static_scratch_bytes(size_t* bytes) {
  VC_REQUIRE(bytes != nullptr, VC_ERR_INVALID_ARG, "vc_draft_static_scratch_bytes: bytes is NULL");
  *bytes = kStaticScratchBytes;
  return VC_OK;
}

extern "C" vc_status vc_draft_attn_static(vc_ctx* ctx, const vc_comp_kv* kv, const void* q, float softmax_scale, void* out,
                                          float* lse, void* stream) {
  const char* who = "vc_draft_attn_static";
  VC_REQUIRE(ctx != nullptr, VC_ERR_INVALID_ARG, "%s: ctx is NULL", who);
  vc_status stt = check_comp(kv, who);
  if (stt != VC_OK) return stt;
  if (kv->n_seqs == 0) return VC_OK;
  size_t need = 0;
  vc_draft_workspace_bytes(kv, &need);
  VC_REQUIRE(need <= kStaticScratchBytes, VC_ERR_WORKSPACE,
             "%s: this batch needs %zu bytes of split partials, the static scratch holds %zu; use vc_draft_attn with a workspace",
             who, need, kStaticScratchBytes);
  VC_REQUIRE(ctx->device >= 0 && ctx->device < kMaxDevices, VC_ERR_UNSUPPORTED, "%s: device %d", who, ctx->device);
  void* ptr = scratch_ptr[ctx->device].load(std::memory_order_acquire);   // looked up by vc_create on this device
  VC_REQUIRE(ptr != nullptr, VC_ERR_HIP, "%s: the scratch address of device %d is unknown", who, ctx->device);
  return draft_attn_impl(who, ctx, kv, q, softmax_scale, out, lse, ptr, kStaticScratchBytes, stream);
}
