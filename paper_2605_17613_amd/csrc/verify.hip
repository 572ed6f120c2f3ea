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
// R <= 128 rows the waves split each 64-token tile two ways, above that every wave takes its own
// 32 rows of a 32-token tile.  K/V tiles stream from HBM straight into a ring of LDS stages
// (direct-to-LDS loads, xor-swizzled 16-byte chunks), several tiles ahead of their use.
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
  int chunk_tok, ns;   // ns = chunks of the longest sequence (one partial per row and chunk)
  int seq0, chunk0, tok_hi;   // this launch: first sequence, first chunk, end of the token range
  int nrb;                    // row blocks of 256 rows per (sequence, KV head); above one, K/V are streamed once per block
  const int* ring_slot;       // staging ring: kf / vf are ring_slots slots of chunk_tok rows, and the chunk of sequence b that
                              // this launch attends to sits in slot ring_slot[b]; nullptr: kf / vf hold every token
  int* list;                  // optional work list of a ragged launch (see verify_worklist_kernel)
  int list_seqs, list_chunks; // sequences and chunks of this launch (the full grid, walked when the list reports an overflow)
  float scale_log2e;
};

constexpr int kVerifyLds = 128 * 1024;          // ring of K/V tiles in LDS
constexpr float kVerifyMargin = 4.f;
constexpr float kMinusBig = -1.0e30f;    // "no key seen yet": finite, so 2^(s - m) needs no special cases

__device__ __forceinline__ float16v mfma32(bf16x8v a, bf16x8v b, float16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8v load_bf16x8(const uint16_t* p) {
  bf16x8v r;
  const uint4 raw = *reinterpret_cast<const uint4*>(p);
  __builtin_memcpy(&r, &raw, 16);
  return r;
}

__device__ __forceinline__ bf16x8v lds_load_bf16x8(uint32_t addr) {   // ds_read_b128
  return __builtin_bit_cast(bf16x8v, lds_load_u32x4(addr));
}
// Transposing LDS read: the 16 lanes of a block fetch a 4 x 16 patch of 16-bit values (lane 4k+c:
// row k, columns 4c..4c+3) and lane i of the block receives column i of the patch (4 rows).
__device__ __forceinline__ short4v lds_read_tr(uint32_t addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_short4v*>(static_cast<size_t>(addr)));
}

// 16-byte chunk c of tile row `row` is stored at chunk position c ^ rot(row), rot = the low four
// row bits rotated left by one.  Rows are 256 bytes with no padding (direct-to-LDS loads write 1 KB
// per wave contiguously); the xor spreads a column of chunks over all banks (K operand reads), and
// because the two lowest row bits land on chunk bits 1 and 2, the four rows of a transposing-read
// patch put their two adjacent chunks on eight different positions (V operand reads).
__device__ __forceinline__ int rot_row(int row) { return ((row << 1) & 14) | ((row >> 3) & 1); }
__device__ __forceinline__ int swz(int row, int chunk) { return row * 256 + ((chunk ^ rot_row(row)) << 4); }

// One wave owns RT row tiles of 32 rows (RT = 1 in every instantiation in use) and, of every LDS tile,
// SUB 32-token slices.  NW = 8/RT waves per workgroup; NTG = token slices per tile; NRG = NW/NTG row groups.
// Tiles travel HBM -> LDS directly (no registers) through a ring of NSTAGE stages, one barrier per tile.
// SUB = 2 (more than 128 rows: every wave has rows, and the wave's matrix instructions and its softmax
// arithmetic each take about half of its time): one code path, compute_pair, pairs the score products of
// one slice with the exponentials of the other inside the wave's instruction stream.
template <int NTG, int RT, int SUB>
__device__ __forceinline__ void verify_body(const VerifyParams& p, char* smem, int kvh, int slot, int t_begin, int t_len,
                                            int w0, int w, int c0, int N, int row0) {
  constexpr int NW = 8 / RT;
  constexpr int NRG = NW / NTG;
  constexpr int TT = 32 * NTG * SUB;           // tokens per tile
  constexpr int SLICE_BYTES = 32 * NTG * 256;  // LDS distance between two slices of one wave
  constexpr int STAGE_BYTES = TT * 512;        // K tile then V tile, 256 bytes per row
  constexpr int NSTAGE = (kVerifyLds / STAGE_BYTES) > 8 ? 8 : (kVerifyLds / STAGE_BYTES);
  constexpr int LPT = TT / (4 * NW);           // 1 KB wave-loads per matrix per wave per tile
  constexpr int DEPTH = NSTAGE - 1;            // tiles in flight
  static_assert(NSTAGE >= 3 && NSTAGE <= 8 && LPT >= 1, "ring geometry");
  const int R = w * p.g;                       // rows of the (sequence, KV head); this workgroup owns row0 .. row0 + 255
  const int total = N + w;
  const int t_end = min(min(total, p.tok_hi), t_begin + t_len);    // tokens [t_begin, t_end) -> partial `slot` of every row
  const int ntiles = (t_end - t_begin + TT - 1) / TT;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rg = wave % NRG, tg = wave / NRG;
  const int n = lane & 31, hh = lane >> 5;
  const bool wave_rows = row0 + rg * 32 * RT < R;

  int iw[RT], hq[RT];
  bool row_ok[RT];
  bf16x8v qb[RT][8];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int r = row0 + (rg * RT + rt) * 32 + n;
    row_ok[rt] = r < R;
    const int rc = row_ok[rt] ? r : R - 1;
    iw[rt] = rc / p.g;
    hq[rt] = rc % p.g;
    const uint16_t* qp = p.qw + (static_cast<size_t>(w0 + iw[rt]) * p.n_q_heads + kvh * p.g + hq[rt]) * kHeadDim + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qb[rt][ks] = load_bf16x8(qp + 16 * ks);
  }
  // pin the query registers here: their loads must be waited for before the ring starts, or the
  // wait would sit inside the loop and also drain the tiles in flight
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qb[rt][ks]));

  float m[RT], l[RT];
  float16v oacc[RT][4];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    m[rt] = kMinusBig;
    l[rt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[rt][dt][i] = 0.f;
  }

  const size_t row_stride = static_cast<size_t>(p.n_kv_heads) * kHeadDim;
  const size_t head_off = static_cast<size_t>(kvh) * kHeadDim;

  // ---- tile loads: wave-load c of this wave covers tile rows 4*(wave + NW*c) .. +3 ----
  const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<size_t>((__attribute__((address_space(3))) char*)smem));
  // fast path (tile entirely inside the full KV): a wave-uniform base address per wave-load (scalar
  // registers, advanced by scalar arithmetic) plus one per-lane byte offset that never changes, so that
  // requesting a tile costs no vector instructions
  const int wrow = 4 * wave + (lane >> 4);     // tile row of this lane in wave-load 0; wave-load c is 4 NW rows further
  const uint32_t lane_off = static_cast<uint32_t>((static_cast<size_t>(lane >> 4) * row_stride + 8 * ((lane & 15) ^ rot_row(wrow))) * 2);
  static_assert((4 * NW) % 16 == 0, "rot_row of a lane's tile row must not depend on the wave-load");
  const uint8_t* kbase_u = reinterpret_cast<const uint8_t*>(p.kf + (static_cast<size_t>(c0 + t_begin + 4 * wave) * row_stride + head_off));
  const uint8_t* vbase_u = reinterpret_cast<const uint8_t*>(p.vf + (static_cast<size_t>(c0 + t_begin + 4 * wave) * row_stride + head_off));
  const size_t tile_step = static_cast<size_t>(TT) * row_stride * 2;          // bytes
  const size_t load_step = static_cast<size_t>(4 * NW) * row_stride * 2;      // bytes between the rows of two wave-loads
  auto issue = [&](int j) {                    // request tile j into stage j % NSTAGE
    const int t = t_begin + j * TT;
    const uint32_t stage = lds_base + (j % NSTAGE) * STAGE_BYTES;
    if (t + TT <= N) {
#pragma unroll
      for (int c = 0; c < LPT; ++c) {
        const int grp = wave + NW * c;
        load_to_lds(kbase_u + static_cast<size_t>(j) * tile_step + c * load_step, lane_off, __builtin_amdgcn_readfirstlane(stage + grp * 1024));
        load_to_lds(vbase_u + static_cast<size_t>(j) * tile_step + c * load_step, lane_off,
                    __builtin_amdgcn_readfirstlane(stage + TT * 256 + grp * 1024));
      }
    } else {
#pragma unroll
      for (int c = 0; c < LPT; ++c) {
        const int grp = wave + NW * c;
        const int row = 4 * grp + (lane >> 4);
        const int chunkpos = (lane & 15) ^ rot_row(row);
        int tok = t + row;
        tok = tok < total ? tok : total - 1;   // rows past the end re-read the last row; their scores are masked
        const bool in_full = tok < N;
        const size_t grow = in_full ? static_cast<size_t>(c0 + tok) : static_cast<size_t>(w0 + tok - N);
        const size_t off = grow * row_stride + head_off + 8 * chunkpos;
        load_to_lds((in_full ? p.kf : p.kw) + off, __builtin_amdgcn_readfirstlane(stage + grp * 1024));
        load_to_lds((in_full ? p.vf : p.vw) + off, __builtin_amdgcn_readfirstlane(stage + TT * 256 + grp * 1024));
      }
    }
  };

  // ---- LDS read addresses of this lane, relative to the stage base ----
  // All operand addresses of a slice derive from three per-lane bases by an xor with a constant and a
  // constant offset (stage bases are multiples of 256, so the xor only ever touches chunk-position bits):
  //   K, k-step ks:        swz(row, 2ks + hh) = kx0 ^ (32 ks)                  row = 32 tg + n
  //   V^T, tile dt, k-step kk, half h2:  swz(row, 4dt + tr_chunk) + tr_sub = (vy0[h2] ^ (64 dt)) + 4096 kk
  //                                                                         row = 32 tg + 16 kk + 8 h2 + tr_row
  // (rot_row(row) only depends on the low four row bits: the low three, which tr_row supplies, and bit 3 = h2.)
  const uint32_t kx0 = swz(32 * tg + n, hh);
  // transposing read: lane -> (token row, 8-byte half of a 16-byte chunk) inside a 4 x 16 patch
  const int blk16 = lane >> 4;
  const int tr_row = 4 * (blk16 >> 1) + ((lane & 15) >> 2);
  const int tr_chunk = 2 * (blk16 & 1) + ((lane & 3) >> 1);
  const int tr_sub = 8 * (lane & 1);
  uint32_t vy0[2];
#pragma unroll
  for (int h2 = 0; h2 < 2; ++h2) vy0[h2] = TT * 256 + swz(32 * tg + 8 * h2 + tr_row, tr_chunk) + tr_sub;

  // One slice = 32 tokens of the tile for this wave's rows.  The operand reads of a slice are issued as a
  // batch, well ahead of the matrix instructions that take them, so that the LDS latency (a hundred cycles
  // and more per read) is paid once per batch and overlaps the softmax arithmetic: left to itself the
  // compiler places every read directly in front of its product and the wave stalls for the full latency
  // on each of the 24 products of a slice.
  auto read_k = [&](int j, int sl, bf16x8v (&kb)[8]) {                  // K operand of a slice: 8 reads of 16 bytes per lane
    const uint32_t sbase = lds_base + (j % NSTAGE) * STAGE_BYTES + sl * SLICE_BYTES;
    const uint32_t kx = sbase + kx0;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kb[ks] = lds_load_bf16x8(kx ^ (32u * ks));
  };
  auto read_v = [&](int j, int sl, bf16x8v (&vb)[2][4]) {              // V^T operand of a slice: 16 transposing reads
    // A element e of k-step kk is token row 16kk + 8(e/4) + 4hh + e%4
    const uint32_t sbase = lds_base + (j % NSTAGE) * STAGE_BYTES + sl * SLICE_BYTES;
    const uint32_t vy[2] = {sbase + vy0[0], sbase + vy0[1]};
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const short4v lo = lds_read_tr((vy[0] ^ (64u * dt)) + 4096u * kk);
        const short4v hi = lds_read_tr((vy[1] ^ (64u * dt)) + 4096u * kk);
        vb[kk][dt] = __builtin_bit_cast(bf16x8v, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }
  };
  auto scores = [&](const bf16x8v (&kb)[8], float16v (&sacc)[RT]) {    // S^T = K Q^T : one K operand feeds RT products
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[rt][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) sacc[rt] = mfma32(kb[ks], qb[rt][ks], sacc[rt]);
  };
  auto softmax = [&](int ts, float16v (&sacc)[RT], bf16x8v (&pb)[RT][2]) {
    // register i of this lane is token row 8*(i/4) + 4*hh + i%4 of the slice, for row n
    const bool edge = ts + 32 > min(N, t_end);  // slice touches the window or the end of the chunk
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      if (edge) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int tok = ts + 8 * (i >> 2) + 4 * hh + (i & 3);
          const bool ok = tok < t_end && (tok < N || tok - N <= iw[rt]);
          sacc[rt][i] = ok ? sacc[rt][i] : -INFINITY;
        }
      }
      float mt = fmaxf(sacc[rt][0], sacc[rt][1]);
#pragma unroll
      for (int i = 2; i < 16; ++i) mt = fmaxf(mt, sacc[rt][i]);
      mt *= p.scale_log2e;                     // the scale is positive: max commutes with it
      if (__any(mt > m[rt] + kVerifyMargin)) {
        const float mx = fmaxf(mt, __shfl_xor(mt, 32, 64));
        const float mn = fmaxf(m[rt], mx);
        const float alpha = __builtin_amdgcn_exp2f(m[rt] - mn);
        l[rt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[rt][dt][i] *= alpha;
        m[rt] = mn;
      }
      float ps0 = 0.f, ps1 = 0.f;
      const float negm = -m[rt];
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[rt][i], p.scale_log2e, negm));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[rt][i + 1], p.scale_log2e, negm));
        ps0 += p0;
        ps1 += p1;
        pb[rt][i >> 3][i & 7] = (__bf16)p0;
        pb[rt][i >> 3][(i & 7) + 1] = (__bf16)p1;
      }
      l[rt] += ps0 + ps1;
    }
  };
  auto output = [&](const bf16x8v (&vb)[2][4], bf16x8v (&pb)[RT][2]) {  // O^T += V^T P^T
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) oacc[rt][dt] = mfma32(vb[kk][dt], pb[rt][kk], oacc[rt][dt]);
  };
  auto compute = [&](int j) {
    if (!wave_rows) return;
    const int ts0 = t_begin + j * TT + 32 * tg;   // first token of this wave's first slice
    if (ts0 >= t_end) return;
#pragma unroll
    for (int sl = 0; sl < SUB; ++sl) {
      const int ts = ts0 + sl * 32 * NTG;
      if (sl > 0 && ts >= t_end) break;          // the chunk ends inside this tile
      bf16x8v kb[8];
      read_k(j, sl, kb);
      float16v sacc[RT];
      scores(kb, sacc);
      // V^T of this slice is requested before the softmax and lands while it runs
      bf16x8v vb[2][4];
      read_v(j, sl, vb);
      __builtin_amdgcn_sched_barrier(0);         // nothing moves across: the reads stay up here
      bf16x8v pb[RT][2];
      softmax(ts, sacc, pb);
      output(vb, pb);
    }
  };

  // The two-slice form (every wave has rows: the kernel is bound by the matrix cores and the vector unit,
  // not by HBM).  A wave's matrix instructions and its softmax arithmetic each take about half of its time,
  // and the waves of a workgroup move in lockstep behind the tile barrier, so nothing overlaps unless the
  // instruction stream of a single wave does it: a matrix instruction runs for 32 cycles once issued, and
  // independent vector instructions issued behind it execute meanwhile.  The pairing - scores of slice B
  // with the exponentials of slice A, output products of A with the exponentials of B - is pinned with
  // scheduling groups (a few vector instructions, then one matrix instruction).
  auto row_max = [&](const float16v& sc) {
    float mt = fmaxf(fmaxf(sc[0], sc[1]), sc[2]);
#pragma unroll
    for (int i = 3; i < 15; i += 2) mt = fmaxf(fmaxf(mt, sc[i]), sc[i + 1]);
    return fmaxf(mt, sc[15]) * p.scale_log2e;
  };
  // RT == 1 only: rescale the row state when the maximum jumps.  `pending` are probabilities that were taken
  // against the old maximum and whose output product has not been issued yet: they are rescaled as well.
  auto raise_max = [&](float mt, bf16x8v* pending) {
    if (__any(mt > m[0] + kVerifyMargin)) {
      const float mx = fmaxf(mt, __shfl_xor(mt, 32, 64));
      const float mn = fmaxf(m[0], mx);
      const float alpha = __builtin_amdgcn_exp2f(m[0] - mn);
      l[0] *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[0][dt][i] *= alpha;
      if (pending) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
          for (int e = 0; e < 8; ++e) pending[kk][e] = (__bf16)(static_cast<float>(pending[kk][e]) * alpha);
      }
      m[0] = mn;
    }
  };
  auto exps = [&](const float16v& sc, bf16x8v (&pb)[2]) {
    float ps0 = 0.f, ps1 = 0.f;
    const float negm = -m[0];
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
      const float p0 = __builtin_amdgcn_exp2f(fmaf(sc[i], p.scale_log2e, negm));
      const float p1 = __builtin_amdgcn_exp2f(fmaf(sc[i + 1], p.scale_log2e, negm));
      ps0 += p0;
      ps1 += p1;
      pb[i >> 3][i & 7] = (__bf16)p0;
      pb[i >> 3][(i & 7) + 1] = (__bf16)p1;
    }
    l[0] += ps0 + ps1;
  };
  auto interleave = [&]() {                      // 8 x (a few vector instructions, then one matrix instruction), then 16 LDS reads
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x002, 16, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);
  };
  auto mask_edge = [&](int ts, float16v& sc) {   // a slice that touches the window or the end of the chunk
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int tok = ts + 8 * (i >> 2) + 4 * hh + (i & 3);
      const bool ok = tok < t_end && (tok < N || tok - N <= iw[0]);
      sc[i] = ok ? sc[i] : -INFINITY;
    }
  };
  // The two-slice form (SUB == 2, RT == 1: every wave has rows), one code path for every tile: the only
  // difference at the edge of the chunk is a mask on the scores (a slice entirely past the end is masked
  // out as a whole and adds zeros).
  auto compute_pair = [&](int j) {
    const int ts0 = t_begin + j * TT;
    const bool edge = ts0 + TT > min(N, t_end);
    bf16x8v kb[8], vb[2][4], pA[2], pB[2];
    float16v sA, sB;
    read_k(j, 0, kb);
#pragma unroll
    for (int i = 0; i < 16; ++i) sA[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) sA = mfma32(kb[ks], qb[0][ks], sA);
    read_k(j, 1, kb);                            // lands while the maximum of slice A is taken
    __builtin_amdgcn_sched_barrier(0);
    if (edge) mask_edge(ts0, sA);
    raise_max(row_max(sA), nullptr);
    __builtin_amdgcn_sched_barrier(0);
    // scores of slice B  |  exponentials of slice A; then the V^T reads of slice A (into the registers K left)
#pragma unroll
    for (int i = 0; i < 16; ++i) sB[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) sB = mfma32(kb[ks], qb[0][ks], sB);
    exps(sA, pA);
    read_v(j, 0, vb);
    interleave();
    __builtin_amdgcn_sched_barrier(0);
    if (edge) mask_edge(ts0 + 32, sB);
    raise_max(row_max(sB), pA);
    __builtin_amdgcn_sched_barrier(0);
    // output products of slice A  |  exponentials of slice B; then the V^T reads of slice B
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) oacc[0][dt] = mfma32(vb[kk][dt], pA[kk], oacc[0][dt]);
    exps(sB, pB);
    read_v(j, 1, vb);
    interleave();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) oacc[0][dt] = mfma32(vb[kk][dt], pB[kk], oacc[0][dt]);
  };

  // ---- ring: tile j is requested DEPTH iterations before it is used ----
#pragma unroll
  for (int j = 0; j < DEPTH; ++j)
    if (j < ntiles) issue(j);
  for (int j = 0; j < ntiles; ++j) {
    // this wave's loads of tile j have landed once at most the loads of the younger tiles are
    // outstanding; near the end fewer tiles are in flight, so the count shrinks
    const int younger = min(DEPTH - 1, ntiles - 1 - j);
    if (younger <= 0) wait_vm<0>();
    else if (younger == 1) wait_vm<(DEPTH > 1 ? 1 : 0) * 2 * LPT>();
    else if (younger == 2) wait_vm<(DEPTH > 2 ? 2 : 0) * 2 * LPT>();
    else if (younger == 3) wait_vm<(DEPTH > 3 ? 3 : 0) * 2 * LPT>();
    else if (younger == 4) wait_vm<(DEPTH > 4 ? 4 : 0) * 2 * LPT>();
    else if (younger == 5) wait_vm<(DEPTH > 5 ? 5 : 0) * 2 * LPT>();
    else wait_vm<(DEPTH > 6 ? 6 : 0) * 2 * LPT>();
    __syncthreads();                            // every wave's share of tile j is in LDS; tile j-1 is no longer read
    if (j + DEPTH < ntiles) issue(j + DEPTH);   // into the stage tile j-1 just left
    if constexpr (SUB == 2 && RT == 1 && NTG == 1) {
      if (wave_rows) compute_pair(j);
    } else {
      compute(j);
    }
  }

  // With two token slices per tile, the two waves that share a row group merge their states
  // through LDS (the ring is idle now), so a workgroup leaves one partial per row and chunk.
  if constexpr (NTG == 2) {
    static_assert(RT == 1, "the slice merge is written for one row tile per wave");
    constexpr int kStateFloats = 66;             // m, l, O[4][16] of one lane
    float* xch = reinterpret_cast<float*>(smem) + rg * (kStateFloats * 64);
    __syncthreads();                             // nobody reads tiles any more
    if (tg == 1 && wave_rows) {
      xch[lane] = m[0];
      xch[64 + lane] = l[0];
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) xch[(2 + 16 * dt + i) * 64 + lane] = oacc[0][dt][i];
    }
    __syncthreads();
    if (tg == 1) return;
    if (wave_rows) {
      const float m1 = xch[lane], l1 = xch[64 + lane];
      const float mn = fmaxf(m[0], m1);
      const float a0 = __builtin_amdgcn_exp2f(m[0] - mn), a1 = __builtin_amdgcn_exp2f(m1 - mn);
      l[0] = l[0] * a0 + l1 * a1;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[0][dt][i] = oacc[0][dt][i] * a0 + xch[(2 + 16 * dt + i) * 64 + lane] * a1;
      m[0] = mn;
    }
  }
  if (!wave_rows) return;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const float lt = l[rt] + __shfl_xor(l[rt], 32, 64);
    if (!row_ok[rt]) continue;
    const size_t grow = static_cast<size_t>(w0 + iw[rt]) * p.n_q_heads + kvh * p.g + hq[rt];
    float* dst = p.ws + (grow * p.ns + slot) * kPartialFloats;
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

// token slices per tile for a given row count: two up to 128 rows (4 row groups x 2 slices), one above
__device__ __forceinline__ int tokens_split(int rows) { return rows <= 128 ? 2 : 1; }

// Layout of the work list (ints): [0] = number of items, or -1 when the list overflowed;
// [kListItems + 2i], [+ 2i + 1] = (sequence, partial slot) of item i; [kListShift + b] = s_b: sequence
// b is cut into pieces of chunk_tok >> s_b tokens, piece k covers tokens from k (chunk_tok >> s_b)
// on and leaves partial k.
constexpr int kMaxListSeqs = 512;
constexpr int kMaxListItems = 1024;
constexpr int kListItems = 2;
constexpr int kListShift = kListItems + 2 * kMaxListItems;
constexpr int kListInts = kListShift + kMaxListSeqs;
constexpr int kMaxShift = 2;

// One piece of work, 8 waves x 32 rows: tokens [slot * len, (slot + 1) * len) of one (sequence, KV head, row block).
__device__ __forceinline__ void verify_item(const VerifyParams& p, char* smem, int b, int kvh, int row0, int slot, int len) {
  const int w0 = p.cu_win[b], w = p.cu_win[b + 1] - w0;
  if (row0 >= w * p.g) return;
  int c0 = p.cu_ctx[b];
  const int N = p.cu_ctx[b + 1] - c0;
  const int t_begin = slot * len;
  if (t_begin >= min(N + w, p.tok_hi)) return;
  // ring: token t of this chunk is row ring_slot[b] * chunk_tok + (t - t_begin) of the staging buffers
  if (p.ring_slot) c0 = p.ring_slot[b] * p.chunk_tok - t_begin;
  if (tokens_split(min(256, w * p.g - row0)) == 2) verify_body<2, 1, 1>(p, smem, kvh, slot, t_begin, len, w0, w, c0, N, row0);
  else verify_body<1, 1, 2>(p, smem, kvh, slot, t_begin, len, w0, w, c0, N, row0);
}

// Grid: (chunk, KV head x row block, sequence); chunks past a sequence's end exit.
__global__ __launch_bounds__(512) void verify_kernel(VerifyParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  verify_item(p, smem, p.seq0 + blockIdx.z, blockIdx.y / p.nrb, (blockIdx.y % p.nrb) * 256, p.chunk0 + blockIdx.x, p.chunk_tok);
}

// Launches with a work list: one workgroup per CU, and every workgroup takes (piece, KV head, row
// block) triples off a queue - the counter list[1], zeroed by the kernel that wrote the list -
// until the queue is empty.  The hardware hands the workgroups of a grid out strictly in order,
// each to the next shader engine in a fixed rotation, so with pieces of unequal length a grid of one
// workgroup per piece leaves CUs idle behind a workgroup that waits for its engine (measured on the
// ragged 32-sequence batch: 150 us of 1050 idle per CU).
__global__ __launch_bounds__(512) void verify_queue_kernel(VerifyParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int taken;
  const int listed = p.list[0];        // -1: walk every (sequence, chunk) of the launch instead (all s_b are 0 then)
  const int per_piece = p.n_kv_heads * p.nrb;
  const int count = (listed >= 0 ? listed : p.list_seqs * p.list_chunks) * per_piece;
  for (;;) {
    if (threadIdx.x == 0) taken = atomicAdd(p.list + 1, 1);
    __syncthreads();
    const int q = taken;
    if (q >= count) break;             // every workgroup gets here: the counter only grows
    const int it = q / per_piece, x = q % per_piece;
    int b, slot, len = p.chunk_tok;
    if (listed >= 0) {
      b = p.list[kListItems + 2 * it];
      slot = p.list[kListItems + 2 * it + 1];
      len >>= p.list[kListShift + b];
    } else {
      b = p.seq0 + it / p.list_chunks;
      slot = p.chunk0 + it % p.list_chunks;
    }
    verify_item(p, smem, b, x / p.nrb, (x % p.nrb) * 256, slot, len);
    __syncthreads();                   // the next piece reuses the ring, and thread 0 `taken`
  }
}

// Ragged batches.  A grid over (chunk, head, sequence) is mostly empty workgroups when lengths
// differ, each of which still waits for a whole CU (the ring takes the LDS), and a workgroup's time
// is its tokens times the cost of its row count: about twice as much per token above 128 rows,
// where the kernel is bound by the matrix cores and LDS, as below, where it is bound by HBM.  This
// kernel writes the work list of a launch:
//  - only the pieces that exist;
//  - tapered: within each of the two cost classes the sequences are ranked by the cost of one of
//    their workgroups (ties: longer first, then by index); those in the first half of the class's
//    work keep chunk_tok tokens per piece, the next three tenths get half, the rest a quarter (never
//    more pieces than a row has partial slots), so that the queue ends with short pieces;
//  - every class sorted by piece cost, costliest first, and the two classes interleaved evenly:
//    matrix-bound and HBM-bound workgroups that run side by side both run faster than among their
//    own kind (measured 380 against 420 us and 200 against 218 us per 10k-token piece).
// The cut of a sequence depends on the whole batch only, not on the sequence / token range of the
// launch, so the launches of a streamed verify and the merge agree on it.
// One workgroup of 256 threads, at most kMaxListSeqs sequences and kMaxListItems pieces (ranks by
// counting, n^2 / 256 steps).
struct ListScan {    // exclusive prefix sums over the kMaxListSeqs ranks; thread t owns ranks 2t, 2t + 1
  long long wave_sum[4];
  __device__ void run(long long v0, long long v1, long long& e0, long long& e1, long long& total) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    long long inc = v0 + v1;
    for (int off = 1; off < 64; off <<= 1) {
      const long long o = __shfl_up(inc, off, 64);
      if (lane >= off) inc += o;
    }
    __syncthreads();                 // the previous scan's sums are no longer read
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    long long base = 0;
    for (int k = 0; k < wave; ++k) base += wave_sum[k];
    e0 = base + inc - (v0 + v1);
    e1 = e0 + v0;
    total = wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
  }
};

__global__ __launch_bounds__(256) void verify_worklist_kernel(const int* cu_ctx, const int* cu_win, int n, int g, int chunk_tok,
                                                              int ns, int max_shift, int seq_begin, int seq_end, int chunk0,
                                                              int tok_hi, int* list) {
  __shared__ unsigned long long key[kMaxListSeqs];
  __shared__ int total_of[kMaxListSeqs], work_of[kMaxListSeqs];       // by sequence
  __shared__ bool heavy_of[kMaxListSeqs];
  __shared__ int seq_of_rank[kMaxListSeqs];
  __shared__ ListScan scan;
  const int tid = threadIdx.x;
  for (int i = tid; i < kMaxListSeqs; i += 256) {
    seq_of_rank[i] = -1;
    if (i >= n) continue;
    const int w = cu_win[i + 1] - cu_win[i];
    const int total = w == 0 ? 0 : cu_ctx[i + 1] - cu_ctx[i] + w;     // a sequence without a window has no work
    const unsigned factor = min(w * g, 256) > 128 ? 2u : 1u;
    const unsigned per_wg = static_cast<unsigned>(min(total, chunk_tok)) >> 6;   // < 2^25
    // cost of one workgroup (26 bits) | length / 64 (25 bits) | reversed index (13-bit field)
    key[i] = (static_cast<unsigned long long>(per_wg * factor) << 38) | (static_cast<unsigned long long>(static_cast<unsigned>(total) >> 6) << 13) |
             static_cast<unsigned long long>(kMaxListSeqs - 1 - i);
    total_of[i] = total;
    work_of[i] = static_cast<int>((static_cast<unsigned>(total) >> 6) * factor);
    heavy_of[i] = factor > 1;
  }
  __syncthreads();
  for (int i = tid; i < n; i += 256) {
    const unsigned long long mine = key[i];
    int rank = 0;
    for (int j = 0; j < n; ++j) rank += key[j] > mine ? 1 : 0;
    seq_of_rank[rank] = i;
  }
  __syncthreads();
  // the cut of every sequence, from the share of its class's work that is ranked before it
  const int r0 = 2 * tid, r1 = 2 * tid + 1;
  const int b0 = seq_of_rank[r0], b1 = seq_of_rank[r1];
  const bool heavy0 = b0 >= 0 && heavy_of[b0], heavy1 = b1 >= 0 && heavy_of[b1];
  long long hb0, hb1, heavy_total, lb0, lb1, light_total;
  scan.run(heavy0 ? work_of[b0] : 0, heavy1 ? work_of[b1] : 0, hb0, hb1, heavy_total);
  scan.run(b0 >= 0 && !heavy0 ? work_of[b0] : 0, b1 >= 0 && !heavy1 ? work_of[b1] : 0, lb0, lb1, light_total);
  auto cut = [&](int b, long long before, long long class_total) {
    if (b < 0) return 0;
    int s = before * 10 < class_total * 5 ? 0 : before * 10 < class_total * 8 ? 1 : 2;
    s = min(s, max_shift);
    while (s > 0 && (total_of[b] + (chunk_tok >> s) - 1) / (chunk_tok >> s) > ns) --s;
    return s;
  };
  const int s0 = cut(b0, heavy0 ? hb0 : lb0, heavy0 ? heavy_total : light_total);
  const int s1 = cut(b1, heavy1 ? hb1 : lb1, heavy1 ? heavy_total : light_total);
  // pieces: of the whole batch (does the list hold them?) and of this launch's range
  auto pieces = [&](int b, int s, bool ranged) {
    if (b < 0) return 0;
    const int len = chunk_tok >> s;
    if (!ranged) return (total_of[b] + len - 1) / len;
    if (b < seq_begin || b >= seq_end) return 0;
    const int hi = min(total_of[b], tok_hi);
    return max(0, (hi + len - 1) / len - (chunk0 << s));
  };
  long long e0, e1, all_pieces;
  scan.run(pieces(b0, s0, false), pieces(b1, s1, false), e0, e1, all_pieces);
  const bool overflow = all_pieces > kMaxListItems;
  const int c0 = pieces(b0, s0, true), c1 = pieces(b1, s1, true);
  long long launch_pieces;
  scan.run(c0, c1, e0, e1, launch_pieces);
  if (b0 >= 0) list[kListShift + b0] = overflow ? 0 : s0;
  if (b1 >= 0) list[kListShift + b1] = overflow ? 0 : s1;
  if (tid == 0) {
    list[0] = overflow ? -1 : static_cast<int>(launch_pieces);
    list[1] = 0;
  }
  if (overflow) return;
  // the pieces of this launch with their cost (tokens x row factor) ...
  __shared__ unsigned long long piece_key[kMaxListItems];
  __shared__ unsigned piece_pos[kMaxListItems];
  __shared__ int piece_seq[kMaxListItems], piece_slot[kMaxListItems];
  auto emit = [&](int b, int s, int first, int cnt) {
    if (b < 0) return;
    const int len = chunk_tok >> s;
    const unsigned factor = heavy_of[b] ? 2u : 1u;
    const int hi = min(total_of[b], tok_hi);
    for (int c = 0; c < cnt; ++c) {
      const int slot = (chunk0 << s) + c;
      const unsigned tokens = static_cast<unsigned>(min(len, hi - slot * len));
      piece_seq[first + c] = b;
      piece_slot[first + c] = slot;
      // class (1 bit) | cost (26 bits) | reversed position (12 bits)
      piece_key[first + c] = (static_cast<unsigned long long>(factor > 1 ? 1 : 0) << 63) | (static_cast<unsigned long long>(tokens * factor) << 12) |
                             static_cast<unsigned>(kMaxListItems - 1 - (first + c));
    }
  };
  emit(b0, s0, static_cast<int>(e0), c0);
  emit(b1, s1, static_cast<int>(e1), c1);
  __syncthreads();
  // ... ranked inside their class (k of n_c, costliest first) and placed at (k + 1/2) / n_c of the queue
  const int m = static_cast<int>(launch_pieces);
  for (int i = tid; i < m; i += 256) {
    const unsigned long long mine = piece_key[i];
    int k = 0, nc = 0;
#pragma unroll 8
    for (int j = 0; j < m; ++j) {
      const unsigned long long other = piece_key[j];
      const bool same = ((other ^ mine) >> 63) == 0;
      nc += same ? 1 : 0;
      k += same && other > mine ? 1 : 0;
    }
    // 20-bit position, then the heavier class first, then the index: unique keys, smallest first
    piece_pos[i] = (static_cast<unsigned>((static_cast<unsigned long long>(2 * k + 1) << 19) / static_cast<unsigned>(nc)) << 11) |
                   ((mine >> 63) != 0 ? 0u : 1u << 10) | static_cast<unsigned>(i & 1023);
  }
  __syncthreads();
  for (int i = tid; i < m; i += 256) {
    const unsigned mine = piece_pos[i];
    int rank = 0;
#pragma unroll 8
    for (int j = 0; j < m; ++j) rank += piece_pos[j] < mine ? 1 : 0;
    list[kListItems + 2 * rank] = piece_seq[i];
    list[kListItems + 2 * rank + 1] = piece_slot[i];
  }
}

struct VerifyMergeParams {
  const float* ws;
  uint16_t* out;
  float* lse;
  const int* cu_ctx;
  const int* cu_win;
  int n_seqs, n_q_heads, g, ns, chunk_tok;
  const int* list;     // work list of a ragged batch (its per-sequence cuts), or nullptr
};

// One workgroup of 256 threads per window row and 8 query heads: thread (half, d) merges channel d
// of 4 heads, with the partials of all four requested before any is consumed - the kernel is pure
// latency, so the fewer, fatter workgroups finish in one resident round.
constexpr int kMergeHeads = 4;

__global__ __launch_bounds__(256) void verify_merge_kernel(VerifyMergeParams p) {
  const int row = blockIdx.y, d = threadIdx.x & 127;
  const int h0 = (blockIdx.x * 2 + (threadIdx.x >> 7)) * kMergeHeads;
  if (h0 >= p.n_q_heads) return;
  int b = 0;                                   // the sequence that owns this window row: last b with cu_win[b] <= row
  for (int hi = p.n_seqs; hi - b > 1;) {
    const int mid = (b + hi) >> 1;
    if (p.cu_win[mid] <= row) b = mid; else hi = mid;
  }
  const int w = p.cu_win[b + 1] - p.cu_win[b];
  const int total = (p.cu_ctx[b + 1] - p.cu_ctx[b]) + w;
  const int nsl = ceil_div_dev(total, p.list ? p.chunk_tok >> p.list[kListShift + b] : p.chunk_tok);
  float mm[kMergeHeads], acc[kMergeHeads], lsum[kMergeHeads];
#pragma unroll
  for (int k = 0; k < kMergeHeads; ++k) { mm[k] = -INFINITY; acc[k] = 0.f; lsum[k] = 0.f; }
  for (int s0 = 0; s0 < nsl; s0 += 4) {
    float m4[kMergeHeads][4], l4[kMergeHeads][4], o4[kMergeHeads][4];
#pragma unroll
    for (int k = 0; k < kMergeHeads; ++k) {
      const int h = min(h0 + k, p.n_q_heads - 1);
      const float* base = p.ws + (static_cast<size_t>(row) * p.n_q_heads + h) * p.ns * kPartialFloats;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int s = min(s0 + i, nsl - 1);
        const float* pp = base + static_cast<size_t>(s) * kPartialFloats;
        m4[k][i] = s0 + i < nsl ? pp[0] : -INFINITY;
        l4[k][i] = pp[1];
        o4[k][i] = pp[2 + d];
      }
    }
#pragma unroll
    for (int k = 0; k < kMergeHeads; ++k) {
      float mn = mm[k];
#pragma unroll
      for (int i = 0; i < 4; ++i) mn = fmaxf(mn, m4[k][i]);
      const float alpha = exp2_diff(mm[k], mn);
      acc[k] *= alpha;
      lsum[k] *= alpha;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float a = exp2_diff(m4[k][i], mn);
        acc[k] = fmaf(a, o4[k][i], acc[k]);
        lsum[k] = fmaf(a, l4[k][i], lsum[k]);
      }
      mm[k] = mn;
    }
  }
#pragma unroll
  for (int k = 0; k < kMergeHeads; ++k) {
    const int h = h0 + k;
    if (h >= p.n_q_heads) break;
    const float o = lsum[k] > 0.f ? acc[k] / lsum[k] : 0.f;
    p.out[(static_cast<size_t>(row) * p.n_q_heads + h) * kHeadDim + d] = static_cast<uint16_t>(float_to_bf16_bits(o));
    if (p.lse && d == 0) p.lse[static_cast<size_t>(row) * p.n_q_heads + h] = lsum[k] > 0.f ? (mm[k] + log2f(lsum[k])) * kLn2 : -INFINITY;
  }
}

struct VerifyPlan {
  int chunk_tok, nchunk, ns;
  int list_items;   // > 0: ragged batch of few enough sequences; launches run from a work list with room for this many items
  int max_shift;    // shortest piece of the list: chunk_tok >> max_shift
};

static VerifyPlan make_verify_plan(const vc_full_kv* kv) {
  VerifyPlan pl{};
  const int lists = kv->n_seqs * kv->n_kv_heads;
  const int total_max = kv->max_ctx + kv->max_win;
  int64_t sum = static_cast<int64_t>(kv->sum_ctx > 0 ? kv->sum_ctx + static_cast<int64_t>(kv->n_seqs) * kv->max_win
                                                      : static_cast<int64_t>(total_max) * kv->n_seqs) * kv->n_kv_heads;
  // One workgroup fills a CU (its ring takes the LDS), so equal chunks of a uniform batch want
  // exactly one round of 256; a ragged batch leaves remainders and balances better with shorter
  // chunks (measured: 256 against 512 workgroups at config-2 shape 652 vs 694 us; the ragged
  // config-4 batch 1470 us with 256, 1241 us with 768).
  const bool uniform = kv->sum_ctx <= 0 || static_cast<int64_t>(kv->max_ctx) * kv->n_seqs * 10 <= static_cast<int64_t>(kv->sum_ctx) * 11;
  const int target = tunable(kTunVerifyWgs, uniform ? 256 : 768, 1, 1 << 20);
  int64_t per = ceil_div64(sum > 0 ? sum : 1, target);
  const int min_tok = tunable(kTunVerifyMinTok, 1024, 128, 1 << 24);
  if (per < min_tok) per = min_tok;
  if (per > total_max) per = total_max > 0 ? total_max : 1;
  per = ceil_div64(per, uniform ? 128 : 128 << kMaxShift) * (uniform ? 128 : 128 << kMaxShift);
  if (kv->chunk_tokens > 0) per = kv->chunk_tokens;
  pl.chunk_tok = static_cast<int>(per);
  pl.nchunk = ceil_div(total_max > 0 ? total_max : 1, pl.chunk_tok);
  pl.ns = pl.nchunk;
  pl.list_items = 0;
  pl.max_shift = 0;
  // The list costs a launch of its own (about 15 us), which pays from a few hundred microseconds of
  // work on: 2^21 token-heads are 1 GB of K and V.  (VC_VERIFY_LIST_MIN = 0 sends every ragged batch
  // through the list: tests.)
  const int64_t list_min = tunable(kTunVerifyListMin, 1 << 21, 0, 1 << 30);
  const bool fits = static_cast<int64_t>(kv->n_seqs) * pl.nchunk * kv->n_kv_heads * ceil_div(kv->max_win * (kv->n_q_heads / kv->n_kv_heads), 256) < (1 << 30);
  if (!uniform && sum >= list_min && fits && kv->ring_slots == 0 && kv->n_seqs >= 2 && kv->n_seqs <= kMaxListSeqs &&
      tunable(kTunVerifyWorklist, 1, 0, 1) != 0) {
    while (pl.max_shift < kMaxShift && (pl.chunk_tok >> (pl.max_shift + 1)) % 128 == 0) ++pl.max_shift;   // pieces stay whole tiles
    pl.max_shift = tunable(kTunVerifyTaper, pl.max_shift, 0, pl.max_shift);
    // every sequence has at most one partial piece: sum / shortest piece + n bounds the list
    const int64_t bound = (static_cast<int64_t>(kv->sum_ctx) + static_cast<int64_t>(kv->n_seqs) * kv->max_win) / (pl.chunk_tok >> pl.max_shift) + kv->n_seqs;
    if (bound <= kMaxListItems) pl.list_items = static_cast<int>(bound);
  }
  (void)lists;
  return pl;
}

// the partials come first in the workspace, the work list of a ragged launch after them
static size_t partial_bytes(const vc_full_kv* kv, int total_win, const VerifyPlan& pl) {
  return static_cast<size_t>(total_win > 0 ? total_win : 1) * kv->n_q_heads * pl.ns * kPartialFloats * sizeof(float);
}

static vc_status check_full(const vc_full_kv* kv, const char* who) {
  VC_REQUIRE(kv != nullptr, VC_ERR_INVALID_ARG, "%s: kv is NULL", who);
  VC_REQUIRE(kv->head_dim == kHeadDim, VC_ERR_UNSUPPORTED, "%s: head_dim %d (only 128)", who, kv->head_dim);
  VC_REQUIRE(kv->n_seqs >= 0 && kv->n_q_heads > 0 && kv->n_kv_heads > 0, VC_ERR_INVALID_ARG, "%s: bad sizes", who);
  VC_REQUIRE(kv->n_q_heads % kv->n_kv_heads == 0, VC_ERR_INVALID_ARG, "%s: n_q_heads %d not a multiple of n_kv_heads %d",
             who, kv->n_q_heads, kv->n_kv_heads);
  VC_REQUIRE(kv->max_ctx >= 0 && kv->max_win >= 0 && kv->sum_ctx >= 0, VC_ERR_INVALID_ARG, "%s: negative count", who);
  VC_REQUIRE(kv->chunk_tokens >= 0 && kv->chunk_tokens % 128 == 0, VC_ERR_INVALID_ARG,
             "%s: chunk_tokens %d is not a multiple of 128", who, kv->chunk_tokens);
  VC_REQUIRE(static_cast<int64_t>(kv->max_win) * (kv->n_q_heads / kv->n_kv_heads) <= 4096, VC_ERR_UNSUPPORTED,
             "%s: window %d x GQA ratio %d exceeds 4096 rows", who, kv->max_win, kv->n_q_heads / kv->n_kv_heads);
  VC_REQUIRE(kv->n_q_heads / kv->n_kv_heads <= 256, VC_ERR_UNSUPPORTED, "%s: GQA ratio above 256", who);
  VC_REQUIRE(kv->n_seqs <= 65535 && kv->n_kv_heads <= 65535 && kv->n_q_heads <= 65535, VC_ERR_UNSUPPORTED,
             "%s: batch too large for one launch", who);
  VC_REQUIRE(kv->ring_slots >= 0, VC_ERR_INVALID_ARG, "%s: ring_slots %d", who, kv->ring_slots);
  if (kv->ring_slots > 0) {
    VC_REQUIRE(kv->chunk_tokens > 0, VC_ERR_INVALID_ARG, "%s: a staging ring needs chunk_tokens (the length of a slot)", who);
    VC_REQUIRE(kv->ring_slot != nullptr, VC_ERR_INVALID_ARG, "%s: a staging ring needs ring_slot", who);
    VC_REQUIRE(static_cast<int64_t>(kv->ring_slots) * kv->chunk_tokens < (1ll << 31), VC_ERR_UNSUPPORTED, "%s: ring of %d x %d rows", who,
               kv->ring_slots, kv->chunk_tokens);
  }
  VC_REQUIRE(kv->cu_ctx != nullptr, VC_ERR_INVALID_ARG, "%s: cu_ctx is NULL", who);
  VC_REQUIRE(kv->max_ctx == 0 || (kv->k && kv->v), VC_ERR_INVALID_ARG, "%s: k or v is NULL", who);
  VC_REQUIRE(aligned16(kv->k) && aligned16(kv->v), VC_ERR_INVALID_ARG, "%s: k/v not 16-byte aligned", who);
  return VC_OK;
}

// the K/V ring needs more dynamic LDS than the default limit: a per-device function attribute
vc_status verify_init_device() {
  VC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(verify_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             kVerifyLds));
  VC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(verify_queue_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             kVerifyLds));
  return VC_OK;
}

}  // namespace vc

using namespace vc;

extern "C" vc_status vc_verify_workspace_bytes(const vc_full_kv* kv, int32_t total_win, size_t* bytes) {
  vc_status st = check_full(kv, "vc_verify_workspace_bytes");
  if (st != VC_OK) return st;
  VC_REQUIRE(bytes != nullptr && total_win >= 0, VC_ERR_INVALID_ARG, "vc_verify_workspace_bytes: bad arguments");
  const VerifyPlan pl = make_verify_plan(kv);
  *bytes = partial_bytes(kv, total_win, pl) + (pl.list_items > 0 ? static_cast<size_t>(kListInts) * sizeof(int) : 0);
  return VC_OK;
}

extern "C" vc_status vc_verify_plan(const vc_full_kv* kv, int32_t* chunk_tokens, int32_t* n_chunks) {
  vc_status st = check_full(kv, "vc_verify_plan");
  if (st != VC_OK) return st;
  const VerifyPlan pl = make_verify_plan(kv);
  if (chunk_tokens) *chunk_tokens = pl.chunk_tok;
  if (n_chunks) *n_chunks = pl.nchunk;
  return VC_OK;
}

static vc_status check_verify_call(vc_ctx* ctx, const vc_full_kv* kv, int32_t total_win, const void* workspace,
                                   size_t workspace_bytes, const char* who) {
  VC_REQUIRE(ctx != nullptr, VC_ERR_INVALID_ARG, "%s: ctx is NULL", who);
  vc_status stt = check_full(kv, who);
  if (stt != VC_OK) return stt;
  VC_REQUIRE(total_win >= 0 && total_win <= 65535, total_win < 0 ? VC_ERR_INVALID_ARG : VC_ERR_UNSUPPORTED,
             "%s: total_win %d", who, total_win);
  size_t need = 0;
  vc_verify_workspace_bytes(kv, total_win, &need);
  VC_REQUIRE(workspace != nullptr && workspace_bytes >= need, VC_ERR_WORKSPACE, "%s: workspace %zu bytes, need %zu", who,
             workspace_bytes, need);
  VC_REQUIRE(aligned16(workspace), VC_ERR_INVALID_ARG, "%s: workspace not 16-byte aligned", who);
  return VC_OK;
}

extern "C" vc_status vc_verify_attn_range(vc_ctx* ctx, const vc_full_kv* kv, const void* q_win, const void* k_win,
                                          const void* v_win, const int32_t* cu_win, int32_t total_win,
                                          float softmax_scale, int32_t seq_begin, int32_t seq_end, int32_t tok_begin,
                                          int32_t tok_end, void* workspace, size_t workspace_bytes, void* stream) {
  vc_status stt = check_verify_call(ctx, kv, total_win, workspace, workspace_bytes, "vc_verify_attn_range");
  if (stt != VC_OK) return stt;
  VC_REQUIRE(seq_begin >= 0 && seq_begin <= seq_end && seq_end <= kv->n_seqs, VC_ERR_INVALID_ARG,
             "vc_verify_attn_range: sequences [%d, %d) of %d", seq_begin, seq_end, kv->n_seqs);
  VC_REQUIRE(tok_begin >= 0 && tok_begin <= tok_end, VC_ERR_INVALID_ARG, "vc_verify_attn_range: tokens [%d, %d)", tok_begin, tok_end);
  if (seq_begin == seq_end || tok_begin == tok_end || total_win == 0 || kv->max_win == 0) return VC_OK;
  VC_REQUIRE(q_win && k_win && v_win && cu_win, VC_ERR_INVALID_ARG, "vc_verify_attn_range: NULL pointer");
  VC_REQUIRE(aligned16(q_win) && aligned16(k_win) && aligned16(v_win), VC_ERR_INVALID_ARG,
             "vc_verify_attn_range: window tensors not 16-byte aligned");
  const VerifyPlan pl = make_verify_plan(kv);
  const int total_max = kv->max_ctx + kv->max_win;
  VC_REQUIRE(tok_begin % pl.chunk_tok == 0, VC_ERR_INVALID_ARG, "vc_verify_attn_range: tok_begin %d is not a multiple of the chunk length %d",
             tok_begin, pl.chunk_tok);
  VC_REQUIRE(tok_end % pl.chunk_tok == 0 || tok_end >= total_max, VC_ERR_INVALID_ARG,
             "vc_verify_attn_range: tok_end %d is neither a multiple of the chunk length %d nor past the end (%d)", tok_end,
             pl.chunk_tok, total_max);
  if (tok_begin >= total_max) return VC_OK;
  if (kv->ring_slots > 0) {
    // one chunk per call: a slot holds no more.  "Past the end" (the last piece of a sequence, which takes its
    // window tokens along) means the rest of that one chunk.
    VC_REQUIRE(tok_end - tok_begin <= pl.chunk_tok || tok_end >= total_max, VC_ERR_INVALID_ARG,
               "vc_verify_attn_range: with a staging ring a call covers one chunk of %d tokens (got [%d, %d))", pl.chunk_tok,
               tok_begin, tok_end);
    if (tok_end - tok_begin > pl.chunk_tok) tok_end = tok_begin + pl.chunk_tok;
  }

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
  vp.seq0 = seq_begin;
  vp.chunk0 = tok_begin / pl.chunk_tok;
  vp.tok_hi = tok_end;
  vp.scale_log2e = softmax_scale * kLog2e;
  vp.ring_slot = kv->ring_slots > 0 ? kv->ring_slot : nullptr;
  const int hi = tok_end < total_max ? tok_end : total_max;
  const int nchunk = ceil_div(hi, pl.chunk_tok) - vp.chunk0;
  vp.nrb = ceil_div(kv->max_win * vp.g, 256);
  dim3 grid(nchunk, kv->n_kv_heads * vp.nrb, seq_end - seq_begin);
  if (pl.list_items > 0) {
    int* list = reinterpret_cast<int*>(static_cast<char*>(workspace) + partial_bytes(kv, total_win, pl));
    hipLaunchKernelGGL(verify_worklist_kernel, dim3(1), dim3(256), 0, st, kv->cu_ctx, cu_win, kv->n_seqs, vp.g, pl.chunk_tok, pl.ns,
                       pl.max_shift, seq_begin, seq_end, vp.chunk0, tok_end, list);
    vp.list = list;
    vp.list_seqs = seq_end - seq_begin;
    vp.list_chunks = nchunk;
    // workgroups of the queue launch: one per CU (each fills the LDS of one)
    grid = dim3(tunable(kTunVerifyQueueWgs, ctx->n_cu > 0 ? ctx->n_cu : 256, 1, 1 << 16), 1, 1);
  }
  // (A variant with 64 rows per wave halves the LDS traffic per flop but leaves one wave per SIMD;
  // it measured slower at every window - 1781 vs 1363 us at w = 64, config-2 shape - and was dropped.)
  mark_begin(ctx, st);
  if (vp.list) hipLaunchKernelGGL(verify_queue_kernel, grid, dim3(512), kVerifyLds, st, vp);
  else hipLaunchKernelGGL(verify_kernel, grid, dim3(512), kVerifyLds, st, vp);
  mark_end(ctx, st);
  VC_HIP(hipGetLastError());
  return VC_OK;
}

extern "C" vc_status vc_verify_finish(vc_ctx* ctx, const vc_full_kv* kv, const int32_t* cu_win, int32_t total_win,
                                      void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  vc_status stt = check_verify_call(ctx, kv, total_win, workspace, workspace_bytes, "vc_verify_finish");
  if (stt != VC_OK) return stt;
  if (kv->n_seqs == 0 || total_win == 0 || kv->max_win == 0) return VC_OK;
  VC_REQUIRE(cu_win && out, VC_ERR_INVALID_ARG, "vc_verify_finish: NULL pointer");
  VC_REQUIRE(aligned16(out), VC_ERR_INVALID_ARG, "vc_verify_finish: out not 16-byte aligned");
  const VerifyPlan pl = make_verify_plan(kv);
  VerifyMergeParams mp{};
  mp.ws = static_cast<const float*>(workspace);
  mp.out = static_cast<uint16_t*>(out);
  mp.lse = lse;
  mp.cu_ctx = kv->cu_ctx;
  mp.cu_win = cu_win;
  mp.n_seqs = kv->n_seqs; mp.n_q_heads = kv->n_q_heads; mp.g = kv->n_q_heads / kv->n_kv_heads; mp.ns = pl.ns;
  mp.chunk_tok = pl.chunk_tok;
  mp.list = pl.list_items > 0 ? reinterpret_cast<const int*>(static_cast<const char*>(workspace) + partial_bytes(kv, total_win, pl)) : nullptr;
  hipLaunchKernelGGL(verify_merge_kernel, dim3(ceil_div(kv->n_q_heads, 2 * kMergeHeads), total_win), dim3(256), 0,
                     static_cast<hipStream_t>(stream), mp);
  VC_HIP(hipGetLastError());
  return VC_OK;
}

extern "C" vc_status vc_verify_attn(vc_ctx* ctx, const vc_full_kv* kv, const void* q_win, const void* k_win,
                                    const void* v_win, const int32_t* cu_win, int32_t total_win, float softmax_scale,
                                    void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  vc_status stt = check_verify_call(ctx, kv, total_win, workspace, workspace_bytes, "vc_verify_attn");
  if (stt != VC_OK) return stt;
  if (kv->n_seqs == 0 || total_win == 0 || kv->max_win == 0) return VC_OK;
  VC_REQUIRE(out != nullptr, VC_ERR_INVALID_ARG, "vc_verify_attn: out is NULL");
  VC_REQUIRE(kv->ring_slots == 0, VC_ERR_INVALID_ARG,
             "vc_verify_attn: a staging ring holds one chunk per sequence at a time; use vc_verify_attn_range chunk by chunk");
  stt = vc_verify_attn_range(ctx, kv, q_win, k_win, v_win, cu_win, total_win, softmax_scale, 0, kv->n_seqs, 0,
                             kv->max_ctx + kv->max_win, workspace, workspace_bytes, stream);
  if (stt != VC_OK) return stt;
  return vc_verify_finish(ctx, kv, cu_win, total_win, out, lse, workspace, workspace_bytes, stream);
}
