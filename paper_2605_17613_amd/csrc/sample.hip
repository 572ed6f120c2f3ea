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
  double inv_t_log2e;   // log2(e) / T: exponentials are taken as powers of two
};

// 2^y in double precision for y <= 0, about 1.5 ulp: y = k/256 + r with |r| <= 1/512, so
// 2^y = 2^(k >> 8) * 2^((k & 255)/256) * e^(r ln 2): a 256-entry table and a degree-4 polynomial,
// free of branches and of the slower conversion / rounding / scaling instructions, so that the
// exponentials of a thread's 32 logits overlap (the statistics pass is bound by these operations,
// not by HBM: each one dropped shows in its time).  The kernels that take one exponential per logit
// keep the table in LDS (exp2_table_to_lds); y below -1020, -infinity and NaN give 2^-1020, which
// vanishes next to the row maximum's term of 1.
constexpr int kExp2Entries = 256;
__device__ const double kExp2Frac[kExp2Entries] = {
    1.0, 1.0027112750502025, 1.0054299011128027, 1.0081558981184175,
    1.0108892860517005, 1.0136300849514894, 1.016378314910953, 1.019133996077738,
    1.0218971486541166, 1.0246677928971357, 1.0274459491187637, 1.030231637686041,
    1.0330248790212284, 1.0358256936019572, 1.0386341019613787, 1.041450124688316,
    1.0442737824274138, 1.0471050958792898, 1.0499440858006872, 1.0527907730046264,
    1.0556451783605572, 1.0585073227945128, 1.061377227289262, 1.0642549128844645,
    1.0671404006768237, 1.0700337118202419, 1.0729348675259756, 1.075843889062791,
    1.0787607977571199, 1.0816856149932152, 1.0846183622133092, 1.0875590609177697,
    1.0905077326652577, 1.0934643990728858, 1.0964290818163769, 1.099401802630222,
    1.102382583307841, 1.1053714457017412, 1.1083684117236787, 1.1113735033448175,
    1.1143867425958924, 1.1174081515673693, 1.1204377524096067, 1.12347556733302,
    1.1265216186082418, 1.129575928566288, 1.1326385195987192, 1.1357094141578055,
    1.1387886347566916, 1.1418762039695616, 1.1449721444318042, 1.148076478840179,
    1.1511892299529827, 1.154310420590216, 1.1574400736337511, 1.1605782120274988,
    1.1637248587775775, 1.1668800369524817, 1.1700437696832502, 1.1732160801636373,
    1.1763969916502812, 1.1795865274628758, 1.182784710984341, 1.1859915656609938,
    1.189207115002721, 1.1924313825831512, 1.1956643920398273, 1.1989061670743806,
    1.202156731452703, 1.2054161090051239, 1.2086843236265816, 1.2119613992768012,
    1.215247359980469, 1.2185422298274085, 1.2218460329727576, 1.2251587936371455,
    1.22848053610687, 1.2318112847340759, 1.2351510639369334, 1.2384998981998165,
    1.241857812073484, 1.245224830175258, 1.2486009771892048, 1.2519862778663162,
    1.255380757024691, 1.2587844395497165, 1.2621973503942507, 1.2656195145788063,
    1.2690509571917332, 1.2724917033894028, 1.275941778396392, 1.2794012075056693,
    1.2828700160787783, 1.2863482295460256, 1.2898358734066657, 1.2933329732290895,
    1.2968395546510096, 1.3003556433796506, 1.3038812651919358, 1.3074164459346773,
    1.3109612115247644, 1.3145155879493546, 1.318079601266064, 1.3216532776031575,
    1.3252366431597413, 1.3288297242059544, 1.3324325470831615, 1.3360451382041458,
    1.339667524053303, 1.3432997311868353, 1.3469417862329458, 1.3505937158920345,
    1.3542555469368927, 1.3579273062129011, 1.3616090206382248, 1.365300717204012,
    1.3690024229745905, 1.3727141650876684, 1.3764359707545302, 1.380167867260238,
    1.383909881963832, 1.387662042298529, 1.3914243757719262, 1.3951969099662003,
    1.3989796725383112, 1.4027726912202048, 1.4065759938190154, 1.4103896082172707,
    1.4142135623730951, 1.4180478843204152, 1.4218926021691656, 1.4257477441054942,
    1.42961333839197, 1.433489413367789, 1.4373759974489824, 1.4412731191286257,
    1.4451808069770467, 1.449099089642035, 1.4530279958490526, 1.4569675544014438,
    1.460917794180647, 1.4648787441464057, 1.4688504333369818, 1.4728328908693675,
    1.4768261459394993, 1.4808302278224719, 1.4848451658727524, 1.488870989524397,
    1.4929077282912648, 1.4969554117672355, 1.5010140696264256, 1.5050837316234065,
    1.5091644275934228, 1.5132561874526098, 1.5173590411982147, 1.5214730189088146,
    1.5255981507445384, 1.529734466947287, 1.533881997840956, 1.5380407738316568,
    1.5422108254079407, 1.5463921831410214, 1.550584877685, 1.5547889397770887,
    1.559004400237837, 1.5632312899713576, 1.567469639965553, 1.5717194812923414,
    1.5759808451078865, 1.5802537626528246, 1.5845382652524937, 1.588834384317164,
    1.593142151342267, 1.597461597908627, 1.6017927556826934, 1.606135656416771,
    1.6104903319492543, 1.6148568142048607, 1.6192351351948637, 1.6236253270173289,
    1.6280274218573478, 1.632441451987275, 1.6368674497669644, 1.6413054476440063,
    1.645755478153965, 1.6502175739206177, 1.6546917676561943, 1.6591780921616162,
    1.6636765803267364, 1.6681872651305825, 1.6727101796415966, 1.6772453570178785,
    1.681792830507429, 1.6863526334483934, 1.6909247992693053, 1.6955093614893326,
    1.7001063537185235, 1.7047158096580513, 1.709337763100463, 1.713972247929926,
    1.718619298122478, 1.723278947746274, 1.7279512309618377, 1.732636182022311,
    1.7373338352737062, 1.7420442251551564, 1.746767386199169, 1.7515033530318782,
    1.7562521603732995, 1.761013843037584, 1.7657884359332727, 1.7705759740635547,
    1.7753764925265212, 1.7801900265154245, 1.785016611318935, 1.789856282321401,
    1.7947090750031072, 1.7995750249405351, 1.804454167806624, 1.809346539371032,
    1.8142521755003989, 1.8191711121586085, 1.8241033854070534, 1.8290490314048973,
    1.8340080864093424, 1.8389805867758937, 1.843966568958626, 1.8489660695104508,
    1.8539791250833855, 1.8590057724288205, 1.864046048397789, 1.8690999899412386,
    1.8741676341103, 1.8792490180565602, 1.8843441790323345, 1.8894531543909392,
    1.8945759815869656, 1.8997126981765553, 1.9048633418176741, 1.9100279502703899,
    1.9152065613971474, 1.9203992131630474, 1.925605943636125, 1.930826790987627,
    1.9360617934922943, 1.9413109895286405, 1.9465744175792332, 1.9518521162309783,
    1.9571441241754002, 1.9624504802089273, 1.9677712232331759, 1.9731063922552343,
    1.978456026387951, 1.9838201648502194, 1.9891988469672663, 1.9945921121709402};

__device__ __forceinline__ double exp2_nonpositive(double y, const double* table) {
  y = fmax(y, -1020.0);
  // adding 1.5 * 2^52 rounds 256 y to the nearest integer k and leaves k in the low word of the sum
  const double kMagic = 6755399441055744.0;
  const double t = fma(y, 256.0, kMagic);
  const int k = __double2loint(t);
  const double r = fma(t - kMagic, -0.00390625, y);
  double poly = 0.009618129107628477;            // (ln 2)^i / i!, i = 4 ... 1
  poly = fma(poly, r, 0.05550410866482158);
  poly = fma(poly, r, 0.24022650695910072);
  poly = fma(poly, r, 0.6931471805599453);
  poly = fma(poly, r, 1.0);
  const double v = table[k & (kExp2Entries - 1)] * poly;      // in [1, 2.01)
  // times 2^(k >> 8) (k <= 0, two's complement) through the exponent field, which stays positive
  return __hiloint2double(__double2hiint(v) + ((k & ~(kExp2Entries - 1)) << 12), __double2loint(v));
}
__device__ __forceinline__ double exp2_nonpositive(double y) { return exp2_nonpositive(y, kExp2Frac); }

// copy of the table in LDS for the per-logit loops (workgroups of 256 threads); the caller's next
// __syncthreads() publishes it
__device__ __forceinline__ void exp2_table_to_lds(double* table) {
  static_assert(kSampleThreads == kExp2Entries, "one table entry per thread");
  table[threadIdx.x] = kExp2Frac[threadIdx.x];
}
constexpr double kLog2e = 1.4426950408889634074;

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
  __shared__ double table[kExp2Entries];
  __shared__ float shm[4];
  exp2_table_to_lds(table);
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
    // masked (-infinity) logits are clamped to 2^-1020, which leaves the sum unchanged next to the
    // maximum's term of 1; y = (x - m) c is taken as one fused multiply-add
    const double mc = -static_cast<double>(m) * p.inv_t_log2e;
#pragma unroll
    for (int i = 0; i < kSamplePerThread; ++i)
      s += exp2_nonpositive(fma(static_cast<double>(x[i]), p.inv_t_log2e, mc), table);
  }
  s = block_sum(s, sh);
  if (threadIdx.x == 0) {
    double* dst = p.seg_stats + (static_cast<size_t>(r) * p.nseg + seg) * 2;
    dst[0] = m;
    dst[1] = s;
  }
}

// pass 2: row maximum and row sum from the segment statistics; one wave per row, lane l takes the
// segments l, l + 64, ... and the lanes are combined in a fixed tree
__global__ __launch_bounds__(256) void sample_rows_kernel(SampleParams p) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (r >= p.total_rows + p.total_win) return;
  const double* st = p.seg_stats + static_cast<size_t>(r) * p.nseg * 2;
  double M = -INFINITY;
  for (int s = lane; s < p.nseg; s += 64) M = fmax(M, st[2 * s]);
  for (int off = 32; off > 0; off >>= 1) M = fmax(M, __shfl_xor(M, off, 64));
  double S = 0.0;
  for (int s = lane; s < p.nseg; s += 64) {
    const double ms = st[2 * s];
    if (ms > -INFINITY) S += st[2 * s + 1] * exp2_nonpositive((ms - M) * p.inv_t_log2e);
  }
  for (int off = 32; off > 0; off >>= 1) S += __shfl_xor(S, off, 64);
  if (lane == 0) {
    p.row_stats[2 * r] = M;
    p.row_stats[2 * r + 1] = S;
  }
}

// probability of a logit x of a row with maximum M and sum of exponentials S
__device__ __forceinline__ double prob_of(const SampleParams& p, double M, double S, float x) {
  const double e = exp2_nonpositive((static_cast<double>(x) - M) * p.inv_t_log2e);
  return x > -INFINITY ? e / S : 0.0;
}

// pass 3: the accept tests of one sequence (one wave per sequence, one lane per drafted position,
// the first failing position wins); picks the row to re-draw from
__global__ __launch_bounds__(64) void sample_decide_kernel(SampleParams p) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int r0 = p.cu_rows[b], r1 = p.cu_rows[b + 1];
  const int w0 = p.cu_win[b], w = p.cu_win[b + 1] - w0;
  int a = w;
  for (int j0 = 0; j0 < w; j0 += 64) {
    const int j = j0 + lane;
    bool reject = false;
    if (j < w) {
      const int t = p.draft_ids[w0 + j];
      const int tr = r0 + j, dr = p.total_rows + w0 + j;
      const double pt = prob_of(p, p.row_stats[2 * tr], p.row_stats[2 * tr + 1], p.target[static_cast<size_t>(tr) * p.vocab + t]);
      const double qt = prob_of(p, p.row_stats[2 * dr], p.row_stats[2 * dr + 1], p.draft[static_cast<size_t>(w0 + j) * p.vocab + t]);
      reject = !(static_cast<double>(p.u_accept[w0 + j]) * qt < pt);
    }
    const unsigned long long mask = __ballot(reject);
    if (mask != 0) {
      a = j0 + __ffsll(static_cast<long long>(mask)) - 1;
      break;
    }
  }
  if (lane != 0) return;
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

// The row that a sequence re-draws from: pointers and statistics, read once per thread.
struct Redraw {
  const float* trow;
  const float* drow;     // nullptr: no draft row (bonus token)
  double tm, tinv, dm, dinv, c;     // row maxima, reciprocals of the sums of exponentials, log2(e) / T
  __device__ Redraw(const SampleParams& p, int tr, int dr) {
    trow = p.target + static_cast<size_t>(tr) * p.vocab;
    tm = p.row_stats[2 * tr];
    tinv = 1.0 / p.row_stats[2 * tr + 1];
    drow = nullptr;
    dm = 0.0;
    dinv = 1.0;
    if (dr >= 0) {
      drow = p.draft + static_cast<size_t>(dr - p.total_rows) * p.vocab;
      dm = p.row_stats[2 * dr];
      dinv = 1.0 / p.row_stats[2 * dr + 1];
    }
    c = p.inv_t_log2e;
  }
  // weight of a vocabulary entry with target logit xt and draft logit xd: p(v), or the positive
  // part of p(v) - q(v)
  __device__ __forceinline__ double weight(float xt, float xd, const double* table) const {
    const double et = exp2_nonpositive((static_cast<double>(xt) - tm) * c, table);
    const double pv = xt > -INFINITY ? et * tinv : 0.0;
    if (drow == nullptr) return pv;
    const double ed = exp2_nonpositive((static_cast<double>(xd) - dm) * c, table);
    const double qv = xd > -INFINITY ? ed * dinv : 0.0;
    const double d = pv - qv;
    return d > 0.0 ? d : 0.0;
  }
  __device__ __forceinline__ double weight(int v, const double* table) const {
    return weight(trow[v], drow != nullptr ? drow[v] : 0.0f, table);
  }
  // the kSamplePerThread consecutive logits from e0 on of one row (16-byte loads when the row allows
  // them); entries past the vocabulary read as -infinity, whose weight is 0
  __device__ __forceinline__ static void load_run(const float* row, int e0, int vocab, float* x) {
    if (row == nullptr) {
#pragma unroll
      for (int i = 0; i < kSamplePerThread; ++i) x[i] = -INFINITY;
      return;
    }
    const bool vec = (vocab & 3) == 0 && (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
    if (vec) {
#pragma unroll
      for (int i = 0; i < kSamplePerThread / 4; ++i) {
        float4 v = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        if (e0 + 4 * i < vocab) v = *reinterpret_cast<const float4*>(row + e0 + 4 * i);
        x[4 * i] = v.x; x[4 * i + 1] = v.y; x[4 * i + 2] = v.z; x[4 * i + 3] = v.w;
      }
    } else {
#pragma unroll
      for (int i = 0; i < kSamplePerThread; ++i) x[i] = e0 + i < vocab ? row[e0 + i] : -INFINITY;
    }
  }
};

// pass 4: segment sums of the re-draw weights (each thread sums its 32 consecutive entries in order)
__global__ __launch_bounds__(kSampleThreads) void sample_weights_kernel(SampleParams p) {
  __shared__ double sh[4];
  __shared__ double table[kExp2Entries];
  const int b = blockIdx.y, seg = blockIdx.x;
  const int tr = p.pick[2 * b], dr = p.pick[2 * b + 1];
  if (tr < 0) return;
  exp2_table_to_lds(table);
  __syncthreads();
  const Redraw row(p, tr, dr);
  const int e0 = seg * kSampleSeg + threadIdx.x * kSamplePerThread;
  float xt[kSamplePerThread], xd[kSamplePerThread];
  Redraw::load_run(row.trow, e0, p.vocab, xt);
  Redraw::load_run(row.drow, e0, p.vocab, xd);
  double s = 0.0;
#pragma unroll
  for (int i = 0; i < kSamplePerThread; ++i) s += row.weight(xt[i], xd[i], table);
  s = block_sum(s, sh);
  if (threadIdx.x == 0) p.res_sums[static_cast<size_t>(b) * p.nseg + seg] = s;
}

// pass 5: inverse CDF - the smallest v whose running sum exceeds u * total
__global__ __launch_bounds__(kSampleThreads) void sample_pick_kernel(SampleParams p) {
  constexpr int kSegCache = 512;
  __shared__ double part[kSampleThreads];
  __shared__ double table[kExp2Entries];
  __shared__ double seg_cache[kSegCache];
  __shared__ double base_sh, thr_sh;
  __shared__ int seg_sh, thread_sh;
  const int b = blockIdx.x;
  const int tr = p.pick[2 * b], dr = p.pick[2 * b + 1];
  if (tr < 0) return;
  exp2_table_to_lds(table);
  const Redraw row(p, tr, dr);
  // the segment sums go through LDS so that their loads overlap (a scan that reads them one by one
  // from global memory pays the full latency per segment)
  const double* ss_global = p.res_sums + static_cast<size_t>(b) * p.nseg;
  for (int s = threadIdx.x; s < min(p.nseg, kSegCache); s += kSampleThreads) seg_cache[s] = ss_global[s];
  __syncthreads();
  if (threadIdx.x == 0) {
    auto ss = [&](int s) { return s < kSegCache ? seg_cache[s] : ss_global[s]; };
    double total = 0.0;
    for (int s = 0; s < p.nseg; ++s) total += ss(s);
    const double thr = static_cast<double>(p.u_resample[b]) * total;
    double run = 0.0;
    int seg = p.nseg - 1;
    for (int s = 0; s < p.nseg; ++s) {
      if (run + ss(s) > thr) {
        seg = s;
        break;
      }
      run += ss(s);
    }
    if (seg == p.nseg - 1 && !(run + ss(seg) > thr)) {
      // rounding left the threshold above the last running sum: restart the last segment's search
      run = 0.0;
      for (int s = 0; s < seg; ++s) run += ss(s);
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
  {
    float xt[kSamplePerThread], xd[kSamplePerThread];
    Redraw::load_run(row.trow, e0, p.vocab, xt);
    Redraw::load_run(row.drow, e0, p.vocab, xd);
#pragma unroll
    for (int i = 0; i < kSamplePerThread; ++i) {
      w[i] = row.weight(xt[i], xd[i], table);
      s += w[i];
    }
  }
  part[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x < 64) {
    // running sums in front of every thread, by the first wave: a lane takes kPer threads' sums in
    // order, the lanes are chained by a shuffle scan; the first thread whose running sum passes the
    // threshold holds the drawn entry
    constexpr int kPer = kSampleThreads / 64;
    const int lane = threadIdx.x;
    double mine[kPer];
    double own = 0.0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      mine[i] = part[lane * kPer + i];
      own += mine[i];
    }
    double inc = own;
    for (int off = 1; off < 64; off <<= 1) {
      const double o = __shfl_up(inc, off, 64);
      if (lane >= off) inc += o;
    }
    const double excl = __shfl_up(inc, 1, 64);
    double run = base_sh + (lane > 0 ? excl : 0.0);
    unsigned first = 0xffffffffu;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      part[lane * kPer + i] = run;           // exclusive running sum in front of that thread
      run += mine[i];
      if (first == 0xffffffffu && run > thr_sh) first = lane * kPer + i;
    }
    for (int off = 32; off > 0; off >>= 1) first = min(first, static_cast<unsigned>(__shfl_xor(static_cast<int>(first), off, 64)));
    if (lane == 0) thread_sh = first == 0xffffffffu ? -1 : static_cast<int>(first);
  }
  __syncthreads();
  int th = thread_sh;
  if (th < 0) {
    // no running sum exceeds the threshold (rounding): take the last entry with a positive weight
    if (threadIdx.x == 0) {
      int last = min(p.vocab, (seg + 1) * kSampleSeg) - 1;
      while (last > 0 && !(row.weight(last, table) > 0.0)) --last;
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
  p.inv_t_log2e = kLog2e / static_cast<double>(temperature);
  const size_t rows = static_cast<size_t>(total_rows) + total_win;
  char* w = static_cast<char*>(workspace);
  p.seg_stats = reinterpret_cast<double*>(w); w += align16(rows * p.nseg * 2 * sizeof(double));
  p.row_stats = reinterpret_cast<double*>(w); w += align16(rows * 2 * sizeof(double));
  p.res_sums = reinterpret_cast<double*>(w); w += align16(static_cast<size_t>(n_seqs) * p.nseg * sizeof(double));
  p.pick = reinterpret_cast<int*>(w);

  hipStream_t st = static_cast<hipStream_t>(stream);
  if (rows > 0) {
    hipLaunchKernelGGL(sample_stats_kernel, dim3(p.nseg, static_cast<unsigned>(rows)), dim3(kSampleThreads), 0, st, p);
    hipLaunchKernelGGL(sample_rows_kernel, dim3(ceil_div(static_cast<int>(rows), 4)), dim3(256), 0, st, p);
  }
  if (n_seqs > 0) hipLaunchKernelGGL(sample_decide_kernel, dim3(n_seqs), dim3(64), 0, st, p);
  hipLaunchKernelGGL(sample_weights_kernel, dim3(p.nseg, n_seqs), dim3(kSampleThreads), 0, st, p);
  hipLaunchKernelGGL(sample_pick_kernel, dim3(n_seqs), dim3(kSampleThreads), 0, st, p);
  VC_HIP(hipGetLastError());
  return VC_OK;
}
