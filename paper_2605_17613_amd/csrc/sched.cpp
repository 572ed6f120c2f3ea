// Admission control of the runtime (paper section 5): the two reserve rings of section 5.1, the
// Admit operation of Algorithm 1 and the three-step execution loop of section 5.2, plus the
// iteration-time model of section 4.2.1 (Eq. 3).  Host code only: nothing here touches the GPU.
// The caller maps the loop's decisions onto vc_swap_in (kick), vc_swap_wait + vc_verify_attn
// (verify) and vc_draft_attn (everything else).
//
// All quantities are IEEE doubles and every expression is evaluated in the order written (this
// file is compiled without contraction or reassociation), so that a decision taken at an equality
// boundary - a window that is exactly full - is reproducible.
#include <math.h>
#include <stdlib.h>

#include <algorithm>
#include <new>
#include <vector>

#include "common.h"

#pragma STDC FP_CONTRACT OFF

struct vc_sched {
  int32_t W;
  double t_iter, bw, hbm, model, resident;
  std::vector<double> T, B;  // ring storage; window i lives in slot (head + i) % W
  int32_t head;
  int64_t now;
  struct Res { int64_t req, first, deadline; double bytes; };
  std::vector<Res> reserved;

  double& t_at(int32_t i) { return T[(head + i) % W]; }
  double& b_at(int32_t i) { return B[(head + i) % W]; }
};

using namespace vc;

namespace {

int32_t span_windows(const vc_sched* s, double kv_full_bytes) {
  // section 5.1: l_r = KV_full / (BW * T_iter), S_r = max(1, ceil(l_r))
  double ell = kv_full_bytes / (s->bw * s->t_iter);
  double c = ceil(ell);
  if (!(c < 2147483647.0)) return 2147483647;
  return std::max<int32_t>(1, static_cast<int32_t>(c));
}

bool span_fits(vc_sched* s, int32_t d, int32_t s_r, double share, double kv) {
  for (int32_t i = d - s_r + 1; i <= d; ++i) {
    if (!(s->t_at(i) + share <= s->t_iter)) return false;                       // BW ring
    if (!(s->model + s->resident + s->b_at(i) + kv <= s->hbm)) return false;    // HBM ring
  }
  return true;
}

}  // namespace

extern "C" vc_status vc_iter_time_model(double model_bytes, double batch, double kv_full_bytes, double c,
                                        double x, double bw_hbm, double bw_inter, double* t_iter,
                                        double* t_gpu, double* t_xfer) {
  VC_REQUIRE(t_iter != nullptr, VC_ERR_INVALID_ARG, "vc_iter_time_model: t_iter is NULL");
  VC_REQUIRE(x > 0 && bw_hbm > 0 && bw_inter > 0, VC_ERR_INVALID_ARG,
             "vc_iter_time_model: x and both bandwidths must be positive");
  double g = (model_bytes + batch * kv_full_bytes * (c + 1.0 / x)) / bw_hbm;
  double t = batch * kv_full_bytes / (x * bw_inter);
  *t_iter = g > t ? g : t;
  if (t_gpu) *t_gpu = g;
  if (t_xfer) *t_xfer = t;
  return VC_OK;
}

extern "C" vc_status vc_sched_create(int32_t windows, double t_iter_s, double bw_bytes_per_s, double hbm_bytes,
                                     double model_bytes, double resident_bytes, vc_sched** out) {
  VC_REQUIRE(out != nullptr, VC_ERR_INVALID_ARG, "vc_sched_create: out is NULL");
  *out = nullptr;
  VC_REQUIRE(windows >= 1 && windows <= (1 << 20), VC_ERR_INVALID_ARG, "vc_sched_create: windows %d", windows);
  VC_REQUIRE(t_iter_s > 0 && bw_bytes_per_s > 0, VC_ERR_INVALID_ARG,
             "vc_sched_create: t_iter and bw must be positive");
  VC_REQUIRE(hbm_bytes >= 0 && model_bytes >= 0 && resident_bytes >= 0, VC_ERR_INVALID_ARG,
             "vc_sched_create: negative byte count");
  vc_sched* s = new (std::nothrow) vc_sched();
  VC_REQUIRE(s != nullptr, VC_ERR_INVALID_ARG, "vc_sched_create: out of host memory");
  s->W = windows;
  s->t_iter = t_iter_s; s->bw = bw_bytes_per_s; s->hbm = hbm_bytes;
  s->model = model_bytes; s->resident = resident_bytes;
  s->T.assign(windows, 0.0); s->B.assign(windows, 0.0);
  s->head = 0; s->now = 0;
  *out = s;
  return VC_OK;
}

extern "C" vc_status vc_sched_destroy(vc_sched* s) {
  delete s;
  return VC_OK;
}

extern "C" vc_status vc_sched_set_resident(vc_sched* s, double resident_bytes) {
  VC_REQUIRE(s != nullptr && resident_bytes >= 0, VC_ERR_INVALID_ARG, "vc_sched_set_resident: bad argument");
  s->resident = resident_bytes;
  return VC_OK;
}

extern "C" vc_status vc_sched_span(const vc_sched* s, double kv_full_bytes, int32_t* span) {
  VC_REQUIRE(s != nullptr && span != nullptr, VC_ERR_INVALID_ARG, "vc_sched_span: NULL argument");
  VC_REQUIRE(kv_full_bytes >= 0, VC_ERR_INVALID_ARG, "vc_sched_span: negative size");
  *span = span_windows(s, kv_full_bytes);
  return VC_OK;
}

extern "C" vc_status vc_sched_admit(vc_sched* s, int64_t req, double kv_full_bytes, int32_t x, int32_t* window) {
  VC_REQUIRE(s != nullptr && window != nullptr, VC_ERR_INVALID_ARG, "vc_sched_admit: NULL argument");
  VC_REQUIRE(kv_full_bytes >= 0, VC_ERR_INVALID_ARG, "vc_sched_admit: negative size");
  *window = -1;
  for (const auto& r : s->reserved)
    VC_REQUIRE(r.req != req, VC_ERR_INVALID_ARG, "vc_sched_admit: request %lld already holds a reservation",
               static_cast<long long>(req));
  const int32_t s_r = span_windows(s, kv_full_bytes);
  const int32_t lo = s_r, hi = s->W - 1;
  if (lo > hi) return VC_OK;  // the span is longer than the horizon: waiting queue
  const double share = (kv_full_bytes / s->bw) / s_r;
  const int32_t anchor = std::min(std::max(x, lo), hi);
  int32_t found = -1;
  if (span_fits(s, anchor, s_r, share, kv_full_bytes)) found = anchor;
  for (int32_t k = 1; found < 0 && k < s->W; ++k) {
    // earlier candidate first, then the later one at the same distance
    const int32_t cand[2] = {anchor - k, anchor + k};
    for (int32_t d : cand) {
      if (d < lo || d > hi) continue;
      if (span_fits(s, d, s_r, share, kv_full_bytes)) { found = d; break; }
    }
  }
  if (found < 0) return VC_OK;
  for (int32_t i = found - s_r + 1; i <= found; ++i) {
    s->t_at(i) += share;
    s->b_at(i) += kv_full_bytes;
  }
  s->reserved.push_back({req, s->now + found - s_r + 1, s->now + found, kv_full_bytes});
  *window = found;
  return VC_OK;
}

extern "C" vc_status vc_sched_cancel(vc_sched* s, int64_t req) {
  VC_REQUIRE(s != nullptr, VC_ERR_INVALID_ARG, "vc_sched_cancel: sched is NULL");
  for (size_t j = 0; j < s->reserved.size(); ++j) {
    if (s->reserved[j].req != req) continue;
    const auto r = s->reserved[j];
    // give back what the windows still ahead hold; the share is recomputed as it was booked
    const int32_t s_r = static_cast<int32_t>(r.deadline - r.first + 1);
    const double share = (r.bytes / s->bw) / s_r;
    for (int64_t a = std::max(r.first, s->now); a <= r.deadline; ++a) {
      const int32_t i = static_cast<int32_t>(a - s->now);
      s->t_at(i) -= share;
      s->b_at(i) -= r.bytes;
    }
    s->reserved.erase(s->reserved.begin() + j);
    return VC_OK;
  }
  return fail(VC_ERR_INVALID_ARG, "vc_sched_cancel: request %lld holds no reservation", static_cast<long long>(req));
}

extern "C" vc_status vc_sched_step(vc_sched* s, int64_t* kick, int32_t* n_kick, int64_t* verify,
                                   int32_t* n_verify, int32_t capacity) {
  VC_REQUIRE(s != nullptr && n_kick != nullptr && n_verify != nullptr, VC_ERR_INVALID_ARG,
             "vc_sched_step: NULL argument");
  VC_REQUIRE(capacity >= 0 && (capacity == 0 || (kick != nullptr && verify != nullptr)), VC_ERR_INVALID_ARG,
             "vc_sched_step: bad output arrays");
  int32_t nk = 0, nv = 0;
  for (const auto& r : s->reserved) {
    nk += r.first == s->now;
    nv += r.deadline == s->now;
  }
  // nothing is changed unless both lists fit
  VC_REQUIRE(nk <= capacity && nv <= capacity, VC_ERR_INVALID_ARG,
             "vc_sched_step: %d kicks / %d verifies exceed capacity %d", nk, nv, capacity);
  nk = nv = 0;
  for (const auto& r : s->reserved) {
    if (r.first == s->now) kick[nk++] = r.req;
    if (r.deadline == s->now) verify[nv++] = r.req;
  }
  std::sort(kick, kick + nk);
  std::sort(verify, verify + nv);
  s->reserved.erase(std::remove_if(s->reserved.begin(), s->reserved.end(),
                                   [&](const vc_sched::Res& r) { return r.deadline == s->now; }),
                    s->reserved.end());
  // slide: window 0 leaves, a fresh empty window enters at the far end
  s->T[s->head] = 0.0;
  s->B[s->head] = 0.0;
  s->head = (s->head + 1) % s->W;
  s->now += 1;
  *n_kick = nk;
  *n_verify = nv;
  return VC_OK;
}

extern "C" vc_status vc_sched_rings(const vc_sched* s, double* t_ring, double* b_ring, int64_t* now) {
  VC_REQUIRE(s != nullptr, VC_ERR_INVALID_ARG, "vc_sched_rings: sched is NULL");
  for (int32_t i = 0; i < s->W; ++i) {
    if (t_ring) t_ring[i] = s->T[(s->head + i) % s->W];
    if (b_ring) b_ring[i] = s->B[(s->head + i) % s->W];
  }
  if (now) *now = s->now;
  return VC_OK;
}
