"""Plain CPU oracle of the runtime's admission control (TEST INFRASTRUCTURE, not a product path).

Paper section 5: a horizon of W future iterations ("windows", window 0 = the current one) with two
reserve rings - T[i], the interconnect time already reserved in window i (constraint
T[i] <= T_iter), and B[i], the in-flight full-KV bytes occupying HBM in window i (constraint
M + KV_resident + B[i] <= HBM) - the Admit operation of Algorithm 1 that places a request's next
verify in a window with spare capacity, and the three-step execution loop (kick off the reloads
whose span starts now, verify the requests whose window is now, slide the horizon).  Section 4.2.1
gives the iteration-time model (Eq. 3) that T_iter comes from.

Everything is a Python float (IEEE double) in the order written here; the library repeats the same
operations in the same order in C++, so the decisions must be identical, not just close.

Readings where the paper leaves a choice (listed again in the design notes):
  * a reload of duration KV_full / BW spans S_r windows and books an equal share of that time,
    (KV_full / BW) / S_r, in each of them;
  * the staging buffer exists for the whole span: B[i] grows by KV_full in every window of it;
  * candidates are tried in the order anchor, anchor-1, anchor+1, anchor-2, anchor+2, ...; a
    candidate outside [S_r, W-1] is skipped (clamping would only repeat an end point);
  * a reservation whose span is [d-S_r+1, d] starts its transfer when window d-S_r+1 becomes the
    current window and is verified when window d becomes the current window.
"""
from __future__ import annotations

import math


def t_iter_model(model_bytes, batch, kv_full_bytes, c, x, bw_hbm, bw_inter):
    """Eq. 3: (T_iter, T_gpu, T_xfer) in seconds for B requests that each keep c*KV_full on the GPU
    and verify once per x drafted tokens."""
    t_gpu = (model_bytes + batch * kv_full_bytes * (c + 1.0 / x)) / bw_hbm
    t_xfer = batch * kv_full_bytes / (x * bw_inter)
    return max(t_gpu, t_xfer), t_gpu, t_xfer


class Rings:
    """The resource model of section 5.1 plus Admit (Algorithm 1) and the execution loop (5.2)."""

    def __init__(self, windows, t_iter, bw, hbm_bytes, model_bytes, resident_bytes=0.0):
        self.W = int(windows)
        self.t_iter = float(t_iter)
        self.bw = float(bw)
        self.hbm = float(hbm_bytes)
        self.model = float(model_bytes)
        self.resident = float(resident_bytes)
        self.T = [0.0] * self.W            # window 0 = now
        self.B = [0.0] * self.W
        self.now = 0                        # absolute iteration of window 0
        self.reserved = {}                  # request id -> (first absolute window, deadline, kv bytes)

    def span_windows(self, kv_full_bytes):
        ell = kv_full_bytes / (self.bw * self.t_iter)
        return max(1, math.ceil(ell))

    def candidates(self, x, s_r):
        lo, hi = s_r, self.W - 1
        if lo > hi:
            return []
        anchor = min(max(int(x), lo), hi)
        out = [anchor]
        for k in range(1, self.W):
            for d in (anchor - k, anchor + k):
                if lo <= d <= hi:
                    out.append(d)
        return out

    def admit(self, req, kv_full_bytes, x):
        """Returns the verify window d (relative to now), or -1: back to the waiting queue."""
        if req in self.reserved:
            raise ValueError("request already holds a reservation")
        s_r = self.span_windows(kv_full_bytes)
        share = (kv_full_bytes / self.bw) / s_r
        for d in self.candidates(x, s_r):
            ok = True
            for i in range(d - s_r + 1, d + 1):
                if not (self.T[i] + share <= self.t_iter):
                    ok = False
                    break
                if not (self.model + self.resident + self.B[i] + kv_full_bytes <= self.hbm):
                    ok = False
                    break
            if ok:
                for i in range(d - s_r + 1, d + 1):
                    self.T[i] += share
                    self.B[i] += kv_full_bytes
                self.reserved[req] = (self.now + d - s_r + 1, self.now + d, float(kv_full_bytes))
                return d
        return -1

    def step(self):
        """One iteration: (requests whose reload starts now, requests verified now), then slide.
        A verified request gives up its reservation (the caller re-admits it)."""
        kick = sorted(r for r, (first, _, _) in self.reserved.items() if first == self.now)
        verify = sorted(r for r, (_, dl, _) in self.reserved.items() if dl == self.now)
        for r in verify:
            del self.reserved[r]
        self.T = self.T[1:] + [0.0]
        self.B = self.B[1:] + [0.0]
        self.now += 1
        return kick, verify

    def peak_hbm(self):
        return self.model + self.resident + max(self.B)
