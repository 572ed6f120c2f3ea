"""CPU pins of the admission-control oracle against what the paper fixes: the worked example of
section 4.2.1 (Mistral 24B on one 96 GB GPU, 10 requests, KV_comp 1 GB, KV_full 4 GB, x = 30) and
the constraints of section 5.1."""
import json
import math
import os

import pytest

from oracle import sched_oracle as S

GB = 1e9
# the example's figures (tests/golden/worked_example_section_4_2_1.json): 64 GB/s link, ~80 ms per
# full-KV transfer (i.e. ~50 GB/s effective), ~35 ms per draft-only iteration for M + B*KV_comp,
# ~37 ms with one verify folded in, peak HBM 64 GB = M + B*KV_comp + KV_full  ->  M = 50 GB
with open(os.path.join(os.path.dirname(__file__), "golden", "worked_example_section_4_2_1.json")) as f:
    EX = json.load(f)
KV_FULL, KV_COMP, NREQ, X = EX["kv_full_GB"] * GB, EX["kv_comp_GB"] * GB, EX["requests"], EX["draft_length_x"]
M = EX["peak_hbm_staggered_GB"] * GB - NREQ * KV_COMP - KV_FULL
BW_EFF = KV_FULL / (EX["transfer_ms_per_verify_approx"] * 1e-3)
BW_HBM = (M + NREQ * KV_COMP) / (EX["draft_only_iteration_ms_approx"] * 1e-3)
LINK = EX["link_GBps_nominal"] * GB


def test_eq3_reproduces_the_example_iteration_times():
    t_iter, t_gpu, t_xfer = S.t_iter_model(M, NREQ, KV_FULL, KV_COMP / KV_FULL, X, BW_HBM, LINK)
    # draft traffic plus one thirtieth of each request's full KV per iteration: between the
    # example's 35 ms (draft only) and 37 ms (one whole verify folded in)
    assert 0.035 < t_gpu < 0.037
    assert math.isclose(t_gpu, (60 * GB + NREQ * KV_FULL / X) / BW_HBM, rel_tol=1e-12)
    assert math.isclose(t_xfer, 40 * GB / (30 * 64 * GB), rel_tol=1e-12) and t_iter == t_gpu
    # one whole verify in an iteration: 64 GB over the same HBM -> the example's ~37 ms
    assert math.isclose((M + NREQ * KV_COMP + KV_FULL) / BW_HBM, 0.0373, abs_tol=2e-4)
    # transfer-bound regime: max() picks the link
    t_iter2, t_gpu2, t_xfer2 = S.t_iter_model(M, 100, KV_FULL, 0.25, 2, BW_HBM, 1 * GB)
    assert t_iter2 == t_xfer2 > t_gpu2


def example_rings(hbm=96 * GB):
    return S.Rings(windows=64, t_iter=0.037, bw=BW_EFF, hbm_bytes=hbm, model_bytes=M, resident_bytes=NREQ * KV_COMP)


def test_worked_example_verifies_land_one_every_three_iterations():
    r = example_rings()
    assert r.span_windows(KV_FULL) == EX["verify_spacing_iterations"] == 3   # 80 ms of link time over 37 ms windows
    ds = [r.admit(i, KV_FULL, X) for i in range(NREQ)]
    assert ds[0] == X                                     # the first request gets its anchor
    assert ds[:4] == [30, 27, 33, 24]                     # then x-1, x+1, x-2, ... until a free span
    assert sorted(ds) == list(range(15, 45, 3))           # "spread one every 3 draft iterations"
    assert all(t <= r.t_iter for t in r.T)
    # only one full KV is ever in flight: peak HBM = M + B*KV_comp + 1*KV_full = 64 GB
    assert r.peak_hbm() == EX["peak_hbm_staggered_GB"] * GB
    # the lock-step alternative of the example: all full KVs resident at once, 40 GB serialised
    assert M + NREQ * KV_FULL == EX["lock_step_peak_hbm_GB"] * GB
    lock_ms = NREQ * KV_FULL / BW_EFF * 1e3
    assert lock_ms == pytest.approx(EX["lock_step_transfer_ms_approx"])
    assert 20 <= lock_ms / 37 < 23 and EX["lock_step_transfer_over_window_approx"] == 20
    # link time booked in total = 10 transfers of 80 ms
    assert math.isclose(sum(r.T), NREQ * 0.080, rel_tol=1e-12)


def test_lock_step_batching_is_refused():
    """All verifies in the same window would need 800 ms of link time in a 37 ms window."""
    r = example_rings()
    assert r.admit(0, KV_FULL, X) == X
    share = (KV_FULL / BW_EFF) / 3
    for i in (28, 29, 30):
        assert r.T[i] == share and r.T[i] + share > r.t_iter
    assert r.admit(1, KV_FULL, X) != X


def test_hbm_ring_constraint_and_waiting_queue():
    # 58 + 4 fits, a second in-flight KV in the same windows would not; with a link fast enough
    # that time never binds, the HBM ring alone spreads the verifies
    r = S.Rings(windows=8, t_iter=1.0, bw=1e15, hbm_bytes=62 * GB, model_bytes=M, resident_bytes=8 * GB)
    assert r.span_windows(KV_FULL) == 1
    ds = [r.admit(i, KV_FULL, 4) for i in range(9)]
    assert ds[:7] == [4, 3, 5, 2, 6, 1, 7]                # every window 1..7 taken once
    assert ds[7:] == [-1, -1]                             # no window left: waiting queue
    # a request whose span is longer than the horizon can never be placed
    r2 = S.Rings(windows=4, t_iter=0.01, bw=BW_EFF, hbm_bytes=96 * GB, model_bytes=M)
    assert r2.span_windows(KV_FULL) == 8 and r2.admit(0, KV_FULL, 2) == -1
    # the anchor is clamped to [S_r, W-1]
    r3 = example_rings()
    assert r3.admit(0, KV_FULL, 1) == 3 and r3.admit(1, KV_FULL, 1000) == 63


def test_execution_loop_kicks_and_verifies_on_time():
    r = example_rings()
    ds = {i: r.admit(i, KV_FULL, X) for i in range(NREQ)}
    kicked, verified = {}, {}
    for t in range(64):
        kick, ver = r.step()
        for q in kick:
            kicked[q] = t
        for q in ver:
            verified[q] = t
    assert verified == ds                                  # verified exactly in the reserved window
    assert all(kicked[q] == ds[q] - 2 for q in ds)         # reload starts S_r - 1 windows earlier
    assert not r.reserved and not any(r.T) and not any(r.B)
    # re-admission after a verify (the loop of section 5.2): steady state keeps the 3-window spacing
    r = example_rings()
    for i in range(NREQ):
        r.admit(i, KV_FULL, X)
    seen = []
    for t in range(200):
        _, ver = r.step()
        for q in ver:
            seen.append(t)
            assert r.admit(q, KV_FULL, X) >= 3
    gaps = [b - a for a, b in zip(seen, seen[1:])]
    assert len(seen) >= 50 and min(gaps) >= 3
