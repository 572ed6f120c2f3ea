"""The library's admission control (host C++: reserve rings, Admit, execution loop, Eq. 3) against
the CPU oracle: identical decisions and identical ring contents, on the paper's worked example
(section 4.2.1) and on seeded random request mixes.  No GPU is needed: nothing here launches."""
import random

import pytest

import paper_2605_17613_amd as vc
from oracle import sched_oracle as S

GB = 1e9
M, KV_FULL, KV_COMP, NREQ, X = 50 * GB, 4 * GB, 1 * GB, 10, 30
BW_EFF = KV_FULL / 0.080


def pair(windows, t_iter, bw, hbm, model, resident=0.0):
    return (S.Rings(windows, t_iter, bw, hbm, model, resident),
            vc.Sched(windows, t_iter, bw, hbm, model, resident))


def same_state(o, g):
    t, b, now = g.rings()
    assert t == o.T and b == o.B and now == o.now          # bit-identical doubles


def test_eq3_model_matches_oracle():
    rng = random.Random(7)
    for _ in range(200):
        a = (rng.uniform(1, 100) * GB, rng.randint(1, 64), rng.uniform(0.1, 16) * GB, rng.uniform(0.05, 1.0),
             rng.randint(1, 64), rng.uniform(0.5, 8) * 1e12, rng.uniform(1, 64) * GB)
        assert vc.vc_iter_time_model(*a) == S.t_iter_model(*a)


def test_worked_example_decisions_and_loop():
    o, g = pair(64, 0.037, BW_EFF, 96 * GB, M, NREQ * KV_COMP)
    assert g.span(KV_FULL) == o.span_windows(KV_FULL) == 3
    for i in range(NREQ):
        assert g.admit(i, KV_FULL, X) == o.admit(i, KV_FULL, X)
    same_state(o, g)
    for _ in range(200):
        ko, vo = o.step()
        kg, vg = g.step()
        assert (kg, vg) == (ko, vo)
        for q in vo:
            assert g.admit(q, KV_FULL, X) == o.admit(q, KV_FULL, X)
        same_state(o, g)


@pytest.mark.parametrize("seed", range(6))
def test_random_mixes_match_oracle(seed):
    rng = random.Random(1000 + seed)
    W = rng.choice([4, 16, 48, 128])
    t_iter = rng.uniform(0.005, 0.05)
    bw = rng.uniform(10, 64) * GB
    hbm = rng.uniform(80, 288) * GB
    o, g = pair(W, t_iter, bw, hbm, 40 * GB, rng.uniform(0, 30) * GB)
    sizes = {}
    waiting = []
    nxt = 0
    for it in range(300):
        # new arrivals and retries of the waiting queue
        for _ in range(rng.randint(0, 2)):
            sizes[nxt] = (rng.choice([0.0, 0.3, 1.0, 2.5, 4.0, 17.2]) * GB, rng.randint(1, 2 * W))
            waiting.append(nxt)
            nxt += 1
        still = []
        for q in waiting:
            kv, x = sizes[q]
            d_o, d_g = o.admit(q, kv, x), g.admit(q, kv, x)
            assert d_o == d_g
            if d_o < 0:
                still.append(q)
        waiting = still[-8:]
        ko, vo = o.step()
        assert g.step() == (ko, vo)
        for q in vo:
            if rng.random() < 0.7:
                waiting.append(q)
        same_state(o, g)
    assert nxt > 100


def test_full_windows_at_exact_equality_and_errors():
    # a window that is exactly full is still usable: two transfers of T_iter/2 fit one window
    o, g = pair(4, 1.0, 8.0, 1e9, 0.0)
    for q in range(3):
        assert g.admit(q, 4.0, 2) == o.admit(q, 4.0, 2)
    same_state(o, g)
    with pytest.raises(vc.VcError):
        g.admit(0, 4.0, 2)                                   # already holds a reservation
    with pytest.raises(vc.VcError):
        g.cancel(99)
    with pytest.raises(vc.VcError):
        vc.Sched(0, 1.0, 1.0, 1.0, 0.0)
    with pytest.raises(vc.VcError):
        vc.Sched(4, 0.0, 1.0, 1.0, 0.0)


def test_cancel_returns_capacity():
    o, g = pair(16, 0.037, BW_EFF, 96 * GB, M, NREQ * KV_COMP)
    assert g.admit(1, KV_FULL, 8) == 8
    g.step(); g.step()
    g.cancel(1)
    t, b, now = g.rings()
    assert now == 2 and not any(t) and not any(b)
    assert g.admit(2, KV_FULL, 6) == 6
    # capacity of the output arrays is enforced without side effects
    small = vc.Sched(8, 1.0, 1e15, 1e15, 0.0, capacity=1)
    assert small.admit(1, 1.0, 1) == 1 and small.admit(2, 1.0, 1) == 1
    small.step()
    with pytest.raises(vc.VcError):
        small.step()
    assert small.rings()[2] == 1
