"""CPU pins of the sampling-acceptance oracle: the property that defines speculative sampling (the
emitted token is distributed exactly as the target distribution, whatever the draft distribution),
its greedy limit (which must coincide with the greedy oracle), and brute-force special cases."""
import numpy as np
import pytest

from oracle import sample_oracle as S
from oracle import vc_oracle as O


def one_seq(target, draft, ids, T, ua, ur, bonus=False):
    w = len(ids)
    rows = w + (1 if bonus else 0)
    return S.accept_sample(np.asarray(target, dtype=np.float64).reshape(rows, -1), np.asarray(draft, dtype=np.float64).reshape(w, -1),
                           [0, rows], np.asarray(ids), [0, w], T, np.asarray(ua, dtype=np.float64), np.asarray([ur], dtype=np.float64))


def test_emitted_token_follows_the_target_distribution_exactly():
    """One drafted position, vocabulary of 4.  Integrate over the draft token (weight q), the
    accept draw and the resample draw on fine grids: the first emitted token (the draft if
    accepted, the correction otherwise) must have distribution p."""
    rng = np.random.default_rng(5)
    for _ in range(3):
        lt, ld = rng.normal(size=4) * 1.5, rng.normal(size=4) * 1.5
        T = 0.8
        p, q = S.softmax_t(lt, T), S.softmax_t(ld, T)
        n = 400
        grid = (np.arange(n) + 0.5) / n
        out = np.zeros(4)
        for t in range(4):
            for ua in grid:
                a, nx, _ = one_seq(lt, ld, [t], T, [ua], 0.0)
                if a[0] == 1:
                    out[t] += q[t] / n
                else:
                    # rejected: integrate the correction over the second draw
                    for ur in grid[::8]:
                        _, nx, _ = one_seq(lt, ld, [t], T, [ua], ur)
                        out[nx[0]] += q[t] / n / len(grid[::8])
        assert np.abs(out - p).max() < 2.5e-2 / 4 + 1.0 / n * 4
        # closed form of the acceptance probability: sum_v min(p, q)
        acc_prob = sum(q[t] * np.mean([one_seq(lt, ld, [t], T, [ua], 0.0)[0][0] for ua in grid]) for t in range(4))
        assert abs(acc_prob - np.minimum(p, q).sum()) < 4.0 / n


def test_low_temperature_limit_is_greedy_acceptance():
    rng = np.random.default_rng(11)
    V, w, B = 50, 6, 8
    target = rng.normal(size=(B * (w + 1), V))
    draft = rng.normal(size=(B * w, V))
    cu_rows = np.arange(0, B * (w + 1) + 1, w + 1)
    cu_win = np.arange(0, B * w + 1, w)
    # draft ids = arg-max of the draft rows (what a near-zero temperature samples), agreeing with
    # the target's arg-max for a seeded prefix
    ids = np.empty(B * w, dtype=np.int64)
    for b in range(B):
        L = int(rng.integers(0, w + 1))
        for j in range(w):
            t_star = int(np.argmax(target[cu_rows[b] + j]))
            if j < L:
                draft[cu_win[b] + j, t_star] = 9.0
            ids[cu_win[b] + j] = int(np.argmax(draft[cu_win[b] + j]))
    ua, ur = rng.random(B * w), rng.random(B)
    a, nx, _ = S.accept_sample(target, draft, cu_rows, ids, cu_win, 1e-3, ua, ur)
    ga, gn, _ = O.accept(target.astype(np.float32), cu_rows, ids, cu_win)
    assert np.array_equal(a, ga) and np.array_equal(nx, gn)


def test_identical_distributions_accept_everything_and_bonus_is_inverse_cdf():
    rng = np.random.default_rng(3)
    V, w = 17, 5
    logits = rng.normal(size=(w + 1, V))
    ids = rng.integers(0, V, size=w)
    for ur in (0.0, 0.37, 0.999999):
        a, nx, (ma, mr) = one_seq(logits, logits[:w], ids, 1.3, rng.random(w), ur, bonus=True)
        assert a[0] == w
        p = S.softmax_t(logits[w], 1.3)
        running, want = 0.0, None
        for v in range(V):                       # brute-force inverse CDF
            running += p[v]
            if running > ur * p.sum() and want is None:
                want = v
        assert nx[0] == want
    a, nx, _ = one_seq(logits[:w], logits[:w], ids, 1.3, rng.random(w), 0.5)
    assert a[0] == w and nx[0] == -1              # no bonus row supplied


def test_disjoint_support_rejects_and_resamples_from_target():
    V = 6
    target = np.full((1, V), -1e9); target[0, [1, 4]] = [0.0, np.log(3.0)]     # p = (1/4, 3/4) on {1, 4}
    draft = np.full((1, V), -1e9); draft[0, [0, 2]] = 0.0
    for ur, want in ((0.1, 1), (0.2499, 1), (0.2501, 4), (0.9, 4)):
        a, nx, _ = one_seq(target, draft, [2], 1.0, [0.3], ur)
        assert a[0] == 0 and nx[0] == want
    # the accept test itself: p(t)/q(t) = 0.5 -> accepted iff u < 0.5
    target = np.log(np.array([[0.25, 0.75]])); draft = np.log(np.array([[0.5, 0.5]]))
    assert one_seq(target, draft, [0], 1.0, [0.49], 0.0)[0][0] == 1
    a, nx, (ma, _) = one_seq(target, draft, [0], 1.0, [0.51], 0.0)
    assert a[0] == 0 and nx[0] == 1 and ma[0] == pytest.approx(0.02, rel=1e-6)   # residual = (0, 0.25)
    # temperature rescales the logits: T = 2 with doubled logits is T = 1
    rng = np.random.default_rng(9)
    lt, ld = rng.normal(size=(3, 9)), rng.normal(size=(3, 9))
    ids, ua = rng.integers(0, 9, size=3), rng.random(3)
    r1 = S.accept_sample(lt, ld, [0, 3], ids, [0, 3], 1.0, ua, [0.4])
    r2 = S.accept_sample(2 * lt, 2 * ld, [0, 3], ids, [0, 3], 2.0, ua, [0.4])
    assert np.array_equal(r1[0], r2[0]) and np.array_equal(r1[1], r2[1])
