"""GPU parity of sampling-based acceptance against the fp64 oracle: identical accept lengths and
drawn tokens on seeded inputs whose every decision the oracle reports to be clear of a tie (the
library and the oracle sum in different orders, so a draw within 1e-9 of a boundary could go either
way; the generator nudges such draws, which it can since the random numbers are inputs)."""
import numpy as np
import pytest
import torch

import paper_2605_17613_amd as vc
from oracle import sample_oracle as S

pytestmark = pytest.mark.gpu
MARGIN = 1e-7


@pytest.fixture(scope="module")
def lib():
    vc.load()
    assert torch.cuda.is_available()
    return vc


@pytest.fixture()
def ctx(lib):
    c = vc.Context(0)
    yield c
    c.close()


def make_case(seed, vocab, wins, bonus, temperature, noise):
    """Target logits ~ N(0, 2); draft logits = target + noise * N(0, 1) (a compressed cache that is
    close to the full one); drafted ids sampled from the draft distribution; a -inf entry per row."""
    rng = np.random.default_rng(seed)
    nseq = len(wins)
    rows = [w + (1 if bonus[b] else 0) for b, w in enumerate(wins)]
    cu_rows = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    cu_win = np.concatenate([[0], np.cumsum(wins)]).astype(np.int32)
    target = (2.0 * rng.standard_normal((int(cu_rows[-1]), vocab))).astype(np.float32)
    draft = np.empty((int(cu_win[-1]), vocab), dtype=np.float32)
    ids = np.empty(int(cu_win[-1]), dtype=np.int32)
    for b in range(nseq):
        for j in range(wins[b]):
            d = target[cu_rows[b] + j] + (noise * rng.standard_normal(vocab)).astype(np.float32)
            d[int(rng.integers(0, vocab))] = -np.inf
            draft[cu_win[b] + j] = d
            q = S.softmax_t(d, temperature)
            ids[cu_win[b] + j] = int(rng.choice(vocab, p=q))
    if len(target):
        target[0, 3 % vocab] = -np.inf
    ua = rng.random(int(cu_win[-1])).astype(np.float32)
    ur = rng.random(nseq).astype(np.float32)
    # keep every decision clear of a tie
    for _ in range(20):
        a, nx, (ma, mr) = S.accept_sample(target, draft, cu_rows, ids, cu_win, temperature, ua, ur)
        bad_a, bad_r = ma < MARGIN, mr < MARGIN
        if not bad_a.any() and not bad_r.any():
            break
        ua[bad_a] *= 0.5
        ur[bad_r] = (ur[bad_r] * 0.5 + 0.123).astype(np.float32) % 1.0
    else:
        raise AssertionError("could not clear the ties")
    return target, draft, cu_rows, cu_win, ids, ua, ur, a, nx


def run_gpu(ctx, target, draft, cu_rows, cu_win, ids, ua, ur, temperature):
    dev = "cuda:0"
    t = lambda x, dt: torch.tensor(x, dtype=dt, device=dev)
    nseq = len(cu_rows) - 1
    acc = torch.full((nseq,), -7, dtype=torch.int32, device=dev)
    nxt = torch.full((nseq,), -7, dtype=torch.int32, device=dev)
    ws = torch.empty(vc.vc_accept_sample_workspace_bytes(target.shape[0], draft.shape[0], nseq, target.shape[1]),
                     dtype=torch.uint8, device=dev)
    vc.vc_accept_sample(ctx, t(target, torch.float32), t(draft, torch.float32), t(cu_rows, torch.int32), t(ids, torch.int32),
                        t(cu_win, torch.int32), temperature, t(ua, torch.float32), t(ur, torch.float32), acc, nxt, workspace=ws)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), nxt.cpu().numpy()


@pytest.mark.parametrize("vocab,temperature,noise", [(1000, 0.7, 0.5), (32001, 1.0, 0.3), (128256, 0.8, 1.2), (8192 * 2 + 5, 1.5, 1.0)])
def test_accept_sample_matches_oracle(lib, ctx, vocab, temperature, noise):
    wins = [5, 0, 12, 1, 7, 3]
    bonus = [True, True, False, True, False, True]
    target, draft, cu_rows, cu_win, ids, ua, ur, a, nx = make_case(100 + vocab % 97, vocab, wins, bonus, temperature, noise)
    ga, gn = run_gpu(ctx, target, draft, cu_rows, cu_win, ids, ua, ur, temperature)
    assert np.array_equal(ga, a), (ga, a)
    assert np.array_equal(gn, nx), (gn, nx)
    # the case exercises every branch: some rejection, some full acceptance with and without bonus
    assert (a < np.array(wins)).any()


def test_accept_sample_identical_distributions_and_greedy_limit(lib, ctx):
    rng = np.random.default_rng(8)
    vocab, wins = 5000, [6, 4, 9]
    cu_win = np.array([0, 6, 10, 19], dtype=np.int32)
    cu_rows = np.array([0, 7, 11, 21], dtype=np.int32)      # first and last bring a bonus row
    target = rng.standard_normal((21, vocab)).astype(np.float32)
    sel = np.concatenate([np.arange(cu_rows[b], cu_rows[b] + wins[b]) for b in range(3)])
    draft = target[sel].copy()
    ids = rng.integers(0, vocab, size=19).astype(np.int32)
    ua = rng.random(19).astype(np.float32)
    ur = np.array([0.25, 0.5, 0.75], dtype=np.float32)
    a, nx, (_, mr) = S.accept_sample(target, draft, cu_rows, ids, cu_win, 1.0, ua, ur)
    assert list(a) == wins and nx[1] == -1 and (mr[[0, 2]] > MARGIN).all()
    ga, gn = run_gpu(ctx, target, draft, cu_rows, cu_win, ids, ua, ur, 1.0)
    assert np.array_equal(ga, a) and np.array_equal(gn, nx)
    # near-zero temperature with arg-max drafts: the greedy rule
    draft2 = rng.standard_normal((19, vocab)).astype(np.float32)
    for i, r in enumerate(sel):
        if i % 4 != 3:
            draft2[i, int(np.argmax(target[r]))] = 20.0
    ids2 = np.argmax(draft2, axis=1).astype(np.int32)
    a2, nx2, _ = S.accept_sample(target, draft2, cu_rows, ids2, cu_win, 1e-2, ua, ur)
    ga2, gn2 = run_gpu(ctx, target, draft2, cu_rows, cu_win, ids2, ua, ur, 1e-2)
    assert np.array_equal(ga2, a2) and np.array_equal(gn2, nx2)
    assert (a2 <= np.array([3, 1, 1])).all()     # positions 3, 7, 11, ... of the concatenated windows were not planted


def test_accept_sample_rejects_bad_arguments(lib, ctx):
    dev = "cuda:0"
    z = torch.zeros((2, 8), dtype=torch.float32, device=dev)
    cu = torch.tensor([0, 2], dtype=torch.int32, device=dev)
    ids = torch.zeros(2, dtype=torch.int32, device=dev)
    u = torch.zeros(2, dtype=torch.float32, device=dev)
    out = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = torch.empty(vc.vc_accept_sample_workspace_bytes(2, 2, 1, 8), dtype=torch.uint8, device=dev)
    with pytest.raises(vc.VcError):
        vc.vc_accept_sample(ctx, z, z, cu, ids, cu, 0.0, u, u[:1], out, out.clone(), workspace=ws)      # temperature
    with pytest.raises(vc.VcError):
        vc.vc_accept_sample(ctx, z, z, cu, ids, cu, 1.0, u, u[:1], out, out.clone(), workspace=ws[:16])  # workspace
    with pytest.raises(vc.VcError):
        vc.vc_accept_sample(ctx, z[:1], z, cu, ids, cu, 1.0, u, u[:1], out, out.clone(), workspace=ws)   # fewer target rows
