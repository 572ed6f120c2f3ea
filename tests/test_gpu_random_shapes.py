"""GPU parity on seeded random batch shapes: every case draws its own number of sequences, lengths
(with empty and one-token sequences), GQA ratio, compression mode per call (kept rows, int4 or int2
records, bf16 tail or none), verify windows, launch-shape tunables and host hints, and compares the
draft, verify and accept entry points with the oracle.  The point is the host logic that turns such a
batch into launches - split lengths, flat and grid launches, two- and four-wave workgroups, the
finish inside the split kernel, the tail as a partial of the split launch, the one-launch accept, row blocks - at combinations no hand-written case lists."""
import numpy as np
import pytest
import torch

from tests import helpers as H
from tests import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context(0)
    yield c
    c.close()


def _case(seed):
    rng = np.random.default_rng(7000 + seed)
    nseq = int(rng.choice([1, 2, 3, 5, 9, 17, 40, 64, 65, 70]))
    hkv = int(rng.choice([1, 2, 4]))
    g = int(rng.choice([1, 2, 4, 8]))
    # mostly short sequences so that the oracle stays quick, one long one per batch to make it ragged
    lens = [int(x) for x in rng.integers(0, 400, nseq)]
    lens[int(rng.integers(0, nseq))] = int(rng.integers(1500, 5000))
    if nseq > 2:
        lens[0], lens[1] = 1, 0
    if sum(lens) == 0:
        lens[-1] = 77
    keep, first, last = [], [], []
    for n in lens:
        k = int(rng.integers(0, n + 1)) if rng.random() < 0.8 else 0
        f = int(rng.integers(0, min(k, 8) + 1))
        keep.append(k)
        first.append(f)
        last.append(int(rng.integers(0, min(k - f, 8) + 1)))
    tails = [int(x) for x in rng.integers(0, 70, nseq)] if rng.random() < 0.7 else None
    wins = [int(x) for x in rng.integers(0, 12, nseq)]
    if rng.random() < 0.3:
        wins[int(rng.integers(0, nseq))] = int(rng.integers(33, 70))   # more than 256 rows at g = 8
    if sum(wins) == 0:
        wins[-1] = 3
    return rng, nseq, hkv, g, lens, keep, first, last, tails, wins


@pytest.mark.parametrize("seed", range(24))
def test_random_batch(lib, ctx, tunables, seed):
    rng, nseq, hkv, g, lens, keep, first, last, tails, wins = _case(seed)
    bits = int(rng.choice([4, 2]))
    print(f"[random] seed {seed}: {nseq} sequences, {hkv} KV heads x {g}, lengths up to {max(lens)}, int{bits}, "
          f"tails {'yes' if tails else 'no'}, windows up to {max(wins)}", flush=True)
    lay = synth.make_layer(8000 + seed, DEV, ctx_len=lens, n_q_heads=hkv * g, n_kv_heads=hkv, keep=keep, keep_first=first,
                           keep_last=last, quant_bits=(bits,), tail_len=tails, win=wins, vocab=int(rng.choice([7, 1001, 32000])),
                           bonus_row=bool(rng.random() < 0.5))
    # launch shapes: small splits so that these short lists are cut several times, either launch form
    tunables.set("VC_DRAFT_MIN_TOK", 128)
    tunables.set("VC_DRAFT_MIN_BLK", 4)
    tunables.set("VC_DRAFT_BF16_WGS", int(rng.choice([8, 64, 300])))
    tunables.set("VC_DRAFT_QUANT_WGS", int(rng.choice([8, 100, 700])))
    tunables.set("VC_DRAFT_FLAT", int(rng.integers(0, 2)))
    tunables.set("VC_DRAFT_ROW_WAVES", int(rng.choice([2, 4])))
    tunables.set("VC_VERIFY_MIN_TOK", int(rng.choice([64, 256, 1024])))
    tunables.set("VC_VERIFY_WGS", int(rng.choice([4, 64, 256])))
    tunables.set("VC_ACCEPT_FUSED", int(rng.integers(0, 2)))
    tunables.set("VC_DRAFT_FUSED", int(rng.choice([0, 64, 512])))
    hints = bool(rng.random() < 0.7)
    tunables.set("VC_DRAFT_TAIL_SPLIT", int(rng.integers(0, 2)))

    def check(tag, hint, **sel):
        kw = H.draft_kwargs(lay, **sel)
        if hints:
            kw.update(hint)
        out, lse = H.gpu_draft(lib, ctx, lay, **kw)
        ref, ref_lse = H.oracle_draft(lay, kw)
        assert H.rel_err(out, ref) <= H.TOL, f"seed {seed} {tag}"
        fin = np.isfinite(ref_lse)
        assert np.array_equal(np.isneginf(lse.cpu().numpy()), np.isneginf(ref_lse)), f"seed {seed} {tag}: empty rows"
        if fin.any():
            assert np.abs(lse.cpu().numpy()[fin] - ref_lse[fin]).max() <= H.LSE_TOL, f"seed {seed} {tag}: lse"

    use_tail = tails is not None or lay.tail_k is not None
    check("kept rows", dict(sum_keep=int(lay.cu_keep[-1])), use_pool=True, use_keep=True, use_tail=use_tail)
    check("records", dict(sum_blk=int(lay.cu_blk[bits][-1])), bits=bits, use_tail=use_tail)
    if seed % 3 == 0:
        check("contiguous rows", dict(sum_keep=int(sum(lens))), use_pool=True)

    out, lse = H.gpu_verify(lib, ctx, lay, sum_ctx=int(sum(lens)) if hints else 0)
    ref, ref_lse = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL, f"seed {seed} verify"
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= H.LSE_TOL, f"seed {seed} verify lse"

    a, n, am = H.gpu_accept(lib, ctx, lay)
    ra, rn, ram = H.oracle_accept(lay)
    assert np.array_equal(am, ram) and np.array_equal(a, ra) and np.array_equal(n, rn), f"seed {seed} accept"
