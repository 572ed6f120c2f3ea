"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times.
The oracle cannot do a whole full-size case in seconds, so it computes sampled outputs one by one
from CPU copies of the very same tensors, in worker processes: for the draft one query head of
EVERY (sequence, KV head) pair, for verify every window row of one (sequence, head) plus one row
of every other pair; accept_len / next_token / arg-max ids and kept-index lists are compared in full."""
import numpy as np
import pytest
import torch

from oracle import vc_oracle as O
from tests import synth
from tests import helpers as H
from tests import oracle_pool as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context(0)
    yield c
    c.close()


def seq_slice(lay, b):
    lo, hi = int(lay.cu_ctx[b]), int(lay.cu_ctx[b + 1])
    return lo, hi


def draft_task(lay, kw, b, h):
    """Oracle task for the draft output of (sequence b, query head h): per-pair CPU copies (numpy)."""
    g = lay.n_q_heads // lay.n_kv_heads
    kvh = h // g
    o = {}
    if "pool_k" in kw:
        lo, hi = seq_slice(lay, b)
        o.update(pool_k=H.bits16(kw["pool_k"][lo:hi, kvh:kvh + 1]), pool_v=H.bits16(kw["pool_v"][lo:hi, kvh:kvh + 1]),
                 cu_ctx=np.array([0, hi - lo]))
        if "keep_idx" in kw:
            cuk = kw["cu_keep"].cpu().numpy()
            nk = int(cuk[b + 1] - cuk[b])
            start = int(cuk[b]) * lay.n_kv_heads + kvh * nk
            o.update(keep_idx=kw["keep_idx"][start:start + nk].cpu().numpy(), cu_keep=np.array([0, nk]))
    if "blocks" in kw:
        cub = kw["cu_blk"].cpu().numpy()
        nb = int(cub[b + 1] - cub[b])
        start = int(cub[b]) * lay.n_kv_heads + kvh * nb
        o.update(blocks=kw["blocks"][start:start + nb].cpu().numpy(), cu_blk=np.array([0, nb]), bits=kw["bits"])
    if "tail_k" in kw:
        cut = kw["cu_tail"].cpu().numpy()
        lo, hi = int(cut[b]), int(cut[b + 1])
        o.update(tail_k=H.bits16(kw["tail_k"][lo:hi, kvh:kvh + 1]), tail_v=H.bits16(kw["tail_v"][lo:hi, kvh:kvh + 1]),
                 cu_tail=np.array([0, hi - lo]))
    return {"q": H.bits16(lay.q[b, h:h + 1]), "scale": lay.scale, "kv": o}


def verify_task(lay, b, h, rows):
    g = lay.n_q_heads // lay.n_kv_heads
    kvh = h // g
    lo, hi = seq_slice(lay, b)
    w0, w1 = int(lay.cu_win[b]), int(lay.cu_win[b + 1])
    return {"q_win": H.bits16(lay.q_win[w0:w1, h:h + 1]), "k_full": H.bits16(lay.k_full[lo:hi, kvh:kvh + 1]),
            "v_full": H.bits16(lay.v_full[lo:hi, kvh:kvh + 1]), "k_win": H.bits16(lay.k_win[w0:w1, kvh:kvh + 1]),
            "v_win": H.bits16(lay.v_win[w0:w1, kvh:kvh + 1]), "rows": list(rows), "scale": lay.scale}


def one_head_per_pair(lay, salt=0):
    """One query head of every (sequence, KV head) pair: the head inside the GQA group rotates."""
    g = lay.n_q_heads // lay.n_kv_heads
    return [(b, kvh * g + (b + kvh + salt) % g) for b in range(len(lay.ctx_len)) for kvh in range(lay.n_kv_heads)]


def assert_samples(tag, pairs):
    """pairs: (label, gpu row, oracle row, gpu lse, oracle lse).  The bound is the spec one,
    max|gpu - oracle| <= 1e-2 * max|oracle|, with the denominator taken from the oracle alone: the
    largest magnitude over all sampled oracle rows of the tensor."""
    denom = max(np.abs(ref).max() for (_, _, ref, _, _) in pairs)
    assert denom > 0
    worst = 0.0
    for (label, got, ref, got_lse, ref_lse) in pairs:
        err = np.abs(got - ref).max()
        worst = max(worst, err / denom)
        assert err <= H.TOL * denom, f"{tag} {label}: |gpu - oracle| {err:.3e} > {H.TOL} * {denom:.3e}"
        assert abs(got_lse - ref_lse) <= H.LSE_TOL, f"{tag} {label}: lse {got_lse} vs {ref_lse}"
    print(f"[full] {tag}: {len(pairs)} sampled outputs against the oracle, worst {worst:.2e} of max|oracle| {denom:.3f}", flush=True)


def check_draft_samples(lib, ctx, lay, kw, samples, tag):
    print(f"[full] draft {tag}: {len(samples)} samples", flush=True)
    out, lse = H.gpu_draft(lib, ctx, lay, **kw)
    outc, lsec = out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy()
    refs = P.run(P.draft_task, [draft_task(lay, kw, b, h) for (b, h) in samples])
    pairs = [(f"(seq {b}, head {h})", outc[b, h], r[0][0][0], lsec[b, h], r[0][0][1]) for (b, h), r in zip(samples, refs)]
    assert_samples(f"draft {tag}", pairs)
    assert torch.isfinite(out.float()).all()


def check_verify_samples(lib, ctx, lay, samples, tag, **kw):
    print(f"[full] verify {tag}: {len(samples)} samples", flush=True)
    out, lse = H.gpu_verify(lib, ctx, lay, **kw)
    outc, lsec = out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy()
    by_pair = {}
    for (b, i, h) in samples:
        by_pair.setdefault((b, h), []).append(i)
    keys = sorted(by_pair)
    refs = P.run(P.verify_task, [verify_task(lay, b, h, by_pair[(b, h)]) for (b, h) in keys])
    pairs = []
    for (b, h), res in zip(keys, refs):
        for i, (ref, ref_lse) in zip(by_pair[(b, h)], res):
            row = int(lay.cu_win[b]) + i
            pairs.append((f"(seq {b}, row {i}, head {h})", outc[row, h], ref, lsec[row, h], ref_lse))
    assert_samples(f"verify {tag}", pairs)
    assert torch.isfinite(out.float()).all()


def verify_samples(lay, full_seq, full_head, salt=0):
    """Every window row of (full_seq, full_head), plus one (row, head) of every other (sequence, KV head) pair."""
    s = [(full_seq, i, full_head) for i in range(lay.win[full_seq])]
    for (b, h) in one_head_per_pair(lay, salt):
        if lay.win[b] > 0 and not (b == full_seq and h == full_head):
            s.append((b, (5 * b + 3 * h + salt) % lay.win[b], h))
    return s


def check_accept_full(lib, ctx, lay):
    a, n, am = H.gpu_accept(lib, ctx, lay)
    ra, rn, ram = H.oracle_accept(lay)
    assert np.array_equal(am, ram) and np.array_equal(a, ra) and np.array_equal(n, rn)
    assert a.tolist() == lay.prefix_len


def test_config0_full(lib, ctx):
    lay = synth.config(0, DEV)
    kw = H.draft_kwargs(lay, bits=4)
    out, _ = H.gpu_draft(lib, ctx, lay, **kw)
    ref, _ = H.oracle_draft(lay, kw)
    assert H.rel_err(out, ref) <= H.TOL
    vout, _ = H.gpu_verify(lib, ctx, lay)
    vref, _ = H.oracle_verify(lay)
    assert H.rel_err(vout, vref) <= H.TOL
    check_accept_full(lib, ctx, lay)


def test_config1_full(lib, ctx):
    lay = synth.config(1, DEV)
    # kept lists: the library's complement of the dropped lists must equal the compressor's lists
    keep = torch.empty_like(lay.keep_idx)
    cu_keep = torch.empty_like(lay.cu_keep)
    lib.vc_keep_from_dropped(ctx, lay.dropped_idx, lay.cu_drop, lay.cu_ctx, lay.n_kv_heads, max(lay.ctx_len), keep, cu_keep)
    torch.cuda.synchronize()
    ref_keep, ref_cu = O.keep_from_dropped(H.npi(lay.dropped_idx), H.npi(lay.cu_drop), lay.ctx_len, lay.n_kv_heads)
    assert np.array_equal(keep.cpu().numpy(), ref_keep) and np.array_equal(cu_keep.cpu().numpy(), ref_cu)
    assert torch.equal(keep, lay.keep_idx)
    kw = H.draft_kwargs(lay, use_pool=True, use_keep=True)
    kw.update(keep_idx=keep, cu_keep=cu_keep, sum_keep=int(cu_keep[-1]))
    check_draft_samples(lib, ctx, lay, kw, one_head_per_pair(lay), "cfg1 gather")          # 64 (sequence, KV head) pairs
    check_verify_samples(lib, ctx, lay, verify_samples(lay, 2, 9), "cfg1 w16")
    check_accept_full(lib, ctx, lay)


def test_config2_full(lib, ctx):
    lay = synth.config(2, DEV)
    for bits in (4, 2):
        kw = H.draft_kwargs(lay, bits=bits)
        kw.update(sum_blk=int(lay.cu_blk[bits][-1]))
        check_draft_samples(lib, ctx, lay, kw, one_head_per_pair(lay, salt=bits), f"cfg2 int{bits}")   # 128 pairs each
    # full KV through pinned host memory in 8192-token chunks, verify waits on the last ticket
    host_k = torch.empty(lay.k_full.shape, dtype=torch.bfloat16, pin_memory=True); host_k.copy_(lay.k_full)
    host_v = torch.empty(lay.v_full.shape, dtype=torch.bfloat16, pin_memory=True); host_v.copy_(lay.v_full)
    dk = torch.full_like(lay.k_full, float("nan")); dv = torch.full_like(lay.v_full, float("nan"))
    row = lay.n_kv_heads * 128 * 2
    total = lay.k_full.shape[0]
    chunks = [(t * row, t * row, min(8192, total - t) * row) for t in range(0, total, 8192)]
    torch.cuda.synchronize()
    lib.vc_swap_in(ctx, host_k, dk, chunks)
    last = lib.vc_swap_in(ctx, host_v, dv, chunks) + len(chunks) - 1
    lib.vc_swap_wait(ctx, last)                       # device-side wait on the current stream
    check_verify_samples(lib, ctx, lay, verify_samples(lay, 8, 20), "cfg2 w32 after swap-in", k_full=dk, v_full=dv)
    assert torch.equal(dk, lay.k_full) and torch.equal(dv, lay.v_full)
    check_accept_full(lib, ctx, lay)


@pytest.mark.parametrize("layer", [0, 15, 31])
def test_config3_layers_full(lib, ctx, layer):
    """Layers 0, 15 and 31 of the 32-layer round (each layer has its own seeded KV), the draft at
    horizon steps 0, 1 and 63 (tail of 0, 1 and 63 drafted tokens), one head of every KV head."""
    lay = synth.config(3, DEV, layer=layer)
    for tail in (0, 1, 63):
        kw = H.draft_kwargs(lay, bits=4, use_tail=True)
        kw.update(cu_tail=torch.tensor([0, tail], dtype=torch.int32, device=DEV), sum_blk=int(lay.cu_blk[4][-1]))
        check_draft_samples(lib, ctx, lay, kw, one_head_per_pair(lay, salt=tail + layer), f"cfg3 layer {layer} int4 + tail {tail}")
    check_verify_samples(lib, ctx, lay, verify_samples(lay, 0, (7 * layer + 12) % 32, salt=layer), f"cfg3 layer {layer} w64")
    if layer == 0:
        check_accept_full(lib, ctx, lay)


def test_config4_ragged_full(lib, ctx):
    lay = synth.config(4, DEV)
    kw = H.draft_kwargs(lay, bits=4, use_pool=True, use_keep=True, use_tail=True)
    kw.update(sum_keep=int(lay.cu_keep[-1]), sum_blk=int(lay.cu_blk[4][-1]))
    check_draft_samples(lib, ctx, lay, kw, one_head_per_pair(lay), "cfg4 ragged mixed")      # 256 (sequence, KV head) pairs
    longest = int(np.argmax(lay.ctx_len))
    check_verify_samples(lib, ctx, lay, verify_samples(lay, longest, 5), "cfg4 ragged windows", sum_ctx=int(sum(lay.ctx_len)))
    check_accept_full(lib, ctx, lay)


def test_config2_compressor_side_full(lib, ctx):
    """Config-2 size: the library's quantiser reproduces the generator's records byte for byte (all
    16 x 8 x 2048 / 1024 records) and the oracle's for sampled (sequence, head) pairs; the inverse
    matches the oracle on the same samples; kept lists from scores match the oracle."""
    lay = synth.config(2, DEV)
    n = lay.ctx_len[0]
    for bits in (4, 2):
        print(f"[full] compress int{bits}", flush=True)
        nb = lay.max_blk[bits]
        blocks = torch.empty_like(lay.blocks[bits])
        lib.vc_compress_quant(ctx, lay.k_full, lay.v_full, lay.cu_ctx, lay.cu_blk[bits], bits, nb, blocks)
        torch.cuda.synchronize()
        assert torch.equal(blocks, lay.blocks[bits])
        ko = torch.empty_like(lay.k_full); vo = torch.empty_like(lay.v_full)
        lib.vc_decompress_quant(ctx, blocks, lay.cu_blk[bits], lay.cu_ctx, bits, nb, ko, vo)
        torch.cuda.synchronize()
        recs = blocks.view(len(lay.ctx_len), lay.n_kv_heads, nb, 5120)
        for (b, h) in [(0, 0), (11, 5)]:
            lo = b * n
            ref = O.quantize_records(H.bits16(lay.k_full[lo:lo + n, h:h + 1]), H.bits16(lay.v_full[lo:lo + n, h:h + 1]), bits)
            assert np.array_equal(recs[b, h].cpu().numpy(), ref[0])
            rk, rv = O.dequantize_records(ref, bits)
            assert np.array_equal(H.bits16(ko[lo:lo + n, h]), rk[:, 0]) and np.array_equal(H.bits16(vo[lo:lo + n, h]), rv[:, 0])
        del ko, vo, blocks
    print("[full] topk", flush=True)
    nseq, hkv, keep_n = len(lay.ctx_len), lay.n_kv_heads, n // 10
    scores = torch.randn(nseq * hkv * n, device=DEV, generator=synth.gen(99, DEV))
    cu_keep = torch.arange(0, (nseq + 1) * keep_n, keep_n, dtype=torch.int32, device=DEV)
    first = torch.full((nseq,), 64, dtype=torch.int32, device=DEV)
    last = torch.full((nseq,), 256, dtype=torch.int32, device=DEV)
    keep = torch.empty(nseq * hkv * keep_n, dtype=torch.int32, device=DEV)
    lib.vc_topk_keep(ctx, scores, lay.cu_ctx, cu_keep, hkv, keep, forced_first=first, forced_last=last)
    torch.cuda.synchronize()
    ref, _ = O.topk_keep(scores.cpu().numpy(), lay.ctx_len, [keep_n] * nseq, hkv, [64] * nseq, [256] * nseq)
    assert np.array_equal(keep.cpu().numpy(), ref)
