"""Chunk-streamed verify: the full KV arrives from pinned host memory chunk by chunk and every
chunk is attended to as soon as its ticket has been waited for; the merged result must equal the
one-shot call bit for bit and match the oracle."""
import numpy as np
import pytest
import torch

from tests import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("ctx_len,win,chunk", [([5000, 2048, 700], [16, 5, 33], 1024), ([9000], [64], 2048),
                                               ([300, 4096], [1, 8], 4096)])
def test_streamed_verify_equals_one_shot_and_oracle(lib, ctx, ctx_len, win, chunk):
    lay = synth.make_layer(90, DEV, ctx_len=ctx_len, n_q_heads=8, n_kv_heads=2, win=win)
    nseq = len(ctx_len)
    hk = torch.empty(lay.k_full.shape, dtype=torch.bfloat16, pin_memory=True); hk.copy_(lay.k_full)
    hv = torch.empty(lay.v_full.shape, dtype=torch.bfloat16, pin_memory=True); hv.copy_(lay.v_full)
    dk = torch.full_like(lay.k_full, float("nan")); dv = torch.full_like(lay.v_full, float("nan"))   # poison
    torch.cuda.synchronize()
    args = dict(k=dk, v=dv, cu_ctx=lay.cu_ctx, max_ctx=max(ctx_len), max_win=max(win), n_seqs=nseq, chunk_tokens=chunk)
    plan_chunk, n_chunks = lib.vc_verify_plan(8, 2, nseq, k=dk, v=dv, cu_ctx=lay.cu_ctx, max_ctx=max(ctx_len),
                                              max_win=max(win), chunk_tokens=chunk)
    assert plan_chunk == chunk and n_chunks == -(-(max(ctx_len) + max(win)) // chunk)
    tw = lay.q_win.shape[0]
    nbytes = lib.vc_verify_workspace_bytes(8, 2, nseq, total_win=tw, k=dk, v=dv, cu_ctx=lay.cu_ctx,
                                           max_ctx=max(ctx_len), max_win=max(win), chunk_tokens=chunk)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    row = 2 * 128 * 2
    for b in range(nseq):
        lo = int(lay.cu_ctx[b])
        n = ctx_len[b]
        for t0 in range(0, n, chunk):
            t1 = min(n, t0 + chunk)
            c = [((lo + t0) * row, (lo + t0) * row, (t1 - t0) * row)]
            lib.vc_swap_in(ctx, hk, dk, c)
            ticket = lib.vc_swap_in(ctx, hv, dv, c)
            lib.vc_swap_wait(ctx, ticket)             # the compute stream waits for this chunk only
            last = t1 == n
            lib.vc_verify_attn_range(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, b, b + 1, t0,
                                     (1 << 30) if last else t1, workspace=ws, **args)
    out = torch.empty_like(lay.q_win)
    lse = torch.empty((tw, 8), dtype=torch.float32, device=DEV)
    lib.vc_verify_finish(ctx, lay.cu_win, out, n_q_heads=8, n_kv_heads=2, workspace=ws, lse=lse, **args)
    torch.cuda.synchronize()
    assert torch.equal(dk, lay.k_full) and torch.equal(dv, lay.v_full)
    assert torch.isfinite(out.float()).all()
    # one-shot call with the same chunking: identical arithmetic, identical bits
    ws2 = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    out2 = torch.empty_like(out)
    lib.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, out2, workspace=ws2, **args)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
    ref, ref_lse = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= H.LSE_TOL


def test_range_alignment_is_enforced(lib, ctx):
    lay = synth.make_layer(91, DEV, ctx_len=[3000], n_q_heads=8, n_kv_heads=2, win=[4])
    args = dict(k=lay.k_full, v=lay.v_full, cu_ctx=lay.cu_ctx, max_ctx=3000, max_win=4, n_seqs=1, chunk_tokens=1024)
    ws = torch.empty(lib.vc_verify_workspace_bytes(8, 2, 1, total_win=4, k=lay.k_full, v=lay.v_full, cu_ctx=lay.cu_ctx,
                                                   max_ctx=3000, max_win=4, chunk_tokens=1024), dtype=torch.uint8, device=DEV)
    with pytest.raises(lib.VcError) as e:
        lib.vc_verify_attn_range(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, 0, 1, 512, 1024, workspace=ws, **args)
    assert e.value.status == 1
    with pytest.raises(lib.VcError) as e:
        lib.vc_verify_attn_range(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, 0, 1, 0, 1500, workspace=ws, **args)
    assert e.value.status == 1
    with pytest.raises(lib.VcError) as e:
        lib.vc_verify_attn_range(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, 0, 2, 0, 1024, workspace=ws, **args)
    assert e.value.status == 1


def _one_shot(lib, ctx, lay, ctx_len, win, chunk):
    nseq = len(ctx_len)
    args = dict(k=lay.k_full, v=lay.v_full, cu_ctx=lay.cu_ctx, max_ctx=max(ctx_len), max_win=max(win), n_seqs=nseq,
                chunk_tokens=chunk)
    tw = lay.q_win.shape[0]
    nbytes = lib.vc_verify_workspace_bytes(8, 2, nseq, total_win=tw, k=lay.k_full, v=lay.v_full, cu_ctx=lay.cu_ctx,
                                           max_ctx=max(ctx_len), max_win=max(win), chunk_tokens=chunk)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    out = torch.empty_like(lay.q_win)
    lib.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, out, workspace=ws, **args)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("slots", [2, 3])
@pytest.mark.parametrize("ctx_len,win,chunk", [([5000, 2048, 700], [16, 5, 33], 1024), ([9000], [64], 2048)])
def test_verify_through_a_staging_ring(lib, ctx, slots, ctx_len, win, chunk):
    """The full KV never exists on the device: every (sequence, chunk) is copied into slot i mod R of a
    ring of R chunks and attended to from there; a slot is reloaded only after the range call that read it
    (vc_swap_after).  Bits equal the one-shot verify over a resident full KV; values match the oracle."""
    lay = synth.make_layer(92, DEV, ctx_len=ctx_len, n_q_heads=8, n_kv_heads=2, win=win)
    nseq = len(ctx_len)
    hk = torch.empty(lay.k_full.shape, dtype=torch.bfloat16, pin_memory=True); hk.copy_(lay.k_full)
    hv = torch.empty(lay.v_full.shape, dtype=torch.bfloat16, pin_memory=True); hv.copy_(lay.v_full)
    ring_k = torch.full((slots * chunk, 2, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    ring_v = torch.full_like(ring_k, float("nan"))
    row = 2 * 128 * 2
    # the stream of (sequence, chunk) pieces; the last piece of a sequence may hold fewer full-KV rows than a
    # slot, or none at all (window tokens only)
    pieces = []
    for b in range(nseq):
        lo, n = int(lay.cu_ctx[b]), ctx_len[b]
        for t0 in range(0, n + win[b], chunk):
            pieces.append((b, t0, lo + t0, max(0, min(n, t0 + chunk) - t0), t0 + chunk >= n + win[b]))
    slot_of = [torch.zeros(nseq, dtype=torch.int32, device=DEV) for _ in pieces]
    for i, (b, _, _, _, _) in enumerate(pieces):
        slot_of[i][b] = i % slots
    desc = dict(k=ring_k, v=ring_v, cu_ctx=lay.cu_ctx, max_ctx=max(ctx_len), max_win=max(win), n_seqs=nseq,
                chunk_tokens=chunk, ring_slots=slots)
    tw = lay.q_win.shape[0]
    qargs = {k: v for k, v in desc.items() if k != "n_seqs"}
    ws = torch.empty(lib.vc_verify_workspace_bytes(8, 2, nseq, total_win=tw, ring_slot=slot_of[0], **qargs),
                     dtype=torch.uint8, device=DEV)
    torch.cuda.synchronize()

    def issue(i):
        b, t0, src_row, rows, _ = pieces[i]
        c = [(src_row * row, (i % slots) * chunk * row, rows * row)]
        lib.vc_swap_in(ctx, hk, ring_k, c)
        return lib.vc_swap_in(ctx, hv, ring_v, c)

    tickets = {i: issue(i) for i in range(min(slots, len(pieces)))}
    for i, (b, t0, _, _, last) in enumerate(pieces):
        lib.vc_swap_wait(ctx, tickets[i])
        lib.vc_verify_attn_range(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, b, b + 1, t0,
                                 (1 << 30) if last else t0 + chunk, workspace=ws, ring_slot=slot_of[i], **desc)
        if i + slots < len(pieces):
            lib.vc_swap_after(ctx, lib.vc_mark(ctx))      # slot i mod R is free once this range call has run
            tickets[i + slots] = issue(i + slots)
    out = torch.empty_like(lay.q_win)
    lse = torch.empty((tw, 8), dtype=torch.float32, device=DEV)
    lib.vc_verify_finish(ctx, lay.cu_win, out, n_q_heads=8, n_kv_heads=2, workspace=ws, lse=lse, ring_slot=slot_of[0], **desc)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    assert torch.equal(out.view(torch.int16), _one_shot(lib, ctx, lay, ctx_len, win, chunk).view(torch.int16))
    ref, ref_lse = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= H.LSE_TOL


def test_ring_launches_batched_over_sequences(lib, ctx):
    """Chunk c of every sequence is in flight together (two slots per sequence) and one range call per c
    attends to all sequences at once, each from its own slot."""
    ctx_len, win, chunk = [3000, 2048, 5000, 900], [8, 5, 33, 64], 1024
    lay = synth.make_layer(93, DEV, ctx_len=ctx_len, n_q_heads=8, n_kv_heads=2, win=win)
    nseq = len(ctx_len)
    slots = 2 * nseq
    hk = torch.empty(lay.k_full.shape, dtype=torch.bfloat16, pin_memory=True); hk.copy_(lay.k_full)
    hv = torch.empty(lay.v_full.shape, dtype=torch.bfloat16, pin_memory=True); hv.copy_(lay.v_full)
    ring_k = torch.full((slots * chunk, 2, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    ring_v = torch.full_like(ring_k, float("nan"))
    row = 2 * 128 * 2
    n_chunks = -(-(max(n + w for n, w in zip(ctx_len, win))) // chunk)
    slot_tab = [torch.tensor([(c % 2) * nseq + b for b in range(nseq)], dtype=torch.int32, device=DEV) for c in range(2)]
    desc = dict(k=ring_k, v=ring_v, cu_ctx=lay.cu_ctx, max_ctx=max(ctx_len), max_win=max(win), n_seqs=nseq,
                chunk_tokens=chunk, ring_slots=slots)
    tw = lay.q_win.shape[0]
    qargs = {k: v for k, v in desc.items() if k != "n_seqs"}
    ws = torch.empty(lib.vc_verify_workspace_bytes(8, 2, nseq, total_win=tw, ring_slot=slot_tab[0], **qargs),
                     dtype=torch.uint8, device=DEV)
    torch.cuda.synchronize()

    def issue(c):
        chunks = []
        for b in range(nseq):
            t0 = c * chunk
            rows = max(0, min(ctx_len[b], t0 + chunk) - t0)
            chunks.append(((int(lay.cu_ctx[b]) + t0) * row, ((c % 2) * nseq + b) * chunk * row, rows * row))
        lib.vc_swap_in(ctx, hk, ring_k, chunks)
        return lib.vc_swap_in(ctx, hv, ring_v, chunks) + nseq - 1

    tickets = {c: issue(c) for c in range(min(2, n_chunks))}
    for c in range(n_chunks):
        lib.vc_swap_wait(ctx, tickets[c])
        lib.vc_verify_attn_range(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, 0, nseq, c * chunk,
                                 (1 << 30) if c == n_chunks - 1 else (c + 1) * chunk, workspace=ws, ring_slot=slot_tab[c % 2], **desc)
        if c + 2 < n_chunks:
            lib.vc_swap_after(ctx, lib.vc_mark(ctx))
            tickets[c + 2] = issue(c + 2)
    out = torch.empty_like(lay.q_win)
    lib.vc_verify_finish(ctx, lay.cu_win, out, n_q_heads=8, n_kv_heads=2, workspace=ws, ring_slot=slot_tab[0], **desc)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), _one_shot(lib, ctx, lay, ctx_len, win, chunk).view(torch.int16))
    ref, _ = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL
    # a ring descriptor is refused by the one-shot call and by a range that spans two chunks
    with pytest.raises(lib.VcError):
        lib.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, out, workspace=ws, ring_slot=slot_tab[0], **desc)
    with pytest.raises(lib.VcError):
        lib.vc_verify_attn_range(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, 0, nseq, 0, 2 * chunk, workspace=ws,
                                 ring_slot=slot_tab[0], **desc)
