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
