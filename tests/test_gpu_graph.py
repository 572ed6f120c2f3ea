"""The attention calls enqueue only kernels (no allocation, no synchronisation, no memset), so a
caller can capture a launch-bound decode step in a HIP graph.  Every replay - with eager work and
synchronisations in between, inputs and the tail length changed in place - must equal the eager
result bit for bit."""
import pytest
import torch

import paper_2605_17613_amd as vc
from tests import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


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


def test_captured_draft_and_verify_replays_equal_eager(lib, ctx):
    dev = "cuda:0"
    lay = synth.make_layer(synth.SEED_BASE + 91, dev, ctx_len=[4096, 2048 + 96, 1024], n_q_heads=8, n_kv_heads=2,
                           keep=[512, 300, 128], keep_first=16, keep_last=32, quant_bits=(4,), tail_len=[24, 24, 24],
                           win=[8, 5, 16], vocab=0)
    nseq = 3
    cu_tail = lay.cu_tail.clone()
    kq = H.draft_kwargs(lay, bits=4, use_tail=True); kq["cu_tail"] = cu_tail
    kg = H.draft_kwargs(lay, use_pool=True, use_keep=True, use_tail=True); kg["cu_tail"] = cu_tail
    # both sources in one call (as for a batch that mixes compressors)
    kb = H.draft_kwargs(lay, bits=4, use_pool=True, use_keep=True, use_tail=True); kb["cu_tail"] = cu_tail
    q = lay.q.clone()
    out_q, out_g = torch.empty_like(q), torch.empty_like(q)
    out_b = torch.empty_like(q)
    vout = torch.empty_like(lay.q_win)
    vargs = dict(k=lay.k_full, v=lay.v_full, cu_ctx=lay.cu_ctx, max_ctx=max(lay.ctx_len), max_win=max(lay.win))
    ws = torch.empty(max(vc.vc_draft_workspace_bytes(8, 2, nseq, **kq), vc.vc_draft_workspace_bytes(8, 2, nseq, **kg),
                         vc.vc_draft_workspace_bytes(8, 2, nseq, **kb),
                         vc.vc_verify_workspace_bytes(8, 2, nseq, total_win=lay.q_win.shape[0], **vargs)),
                     dtype=torch.uint8, device=dev)

    def step():
        vc.vc_draft_attn(ctx, q, lay.scale, out_q, n_kv_heads=2, workspace=ws, **kq)
        vc.vc_draft_attn(ctx, q, lay.scale, out_g, n_kv_heads=2, workspace=ws, **kg)
        vc.vc_draft_attn(ctx, q, lay.scale, out_b, n_kv_heads=2, workspace=ws, **kb)
        vc.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, vout, n_seqs=nseq, workspace=ws, **vargs)

    step()                                    # first calls set kernel attributes: outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    g = synth.gen(5, dev)
    tails = [lay.cu_tail.clone(), torch.tensor([0, 3, 3 + 24, 3 + 24 + 10], dtype=torch.int32, device=dev),
             torch.tensor([0, 0, 0, 0], dtype=torch.int32, device=dev), lay.cu_tail.clone()]
    for rep, ct in enumerate(tails):
        q.copy_(synth.randn_bf16(tuple(q.shape), g))
        # the tails of a sequence stay where they are; only their lengths change (offsets are the
        # original ones, so shorter tails are read from the same rows)
        cu_tail.copy_(lay.cu_tail if rep in (0, 3) else ct)
        if rep in (1, 2):
            cu_tail.copy_(ct)
        torch.cuda.synchronize()
        step()
        torch.cuda.synchronize()
        want = (out_q.clone(), out_g.clone(), vout.clone(), out_b.clone())
        out_q.zero_(); out_g.zero_(); vout.zero_(); out_b.zero_()
        scratch = torch.randn(1 << 20, device=dev).sum()      # unrelated eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_q.view(torch.int16), want[0].view(torch.int16)), rep
        assert torch.equal(out_g.view(torch.int16), want[1].view(torch.int16)), rep
        assert torch.equal(vout.view(torch.int16), want[2].view(torch.int16)), rep
        assert torch.equal(out_b.view(torch.int16), want[3].view(torch.int16)), rep
        assert torch.isfinite(scratch)


def test_captured_accept_replays_equal_eager(lib, ctx):
    """The one-launch accept counts its workgroups on counters of the context that it leaves at zero:
    a captured call is replayed with eager calls (which use other counter sets, and after 16 of them the
    same one) in between, drafted ids changed in place."""
    dev = "cuda:0"
    lay = synth.make_layer(synth.SEED_BASE + 92, dev, ctx_len=[8] * 4, n_q_heads=4, n_kv_heads=2, win=[5, 1, 9, 3],
                           vocab=32000, bonus_row=True, prefix_len=[5, 0, 4, 3])
    nseq, rows = 4, lay.logits.shape[0]
    ids = lay.draft_ids.clone()
    acc, nxt = (torch.full((nseq,), -7, dtype=torch.int32, device=dev) for _ in range(2))
    amax = torch.full((rows,), -7, dtype=torch.int32, device=dev)
    ws = torch.empty(max(vc.vc_accept_workspace_bytes(rows, 32000), 16), dtype=torch.uint8, device=dev)

    def step():
        vc.vc_accept_len(ctx, lay.logits, lay.cu_rows, ids, lay.cu_win, acc, nxt, amax, workspace=ws)

    step()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    g = torch.Generator(device=dev)
    g.manual_seed(3)
    for rep in range(4):
        ids.copy_(lay.draft_ids)
        if rep:
            flip = torch.randint(0, ids.numel(), (2,), generator=g, device=dev)
            ids[flip] += 1                                       # a mismatch somewhere else every time
        for _ in range(5 + 6 * rep):                             # eager calls walk through the counter sets
            step()
        torch.cuda.synchronize()
        want = (acc.clone(), nxt.clone(), amax.clone())
        acc.fill_(-7); nxt.fill_(-7); amax.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(acc, want[0]) and torch.equal(nxt, want[1]) and torch.equal(amax, want[2]), rep
    assert acc.tolist() != [-7] * nseq
