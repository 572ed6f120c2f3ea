"""Ragged verify launches that run from the device-built work list (pieces of per-sequence length
taken off a queue by one workgroup per CU): results against the oracle, streamed launches against
the one-shot call bit for bit, and the walk over every (sequence, chunk) that replaces a list too
long to hold.  The tunable VC_VERIFY_LIST_MIN = 0 sends these small batches down the path large ones take."""
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


def _kv(lay, ctx_len, win, **extra):
    return dict(k=lay.k_full, v=lay.v_full, cu_ctx=lay.cu_ctx, max_ctx=max(ctx_len), max_win=max(win),
                n_seqs=len(ctx_len), **extra)


@pytest.mark.parametrize("ctx_len,win,hq,hkv", [
    ([5000, 2048, 700, 9000], [16, 5, 33, 64], 8, 2),           # rows 64, 20, 132, 256: both cost classes
    ([12000, 300, 0, 4100, 6000, 2500], [40, 3, 7, 0, 64, 1], 16, 4),   # an empty context and an empty window
    ([3000, 20000], [80, 9], 8, 2),                             # 320 rows: two row blocks per KV head
])
def test_worklist_verify_matches_oracle(lib, ctx, tunables, ctx_len, win, hq, hkv):
    tunables.set("VC_VERIFY_LIST_MIN", 0)
    lay = synth.make_layer(95, DEV, ctx_len=ctx_len, n_q_heads=hq, n_kv_heads=hkv, win=win)
    kv = _kv(lay, ctx_len, win, sum_ctx=sum(ctx_len))
    tw = lay.q_win.shape[0]
    nbytes = lib.vc_verify_workspace_bytes(hq, hkv, total_win=tw, **kv)
    tunables.set("VC_VERIFY_WORKLIST", 0)
    plain = lib.vc_verify_workspace_bytes(hq, hkv, total_win=tw, **kv)
    tunables.set("VC_VERIFY_WORKLIST", 1)
    assert nbytes > plain                                        # the list is on: its area follows the partials
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=DEV)       # poison (NaN partials, huge counters)
    out = torch.empty_like(lay.q_win)
    lse = torch.empty((tw, hq), dtype=torch.float32, device=DEV)
    for _ in range(2):                                           # the second call finds the first one's list and counter
        lib.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, out, workspace=ws, lse=lse, **kv)
    torch.cuda.synchronize()
    ref, ref_lse = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= H.LSE_TOL


def test_few_resident_workgroups_take_many_pieces_each(lib, ctx, tunables):
    """Three resident workgroups instead of one per CU: each takes dozens of pieces in turn, of both row
    variants, reusing its LDS ring every time; the result is the same bits as with the full grid."""
    tunables.set("VC_VERIFY_LIST_MIN", 0)
    ctx_len, win = [9000, 2048, 700, 5000, 3300], [64, 5, 33, 16, 40]
    lay = synth.make_layer(94, DEV, ctx_len=ctx_len, n_q_heads=8, n_kv_heads=2, win=win)
    kv = _kv(lay, ctx_len, win, sum_ctx=sum(ctx_len))
    tw = lay.q_win.shape[0]
    ws = torch.empty(lib.vc_verify_workspace_bytes(8, 2, total_win=tw, **kv), dtype=torch.uint8, device=DEV)
    out_full = torch.empty_like(lay.q_win)
    lib.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, out_full, workspace=ws, **kv)
    tunables.set("VC_VERIFY_QUEUE_WGS", 3)
    out_few = torch.empty_like(lay.q_win)
    lib.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, out_few, workspace=ws, **kv)
    torch.cuda.synchronize()
    assert torch.equal(out_full.view(torch.int16), out_few.view(torch.int16))
    ref, _ = H.oracle_verify(lay)
    assert H.rel_err(out_few, ref) <= H.TOL


def test_worklist_streamed_launches_equal_one_shot(lib, ctx, tunables):
    tunables.set("VC_VERIFY_LIST_MIN", 0)
    ctx_len, win, chunk = [7000, 2048, 700, 3100], [16, 5, 33, 64], 1024
    lay = synth.make_layer(96, DEV, ctx_len=ctx_len, n_q_heads=8, n_kv_heads=2, win=win)
    kv = _kv(lay, ctx_len, win, sum_ctx=sum(ctx_len), chunk_tokens=chunk)
    tw = lay.q_win.shape[0]
    nbytes = lib.vc_verify_workspace_bytes(8, 2, total_win=tw, **kv)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    out1 = torch.empty_like(lay.q_win)
    lib.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, out1, workspace=ws, **kv)
    # the same verify as launches over token ranges (all sequences), then over sequence ranges
    ws2 = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    total_max = max(ctx_len) + max(win)
    for t0 in range(0, total_max, 2 * chunk):
        last = t0 + 2 * chunk >= total_max
        lib.vc_verify_attn_range(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, 0, 4, t0,
                                 (1 << 30) if last else t0 + 2 * chunk, workspace=ws2, **kv)
    out2 = torch.empty_like(out1)
    lib.vc_verify_finish(ctx, lay.cu_win, out2, n_q_heads=8, n_kv_heads=2, workspace=ws2, **kv)
    ws3 = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    for b0, b1 in ((2, 4), (0, 1), (1, 2)):
        lib.vc_verify_attn_range(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, b0, b1, 0, 1 << 30,
                                 workspace=ws3, **kv)
    out3 = torch.empty_like(out1)
    lib.vc_verify_finish(ctx, lay.cu_win, out3, n_q_heads=8, n_kv_heads=2, workspace=ws3, **kv)
    torch.cuda.synchronize()
    assert torch.equal(out1.view(torch.int16), out2.view(torch.int16))
    assert torch.equal(out1.view(torch.int16), out3.view(torch.int16))
    ref, _ = H.oracle_verify(lay)
    assert H.rel_err(out1, ref) <= H.TOL


def test_worklist_overflow_walks_every_chunk(lib, ctx, tunables):
    """A caller that understates sum_ctx gets a list with room for too few pieces; the kernels then
    walk every (sequence, chunk) of the launch, with the same results."""
    tunables.set("VC_VERIFY_LIST_MIN", 0)
    ctx_len, win = [150000, 50000, 128], [4, 2, 1]
    lay = synth.make_layer(97, DEV, ctx_len=ctx_len, n_q_heads=8, n_kv_heads=2, win=win)
    kv = _kv(lay, ctx_len, win, sum_ctx=20000, chunk_tokens=128)        # 1564 pieces exist, the bound says 160
    tw = lay.q_win.shape[0]
    ws = torch.empty(lib.vc_verify_workspace_bytes(8, 2, total_win=tw, **kv), dtype=torch.uint8, device=DEV)
    out = torch.empty_like(lay.q_win)
    lib.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, out, workspace=ws, **kv)
    torch.cuda.synchronize()
    ref, _ = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL


def test_worklist_verify_in_a_captured_graph(lib, ctx, tunables):
    """The list kernel zeroes the queue's counter itself, so a captured verify replays correctly: every
    replay, with the queries changed in place and eager work in between, equals the eager call."""
    tunables.set("VC_VERIFY_LIST_MIN", 0)
    ctx_len, win = [6000, 1500, 300, 4100], [16, 40, 3, 64]
    lay = synth.make_layer(98, DEV, ctx_len=ctx_len, n_q_heads=8, n_kv_heads=2, win=win)
    kv = _kv(lay, ctx_len, win, sum_ctx=sum(ctx_len))
    tw = lay.q_win.shape[0]
    ws = torch.empty(lib.vc_verify_workspace_bytes(8, 2, total_win=tw, **kv), dtype=torch.uint8, device=DEV)
    qw = lay.q_win.clone()
    out = torch.empty_like(qw)

    def step():
        lib.vc_verify_attn(ctx, qw, lay.k_win, lay.v_win, lay.cu_win, lay.scale, out, workspace=ws, **kv)

    step()                                    # first call sets kernel attributes: outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    g = synth.gen(6, DEV)
    for rep in range(3):
        qw.copy_(synth.randn_bf16(tuple(qw.shape), g))
        torch.cuda.synchronize()
        step()
        torch.cuda.synchronize()
        want = out.clone()
        out.zero_()
        scratch = torch.randn(1 << 20, device=DEV).sum()      # unrelated eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16)), rep
        assert torch.isfinite(scratch)
    lay.q_win.copy_(qw)
    ref, _ = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL


@pytest.mark.parametrize("nseq", [400, 600])
def test_many_short_sequences(lib, ctx, tunables, nseq):
    """400 sequences still go through the list (its ranking loops run over all of them); 600 are more
    than a list holds and take the plain grid."""
    tunables.set("VC_VERIFY_LIST_MIN", 0)
    rng = np.random.default_rng(nseq)
    ctx_len = [int(x) for x in rng.integers(0, 700, nseq)]
    ctx_len[7] = 5000                                            # one long sequence makes the batch ragged
    win = [int(x) for x in rng.integers(0, 5, nseq)]
    win[7] = 40
    lay = synth.make_layer(99, DEV, ctx_len=ctx_len, n_q_heads=8, n_kv_heads=2, win=win)
    kv = _kv(lay, ctx_len, win, sum_ctx=sum(ctx_len))
    tw = lay.q_win.shape[0]
    nbytes = lib.vc_verify_workspace_bytes(8, 2, total_win=tw, **kv)
    tunables.set("VC_VERIFY_WORKLIST", 0)
    plain = lib.vc_verify_workspace_bytes(8, 2, total_win=tw, **kv)
    tunables.set("VC_VERIFY_WORKLIST", 1)
    assert (nbytes > plain) == (nseq <= 512)
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=DEV)
    out = torch.empty_like(lay.q_win)
    lib.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, out, workspace=ws, **kv)
    torch.cuda.synchronize()
    ref, _ = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL
