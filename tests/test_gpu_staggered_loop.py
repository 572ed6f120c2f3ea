"""The execution loop of the paper's section 5.2 on the GPU, driven by the library's admission
control: every verify the loop runs (on KV that was reloaded from pinned host memory under its
ticket) must equal a one-shot verify of the same request and window over resident KV, and its
accept result must equal the oracle's."""
import numpy as np
import pytest
import torch

import paper_2605_17613_amd as vc
from oracle import vc_oracle as O
from tests import synth
from paper_2605_17613_amd.runtime import StaggeredLayer
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


def test_staggered_loop_verifies_match_one_shot_and_oracle(lib, ctx):
    dev = "cuda:0"
    R, W, X = 5, 12, 5
    lens = [2048, 1536, 4096, 1024, 2560]
    lay = synth.make_layer(synth.SEED_BASE + 77, dev, ctx_len=lens, n_q_heads=8, n_kv_heads=2, quant_bits=(4,),
                           win=[W] * R, vocab=1000)
    host_k = torch.empty(lay.k_full.shape, dtype=torch.bfloat16, pin_memory=True); host_k.copy_(lay.k_full)
    host_v = torch.empty(lay.v_full.shape, dtype=torch.bfloat16, pin_memory=True); host_v.copy_(lay.v_full)
    # a link slow enough (in the model) that reloads span several windows and cannot all share one
    kv = 2.0 * 2048 * 2 * 256
    loop = StaggeredLayer(ctx, lay, 4, host_k, host_v, windows=W, x=X, t_iter=1e-3, link_bw=kv / 2.5e-3,
                          hbm_bytes=1e12, chunk_tokens=512)
    loop.stage_k.fill_(float("nan")); loop.stage_v.fill_(float("nan"))
    snaps = []
    orig = loop._verify

    def verify_and_snapshot(it, r):
        cnt = min(loop.drafted[r], W)
        orig(it, r)
        w0 = loop.w0[r]
        snaps.append((it, r, cnt, loop.vout[w0:w0 + cnt].clone(), loop.acc[r:r + 1].clone(), loop.nxt[r:r + 1].clone()))

    loop._verify = verify_and_snapshot
    log = loop.run(60)
    torch.cuda.synchronize(); vc.vc_swap_sync(ctx)
    assert len(log) == len(snaps) >= 2 * R and {r for (_, r, _) in log} == set(range(R))
    assert all(1 <= c <= W for (_, _, c) in log)
    # every reloaded request's staging rows are the host's bytes
    for r in {r for (_, r, _) in log}:
        lo, n = loop.c0[r], lens[r]
        assert torch.equal(loop.stage_k[lo:lo + n].view(torch.int16), lay.k_full[lo:lo + n].view(torch.int16))
        assert torch.equal(loop.stage_v[lo:lo + n].view(torch.int16), lay.v_full[lo:lo + n].view(torch.int16))
    # spacing: a request verifies again only after at least one draft, and the reserve rings are
    # respected (never more link time booked in a window than the window holds)
    t_ring, _, _ = loop.sched.rings()
    assert max(t_ring) <= 1e-3
    cu_cnt = {c: torch.tensor([0, c], dtype=torch.int32, device=dev) for c in range(W + 1)}
    for (it, r, cnt, out, acc, nxt) in snaps[:: max(1, len(snaps) // 12)]:
        lo, n, w0, r0 = loop.c0[r], lens[r], loop.w0[r], loop.r0[r]
        # one-shot verify over the resident KV
        args = dict(k=lay.k_full[lo:lo + n], v=lay.v_full[lo:lo + n], cu_ctx=loop.cu_ctx1[r], max_ctx=n, max_win=W, sum_ctx=n)
        ws = torch.empty(vc.vc_verify_workspace_bytes(8, 2, 1, total_win=W, **args), dtype=torch.uint8, device=dev)
        ref = torch.empty_like(out)
        vc.vc_verify_attn(ctx, lay.q_win[w0:w0 + cnt], lay.k_win[w0:w0 + cnt], lay.v_win[w0:w0 + cnt], cu_cnt[cnt],
                          lay.scale, ref, n_seqs=1, workspace=ws, **args)
        torch.cuda.synchronize()
        assert torch.equal(ref.view(torch.int16), out.view(torch.int16)), (it, r, cnt)
        # ... and the oracle
        want, _ = O.verify_attn(H.bits16(lay.q_win[w0:w0 + cnt]), H.bits16(lay.k_full[lo:lo + n]), H.bits16(lay.v_full[lo:lo + n]),
                                H.bits16(lay.k_win[w0:w0 + cnt]), H.bits16(lay.v_win[w0:w0 + cnt]),
                                np.array([0, n], dtype=np.int32), np.array([0, cnt], dtype=np.int32), lay.scale,
                                n_q_heads=8, n_kv_heads=2)
        assert H.rel_err(out, want) <= H.TOL
        a, nx, _ = O.accept(H.npi(lay.logits[r0:r0 + cnt]), np.array([0, cnt], dtype=np.int32),
                            H.npi(lay.draft_ids[w0:w0 + cnt]), np.array([0, cnt], dtype=np.int32))
        assert int(acc) == int(a[0]) and int(nxt) == int(nx[0])
