"""The draft entry point that allocates nothing (vc_draft_attn_static): called through the C ABI twice
in a row, the second time on a smaller batch (so that the scratch still holds the first call's
partials), and compared with vc_draft_attn on the same inputs (same kernels: equal bits) and with the
oracle (the usual bound for bf16 attention outputs).  Also: a batch too large for the scratch is
refused, and the call really leaves the device allocator alone."""
import numpy as np
import pytest
import torch

from tests import helpers as H
from tests import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _static_draft(lib, ctx, lay, kw):
    nseq = lay.q.shape[0]
    out = torch.full_like(lay.q, float("nan"))
    lse = torch.full((nseq, lay.n_q_heads), float("nan"), dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    free_before, _ = torch.cuda.mem_get_info()
    lib.vc_draft_attn_static(ctx, lay.q, lay.scale, out, n_kv_heads=lay.n_kv_heads, lse=lse, **kw)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before                  # no device allocation behind torch's back either
    return out, lse


def test_static_draft_twice_second_smaller(lib):
    ctx = lib.Context(0)
    try:
        assert lib.vc_draft_static_scratch_bytes() == 8 << 20
        big = synth.make_layer(301, DEV, ctx_len=[32 * 300 + 7, 32 * 41, 32 * 128], n_q_heads=8, n_kv_heads=2,
                               keep=[900, 0, 64], keep_first=[8, 0, 2], keep_last=[16, 0, 4], quant_bits=(4,),
                               tail_len=[5, 0, 33])
        small = synth.make_layer(302, DEV, ctx_len=[32 * 9 + 3], n_q_heads=8, n_kv_heads=2, quant_bits=(4,), tail_len=[2])
        for tag, lay, sel in (("first call: three sequences, kept rows + int4 records + tail", big,
                               dict(bits=4, use_pool=True, use_keep=True, use_tail=True)),
                              ("second call: one short sequence, int4 records + tail", small, dict(bits=4, use_tail=True))):
            print(f"[static] {tag}", flush=True)
            kw = H.draft_kwargs(lay, **sel)
            out, lse = _static_draft(lib, ctx, lay, kw)
            ref_out, ref_lse = H.gpu_draft(lib, ctx, lay, **kw)           # the entry point with a caller workspace
            assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16))
            assert torch.equal(lse, ref_lse)
            o_ref, o_lse = H.oracle_draft(lay, kw)
            assert H.rel_err(out, o_ref) <= H.TOL
            fin = np.isfinite(o_lse)
            assert np.abs(lse.cpu().numpy()[fin] - o_lse[fin]).max() <= H.LSE_TOL
    finally:
        ctx.close()


def test_static_draft_rejects_a_batch_beyond_the_scratch(lib):
    ctx = lib.Context(0)
    try:
        # descriptor only: 4096 sequences x 64 query heads need more partial slots than 8 MiB hold; the
        # call must fail on the host before anything is enqueued (the pointers are never dereferenced)
        nseq, hq, hkv = 4096, 64, 8
        q = torch.zeros((nseq, hq, 128), dtype=torch.bfloat16, device=DEV)
        out = torch.empty_like(q)
        blocks = torch.zeros((16, 5120), dtype=torch.uint8, device=DEV)
        cu = torch.zeros(nseq + 1, dtype=torch.int32, device=DEV)
        kw = dict(blocks=blocks, cu_blk=cu, max_blk=64, bits=4)
        assert lib.vc_draft_workspace_bytes(hq, hkv, nseq, **kw) > lib.vc_draft_static_scratch_bytes()
        with pytest.raises(lib.VcError) as e:
            lib.vc_draft_attn_static(ctx, q, 0.1, out, n_kv_heads=hkv, **kw)
        assert e.value.status == 3 and "static scratch" in str(e.value)
        torch.cuda.synchronize()
    finally:
        ctx.close()
