"""GPU parity of vc_swap_in_rows (reload of the dropped rows only): byte-exact against the oracle,
rows that are not named stay untouched, and a verify over the completed pool matches the oracle's
verify over the full KV."""
import numpy as np
import pytest
import torch

from oracle import vc_oracle as O
from tests import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context(0)
    yield c
    c.close()


def resident_pool(lay):
    """Device pools that hold only the kept rows (everything else NaN), as after token dropping."""
    dk = torch.full_like(lay.k_full, float("nan")); dv = torch.full_like(lay.v_full, float("nan"))
    cu_keep = lay.cu_keep.cpu().numpy()
    hkv = lay.n_kv_heads
    keep = lay.keep_idx.cpu().numpy()
    for b, n in enumerate(lay.ctx_len):
        nk = int(cu_keep[b + 1] - cu_keep[b])
        lo = int(lay.cu_ctx[b])
        for h in range(hkv):
            idx = torch.tensor(keep[cu_keep[b] * hkv + h * nk: cu_keep[b] * hkv + (h + 1) * nk], device=DEV, dtype=torch.long) + lo
            dk[idx, h] = lay.k_full[idx, h]
            dv[idx, h] = lay.v_full[idx, h]
    return dk, dv


def pinned(t):
    h = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
    h.copy_(t)
    return h


def packed_host(lib, ctx, lay, nd):
    """The host's share of a token-dropped layer: its dropped rows, packed by the library."""
    rows = int(lay.cu_drop[-1]) * lay.n_kv_heads
    pk = torch.empty((max(rows, 1), 128), dtype=torch.bfloat16, device=DEV)
    pv = torch.empty_like(pk)
    lib.vc_pack_rows(ctx, lay.k_full, lay.v_full, lay.dropped_idx, lay.cu_drop, lay.cu_ctx, lay.n_kv_heads, max(nd), pk, pv)
    torch.cuda.synchronize()
    rk, rv = O.pack_rows(H.bits16(lay.k_full), H.bits16(lay.v_full), H.npi(lay.dropped_idx), H.npi(lay.cu_drop),
                         H.npi(lay.cu_ctx), lay.n_kv_heads)
    assert np.array_equal(H.bits16(pk)[:rows], rk) and np.array_equal(H.bits16(pv)[:rows], rv)
    return pinned(pk), pinned(pv)


def test_reload_rows_then_verify(lib, ctx):
    lens = [700, 64, 1500, 333]
    keep = [70, 64, 151, 34]                                  # sequence 1 drops nothing
    lay = synth.make_layer(31, DEV, ctx_len=lens, n_q_heads=8, n_kv_heads=2, keep=keep, keep_first=4, keep_last=8,
                           win=[8, 3, 16, 5])
    nd = [n - k for n, k in zip(lens, keep)]
    hk, hv = packed_host(lib, ctx, lay, nd)
    dk, dv = resident_pool(lay)
    stage_k = torch.empty((max(nd) * 2, 128), dtype=torch.bfloat16, device=DEV); stage_v = torch.empty_like(stage_k)
    cu_drop_host = lay.cu_drop.cpu()
    args = (lay.dropped_idx, lay.cu_drop, cu_drop_host, lay.cu_ctx, 2)
    torch.cuda.synchronize()
    # sequences 0 and 1 first: the other two must stay as they are
    print("[rows] sequences 0..1", flush=True)
    t0 = lib.vc_swap_in_rows(ctx, hk, hv, stage_k, stage_v, dk, dv, *args, 0, 2)
    lib.vc_swap_wait(ctx, t0 + 1)
    torch.cuda.synchronize()
    dk0, dv0 = resident_pool(lay)
    rk, rv = O.swap_in_rows(H.bits16(hk), H.bits16(hv), H.bits16(dk0), H.bits16(dv0),
                            H.npi(lay.dropped_idx), H.npi(lay.cu_drop), H.npi(lay.cu_ctx), 2, [0, 1])
    assert np.array_equal(H.bits16(dk), rk) and np.array_equal(H.bits16(dv), rv)
    print("[rows] sequences 2..3", flush=True)
    t1 = lib.vc_swap_in_rows(ctx, hk, hv, stage_k, stage_v, dk, dv, *args, 2, 4)
    assert t1 == t0 + 2
    lib.vc_swap_wait(ctx, t1 + 1)
    assert lib.vc_swap_query(ctx, t1) in (True, False)
    lib.vc_swap_sync(ctx)
    assert lib.vc_swap_query(ctx, t1 + 1)
    assert torch.equal(dk.view(torch.int16), lay.k_full.view(torch.int16))
    assert torch.equal(dv.view(torch.int16), lay.v_full.view(torch.int16))
    out, lse = H.gpu_verify(lib, ctx, lay, k_full=dk, v_full=dv)
    ref, ref_lse = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= H.LSE_TOL


def test_reload_rows_rejects_bad_buffers_and_empty_range(lib, ctx):
    lay = synth.make_layer(32, DEV, ctx_len=[128], n_q_heads=4, n_kv_heads=1, keep=[16], keep_first=2, keep_last=2)
    hk, hv = packed_host(lib, ctx, lay, [112])
    dk, dv = resident_pool(lay)
    stage = torch.empty((112, 128), dtype=torch.bfloat16, device=DEV)
    cu_h = lay.cu_drop.cpu()
    tail = (lay.dropped_idx, lay.cu_drop, cu_h, lay.cu_ctx, 1)
    pageable = hk.clone()
    with pytest.raises(lib.VcError):                      # pageable source
        lib.vc_swap_in_rows(ctx, pageable, pageable, stage, stage.clone(), dk, dv, *tail, 0, 1)
    with pytest.raises(lib.VcError):                      # destination must be device memory
        lib.vc_swap_in_rows(ctx, hk, hv, stage, stage.clone(), hk, hv, *tail, 0, 1)
    with pytest.raises(lib.VcError):                      # staging too small for the sequence
        lib.vc_swap_in_rows(ctx, hk, hv, stage[:64], stage[:64].clone(), dk, dv, *tail, 0, 1)
    before = dk.clone()
    t = lib.vc_swap_in_rows(ctx, hk, hv, stage, stage.clone(), dk, dv, *tail, 1, 1)   # empty range
    lib.vc_swap_sync(ctx)
    assert torch.equal(before.view(torch.int16), dk.view(torch.int16)) and t >= 0
