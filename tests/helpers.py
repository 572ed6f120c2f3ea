"""Glue for the GPU parity tests: run a synth.Layer through the library's binding, and through the
oracle on CPU copies of the very same tensors."""
from __future__ import annotations

import numpy as np
import torch

from oracle import vc_oracle as O

TOL = 1e-2          # max|gpu - oracle| / max|oracle| for bf16 attention outputs (spec bound)
LSE_TOL = 5e-3      # absolute, natural-log units


def bits16(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> numpy uint16 bit patterns (on the CPU)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def npi(t):
    return None if t is None else t.detach().cpu().numpy()


def rel_err(gpu: torch.Tensor, ref: np.ndarray) -> float:
    g = gpu.detach().double().cpu().numpy()
    denom = np.abs(ref).max()
    return float(np.abs(g - ref).max() / (denom if denom > 0 else 1.0))


def draft_kwargs(lay, bits=None, use_pool=False, use_keep=False, use_tail=False):
    """The vc_comp_kv fields (as binding keyword arguments) for one way of reading a Layer."""
    kw = {}
    if use_pool:
        kw.update(pool_k=lay.k_full, pool_v=lay.v_full, cu_ctx=lay.cu_ctx)
        if use_keep:
            kw.update(keep_idx=lay.keep_idx, cu_keep=lay.cu_keep, max_keep=lay.max_keep)
        else:
            kw.update(max_keep=max(lay.ctx_len))
    if bits:
        kw.update(blocks=lay.blocks[bits], cu_blk=lay.cu_blk[bits], max_blk=lay.max_blk[bits], bits=bits)
    if use_tail and lay.tail_k is not None:
        kw.update(tail_k=lay.tail_k, tail_v=lay.tail_v, cu_tail=lay.cu_tail, max_tail=lay.max_tail)
    return kw


def gpu_draft(vc, ctx, lay, **kw):
    nseq = lay.q.shape[0]
    out = torch.empty_like(lay.q)
    lse = torch.empty((nseq, lay.n_q_heads), dtype=torch.float32, device=lay.q.device)
    nbytes = vc.vc_draft_workspace_bytes(lay.n_q_heads, lay.n_kv_heads, nseq, **kw)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=lay.q.device)
    vc.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=lay.n_kv_heads, lse=lse, workspace=ws, **kw)
    torch.cuda.synchronize()
    return out, lse


def oracle_kv_args(kw):
    """Binding keyword arguments -> oracle keyword arguments (CPU numpy copies)."""
    o = {}
    if "pool_k" in kw:
        o.update(pool_k=bits16(kw["pool_k"]), pool_v=bits16(kw["pool_v"]), cu_ctx=npi(kw["cu_ctx"]))
        if "keep_idx" in kw:
            o.update(keep_idx=npi(kw["keep_idx"]), cu_keep=npi(kw["cu_keep"]))
    if "blocks" in kw:
        o.update(blocks=npi(kw["blocks"]), cu_blk=npi(kw["cu_blk"]), bits=kw["bits"])
    if "tail_k" in kw:
        o.update(tail_k=bits16(kw["tail_k"]), tail_v=bits16(kw["tail_v"]), cu_tail=npi(kw["cu_tail"]))
    return o


def oracle_draft(lay, kw):
    return O.draft_attn(bits16(lay.q), lay.scale, n_q_heads=lay.n_q_heads, n_kv_heads=lay.n_kv_heads,
                        **oracle_kv_args(kw))


def gpu_verify(vc, ctx, lay, k_full=None, v_full=None, sum_ctx=0):
    k_full = lay.k_full if k_full is None else k_full
    v_full = lay.v_full if v_full is None else v_full
    nseq = len(lay.ctx_len)
    tw = lay.q_win.shape[0]
    out = torch.empty_like(lay.q_win)
    lse = torch.empty((tw, lay.n_q_heads), dtype=torch.float32, device=lay.q_win.device)
    args = dict(k=k_full, v=v_full, cu_ctx=lay.cu_ctx, max_ctx=max(lay.ctx_len), max_win=max(lay.win), sum_ctx=sum_ctx)
    nbytes = vc.vc_verify_workspace_bytes(lay.n_q_heads, lay.n_kv_heads, nseq, total_win=tw, **args)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=lay.q_win.device)
    vc.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, out, n_seqs=nseq, lse=lse,
                      workspace=ws, **args)
    torch.cuda.synchronize()
    return out, lse


def oracle_verify(lay):
    return O.verify_attn(bits16(lay.q_win), bits16(lay.k_full), bits16(lay.v_full), bits16(lay.k_win),
                         bits16(lay.v_win), npi(lay.cu_ctx), npi(lay.cu_win), lay.scale,
                         n_q_heads=lay.n_q_heads, n_kv_heads=lay.n_kv_heads)


def gpu_accept(vc, ctx, lay):
    dev = lay.logits.device
    nseq = lay.cu_rows.numel() - 1
    rows, vocab = lay.logits.shape
    acc = torch.full((nseq,), -7, dtype=torch.int32, device=dev)
    nxt = torch.full((nseq,), -7, dtype=torch.int32, device=dev)
    amax = torch.full((max(rows, 1),), -7, dtype=torch.int32, device=dev)
    ws = torch.empty(max(vc.vc_accept_workspace_bytes(rows, vocab), 16), dtype=torch.uint8, device=dev)
    vc.vc_accept_len(ctx, lay.logits, lay.cu_rows, lay.draft_ids, lay.cu_win, acc, nxt, amax, workspace=ws)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), nxt.cpu().numpy(), amax[:rows].cpu().numpy()


def oracle_accept(lay):
    return O.accept(npi(lay.logits), npi(lay.cu_rows), npi(lay.draft_ids), npi(lay.cu_win))
