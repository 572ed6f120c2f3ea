"""ctypes binding over libvericache.so: argument marshalling only.

Every function takes torch tensors (device memory and streams are torch's), checks dtype / device
/ contiguity, and passes raw pointers and sizes through the C ABI declared in
include/vericache.h.  There is no fallback: if the library is not built the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

VC_OK, VC_ERR_INVALID_ARG, VC_ERR_UNSUPPORTED, VC_ERR_WORKSPACE, VC_ERR_HIP, VC_ERR_NOT_READY = range(6)


class VcError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"vericache status {status}: {msg}")
        self.status = status


class vc_comp_kv(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("bits", C.c_int32), ("max_keep", C.c_int32),
                ("max_blk", C.c_int32), ("max_tail", C.c_int32), ("sum_keep", C.c_int32), ("sum_blk", C.c_int32),
                ("pool_k", C.c_void_p), ("pool_v", C.c_void_p), ("cu_ctx", C.c_void_p),
                ("keep_idx", C.c_void_p), ("cu_keep", C.c_void_p), ("blocks", C.c_void_p),
                ("cu_blk", C.c_void_p), ("tail_k", C.c_void_p), ("tail_v", C.c_void_p),
                ("cu_tail", C.c_void_p)]


class vc_full_kv(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("max_ctx", C.c_int32), ("max_win", C.c_int32), ("sum_ctx", C.c_int32),
                ("chunk_tokens", C.c_int32),
                ("k", C.c_void_p), ("v", C.c_void_p), ("cu_ctx", C.c_void_p),
                ("ring_slots", C.c_int32), ("ring_slot", C.c_void_p)]


class vc_chunk(C.Structure):
    _fields_ = [("src_off", C.c_size_t), ("dst_off", C.c_size_t), ("bytes", C.c_size_t)]


EXPORTS = ["vc_create", "vc_destroy", "vc_last_error", "vc_version", "vc_time_main_kernel",
           "vc_set_tunable", "vc_get_tunable", "vc_stream_status", "vc_validate_comp_kv", "vc_validate_full_kv",
           "vc_draft_workspace_bytes", "vc_draft_attn", "vc_draft_static_scratch_bytes", "vc_draft_attn_static", "vc_verify_workspace_bytes", "vc_verify_attn",
           "vc_verify_plan", "vc_verify_attn_range", "vc_verify_finish",
           "vc_accept_workspace_bytes", "vc_accept_len", "vc_accept_sample_workspace_bytes", "vc_accept_sample", "vc_swap_in", "vc_swap_in_rows", "vc_pack_rows", "vc_swap_wait", "vc_mark", "vc_swap_after", "vc_swap_query", "vc_swap_sync",
           "vc_keep_from_dropped", "vc_compress_quant", "vc_decompress_quant", "vc_topk_keep",
           "vc_iter_time_model", "vc_sched_create", "vc_sched_destroy", "vc_sched_set_resident", "vc_sched_span",
           "vc_sched_admit", "vc_sched_cancel", "vc_sched_step", "vc_sched_rings"]


def library_path() -> str:
    return os.path.join(_HERE, "libvericache.so")


def load():
    """Load the built library (once).  Raises if it is missing: there is no other code path."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(path)
    lib.vc_last_error.restype = C.c_char_p
    lib.vc_version.restype = C.c_char_p
    lib.vc_create.argtypes = [C.c_int, C.POINTER(C.c_void_p)]
    lib.vc_destroy.argtypes = [C.c_void_p]
    lib.vc_time_main_kernel.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.vc_set_tunable.argtypes = [C.c_char_p, C.c_int32]
    lib.vc_get_tunable.argtypes = [C.c_char_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.vc_stream_status.argtypes = [C.c_void_p, C.c_void_p]
    lib.vc_validate_comp_kv.argtypes = [C.c_void_p, C.POINTER(vc_comp_kv), C.c_void_p, C.c_void_p]
    lib.vc_validate_full_kv.argtypes = [C.c_void_p, C.POINTER(vc_full_kv), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.vc_draft_workspace_bytes.argtypes = [C.POINTER(vc_comp_kv), C.POINTER(C.c_size_t)]
    lib.vc_draft_attn.argtypes = [C.c_void_p, C.POINTER(vc_comp_kv), C.c_void_p, C.c_float, C.c_void_p,
                                  C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.vc_draft_static_scratch_bytes.argtypes = [C.POINTER(C.c_size_t)]
    lib.vc_draft_attn_static.argtypes = [C.c_void_p, C.POINTER(vc_comp_kv), C.c_void_p, C.c_float, C.c_void_p,
                                         C.c_void_p, C.c_void_p]
    lib.vc_verify_workspace_bytes.argtypes = [C.POINTER(vc_full_kv), C.c_int32, C.POINTER(C.c_size_t)]
    lib.vc_verify_attn.argtypes = [C.c_void_p, C.POINTER(vc_full_kv), C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_size_t, C.c_void_p]
    lib.vc_verify_plan.argtypes = [C.POINTER(vc_full_kv), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.vc_verify_attn_range.argtypes = [C.c_void_p, C.POINTER(vc_full_kv), C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_int32, C.c_float, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                         C.c_void_p, C.c_size_t, C.c_void_p]
    lib.vc_verify_finish.argtypes = [C.c_void_p, C.POINTER(vc_full_kv), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_size_t, C.c_void_p]
    lib.vc_accept_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
    lib.vc_accept_len.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                  C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_size_t, C.c_void_p]
    lib.vc_accept_sample_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
    lib.vc_accept_sample.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                     C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.vc_swap_in.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(vc_chunk), C.c_int32,
                               C.POINTER(C.c_int64)]
    lib.vc_swap_in_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                    C.c_int32, C.POINTER(C.c_int64)]
    lib.vc_pack_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                 C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.vc_swap_wait.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
    lib.vc_mark.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int64)]
    lib.vc_swap_after.argtypes = [C.c_void_p, C.c_int64]
    lib.vc_swap_query.argtypes = [C.c_void_p, C.c_int64]
    lib.vc_swap_sync.argtypes = [C.c_void_p]
    lib.vc_keep_from_dropped.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                         C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.vc_compress_quant.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.vc_decompress_quant.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                        C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.vc_topk_keep.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                 C.c_int32, C.c_void_p, C.c_void_p]
    lib.vc_iter_time_model.argtypes = [C.c_double] * 7 + [C.POINTER(C.c_double)] * 3
    lib.vc_sched_create.argtypes = [C.c_int32] + [C.c_double] * 5 + [C.POINTER(C.c_void_p)]
    lib.vc_sched_destroy.argtypes = [C.c_void_p]
    lib.vc_sched_set_resident.argtypes = [C.c_void_p, C.c_double]
    lib.vc_sched_span.argtypes = [C.c_void_p, C.c_double, C.POINTER(C.c_int32)]
    lib.vc_sched_admit.argtypes = [C.c_void_p, C.c_int64, C.c_double, C.c_int32, C.POINTER(C.c_int32)]
    lib.vc_sched_cancel.argtypes = [C.c_void_p, C.c_int64]
    lib.vc_sched_step.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int32), C.POINTER(C.c_int64),
                                  C.POINTER(C.c_int32), C.c_int32]
    lib.vc_sched_rings.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    _LIB = lib
    return lib


def _check(status: int):
    if status != VC_OK:
        raise VcError(status, load().vc_last_error().decode())


def _ptr(t, dtype=None, name="tensor"):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name}: expected a torch tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def vc_version() -> str:
    return load().vc_version().decode()


class Context:
    """vc_ctx: owns the copy stream and chunk events of one device."""

    def __init__(self, device: int = 0):
        self._h = C.c_void_p()
        _check(load().vc_create(int(device), C.byref(self._h)))
        self.device = int(device)

    def close(self):
        if self._h:
            load().vc_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h


def _comp_desc(n_q_heads, n_kv_heads, n_seqs, *, pool_k=None, pool_v=None, cu_ctx=None, keep_idx=None,
               cu_keep=None, max_keep=0, blocks=None, cu_blk=None, max_blk=0, bits=4,
               tail_k=None, tail_v=None, cu_tail=None, max_tail=0, sum_keep=0, sum_blk=0,
               head_dim=128):
    d = vc_comp_kv()
    d.n_seqs, d.n_q_heads, d.n_kv_heads, d.head_dim = n_seqs, n_q_heads, n_kv_heads, head_dim
    d.bits, d.max_keep, d.max_blk, d.max_tail = bits, max_keep, max_blk, max_tail
    d.sum_keep, d.sum_blk = sum_keep, sum_blk
    d.pool_k = _ptr(pool_k, torch.bfloat16, "pool_k"); d.pool_v = _ptr(pool_v, torch.bfloat16, "pool_v")
    d.cu_ctx = _ptr(cu_ctx, torch.int32, "cu_ctx")
    d.keep_idx = _ptr(keep_idx, torch.int32, "keep_idx"); d.cu_keep = _ptr(cu_keep, torch.int32, "cu_keep")
    d.blocks = _ptr(blocks, torch.uint8, "blocks"); d.cu_blk = _ptr(cu_blk, torch.int32, "cu_blk")
    d.tail_k = _ptr(tail_k, torch.bfloat16, "tail_k"); d.tail_v = _ptr(tail_v, torch.bfloat16, "tail_v")
    d.cu_tail = _ptr(cu_tail, torch.int32, "cu_tail")
    return d


def vc_set_tunable(name: str, value: int):
    """Override a launch-shape tunable for the process; value < 0 restores the library default."""
    _check(load().vc_set_tunable(name.encode(), int(value)))


def vc_get_tunable(name: str):
    """Returns the set value, or None when the tunable is at its library default."""
    v, isset = C.c_int32(), C.c_int32()
    _check(load().vc_get_tunable(name.encode(), C.byref(v), C.byref(isset)))
    return v.value if isset.value else None


def vc_stream_status(ctx: Context, stream=None) -> bool:
    """True when everything enqueued on the stream has finished, False while work is in flight."""
    st = load().vc_stream_status(ctx.handle, _stream(stream))
    if st == VC_ERR_NOT_READY:
        return False
    _check(st)
    return True


def vc_validate_comp_kv(ctx: Context, report, *, n_q_heads, n_kv_heads, n_seqs, stream=None, **kv):
    """report: device int64[2], written asynchronously (violations, smallest violation key or -1)."""
    d = _comp_desc(n_q_heads, n_kv_heads, n_seqs, **kv)
    _check(load().vc_validate_comp_kv(ctx.handle, C.byref(d), _ptr(report, torch.int64, "report"), _stream(stream)))


def vc_validate_full_kv(ctx: Context, report, cu_win, total_win, *, n_q_heads, n_kv_heads, n_seqs, k, v, cu_ctx,
                        max_ctx, max_win, stream=None, sum_ctx=0, chunk_tokens=0):
    d = _full_desc(n_q_heads, n_kv_heads, n_seqs, k, v, cu_ctx, max_ctx, max_win, sum_ctx=sum_ctx,
                   chunk_tokens=chunk_tokens)
    _check(load().vc_validate_full_kv(ctx.handle, C.byref(d), _ptr(cu_win, torch.int32, "cu_win"), int(total_win),
                                      _ptr(report, torch.int64, "report"), _stream(stream)))


def vc_draft_workspace_bytes(n_q_heads, n_kv_heads, n_seqs, **kv) -> int:
    d = _comp_desc(n_q_heads, n_kv_heads, n_seqs, **kv)
    n = C.c_size_t()
    _check(load().vc_draft_workspace_bytes(C.byref(d), C.byref(n)))
    return n.value


def vc_draft_attn(ctx: Context, q, softmax_scale, out, *, n_kv_heads, lse=None, workspace=None, stream=None, **kv):
    """q, out: bf16 [n_seqs, n_q_heads, 128] device tensors; kv: the vc_comp_kv fields by name."""
    n_seqs, n_q_heads = q.shape[0], q.shape[1]
    d = _comp_desc(n_q_heads, n_kv_heads, n_seqs, head_dim=q.shape[2], **kv)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().vc_draft_attn(ctx.handle, C.byref(d), _ptr(q, torch.bfloat16, "q"), float(softmax_scale),
                                _ptr(out, torch.bfloat16, "out"), _ptr(lse, torch.float32, "lse"),
                                _ptr(workspace, None, "workspace"), ws_bytes, _stream(stream)))
    return out


def vc_draft_static_scratch_bytes() -> int:
    n = C.c_size_t()
    _check(load().vc_draft_static_scratch_bytes(C.byref(n)))
    return n.value


def vc_draft_attn_static(ctx: Context, q, softmax_scale, out, *, n_kv_heads, lse=None, stream=None, **kv):
    """vc_draft_attn without a workspace: the split partials live in the library's static scratch."""
    n_seqs, n_q_heads = q.shape[0], q.shape[1]
    d = _comp_desc(n_q_heads, n_kv_heads, n_seqs, head_dim=q.shape[2], **kv)
    _check(load().vc_draft_attn_static(ctx.handle, C.byref(d), _ptr(q, torch.bfloat16, "q"), float(softmax_scale),
                                       _ptr(out, torch.bfloat16, "out"), _ptr(lse, torch.float32, "lse"),
                                       _stream(stream)))
    return out


def _full_desc(n_q_heads, n_kv_heads, n_seqs, k, v, cu_ctx, max_ctx, max_win, head_dim=128, sum_ctx=0,
               chunk_tokens=0, ring_slots=0, ring_slot=None):
    d = vc_full_kv()
    d.ring_slots = ring_slots
    d.ring_slot = _ptr(ring_slot, torch.int32, "ring_slot")
    d.n_seqs, d.n_q_heads, d.n_kv_heads, d.head_dim = n_seqs, n_q_heads, n_kv_heads, head_dim
    d.max_ctx, d.max_win, d.sum_ctx, d.chunk_tokens = max_ctx, max_win, sum_ctx, chunk_tokens
    d.k = _ptr(k, torch.bfloat16, "k"); d.v = _ptr(v, torch.bfloat16, "v")
    d.cu_ctx = _ptr(cu_ctx, torch.int32, "cu_ctx")
    return d


def vc_verify_workspace_bytes(n_q_heads, n_kv_heads, n_seqs, *, k, v, cu_ctx, max_ctx, max_win, total_win,
                              sum_ctx=0, chunk_tokens=0, ring_slots=0, ring_slot=None) -> int:
    d = _full_desc(n_q_heads, n_kv_heads, n_seqs, k, v, cu_ctx, max_ctx, max_win, sum_ctx=sum_ctx,
                   chunk_tokens=chunk_tokens, ring_slots=ring_slots, ring_slot=ring_slot)
    n = C.c_size_t()
    _check(load().vc_verify_workspace_bytes(C.byref(d), int(total_win), C.byref(n)))
    return n.value


def vc_verify_attn(ctx: Context, q_win, k_win, v_win, cu_win, softmax_scale, out, *, k, v, cu_ctx, max_ctx,
                   max_win, n_seqs, lse=None, workspace=None, stream=None, sum_ctx=0, chunk_tokens=0, ring_slots=0,
                   ring_slot=None):
    total_win, n_q_heads = q_win.shape[0], q_win.shape[1]
    n_kv_heads = k_win.shape[1]
    d = _full_desc(n_q_heads, n_kv_heads, n_seqs, k, v, cu_ctx, max_ctx, max_win, head_dim=q_win.shape[2],
                   sum_ctx=sum_ctx, chunk_tokens=chunk_tokens, ring_slots=ring_slots, ring_slot=ring_slot)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().vc_verify_attn(ctx.handle, C.byref(d), _ptr(q_win, torch.bfloat16, "q_win"),
                                 _ptr(k_win, torch.bfloat16, "k_win"), _ptr(v_win, torch.bfloat16, "v_win"),
                                 _ptr(cu_win, torch.int32, "cu_win"), int(total_win), float(softmax_scale),
                                 _ptr(out, torch.bfloat16, "out"), _ptr(lse, torch.float32, "lse"),
                                 _ptr(workspace, None, "workspace"), ws_bytes, _stream(stream)))
    return out


def vc_verify_plan(n_q_heads, n_kv_heads, n_seqs, *, k, v, cu_ctx, max_ctx, max_win, sum_ctx=0, chunk_tokens=0,
                   ring_slots=0, ring_slot=None):
    """Returns (chunk_tokens, n_chunks) of the verify launch plan."""
    d = _full_desc(n_q_heads, n_kv_heads, n_seqs, k, v, cu_ctx, max_ctx, max_win, sum_ctx=sum_ctx,
                   chunk_tokens=chunk_tokens, ring_slots=ring_slots, ring_slot=ring_slot)
    ct, nc = C.c_int32(), C.c_int32()
    _check(load().vc_verify_plan(C.byref(d), C.byref(ct), C.byref(nc)))
    return ct.value, nc.value


def vc_verify_attn_range(ctx: Context, q_win, k_win, v_win, cu_win, softmax_scale, seq_begin, seq_end, tok_begin,
                         tok_end, *, k, v, cu_ctx, max_ctx, max_win, n_seqs, workspace, stream=None, sum_ctx=0,
                         chunk_tokens=0, ring_slots=0, ring_slot=None):
    total_win, n_q_heads = q_win.shape[0], q_win.shape[1]
    d = _full_desc(n_q_heads, k_win.shape[1], n_seqs, k, v, cu_ctx, max_ctx, max_win, head_dim=q_win.shape[2],
                   sum_ctx=sum_ctx, chunk_tokens=chunk_tokens, ring_slots=ring_slots, ring_slot=ring_slot)
    _check(load().vc_verify_attn_range(ctx.handle, C.byref(d), _ptr(q_win, torch.bfloat16, "q_win"),
                                       _ptr(k_win, torch.bfloat16, "k_win"), _ptr(v_win, torch.bfloat16, "v_win"),
                                       _ptr(cu_win, torch.int32, "cu_win"), int(total_win), float(softmax_scale),
                                       int(seq_begin), int(seq_end), int(tok_begin), int(tok_end),
                                       _ptr(workspace, None, "workspace"), workspace.numel() * workspace.element_size(),
                                       _stream(stream)))


def vc_verify_finish(ctx: Context, cu_win, out, *, n_q_heads, n_kv_heads, k, v, cu_ctx, max_ctx, max_win, n_seqs,
                     workspace, lse=None, stream=None, sum_ctx=0, chunk_tokens=0, ring_slots=0, ring_slot=None):
    d = _full_desc(n_q_heads, n_kv_heads, n_seqs, k, v, cu_ctx, max_ctx, max_win, sum_ctx=sum_ctx,
                   chunk_tokens=chunk_tokens, ring_slots=ring_slots, ring_slot=ring_slot)
    _check(load().vc_verify_finish(ctx.handle, C.byref(d), _ptr(cu_win, torch.int32, "cu_win"), int(out.shape[0]),
                                   _ptr(out, torch.bfloat16, "out"), _ptr(lse, torch.float32, "lse"),
                                   _ptr(workspace, None, "workspace"), workspace.numel() * workspace.element_size(),
                                   _stream(stream)))
    return out


def vc_accept_workspace_bytes(total_rows: int, vocab: int) -> int:
    n = C.c_size_t()
    _check(load().vc_accept_workspace_bytes(int(total_rows), int(vocab), C.byref(n)))
    return n.value


def vc_accept_len(ctx: Context, logits, cu_rows, draft_ids, cu_win, accept_len, next_token, argmax_ids,
                  workspace=None, stream=None):
    total_rows, vocab = logits.shape
    n_seqs = cu_rows.numel() - 1
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().vc_accept_len(ctx.handle, _ptr(logits, torch.float32, "logits"), int(vocab),
                                _ptr(cu_rows, torch.int32, "cu_rows"), int(total_rows),
                                _ptr(draft_ids, torch.int32, "draft_ids"), _ptr(cu_win, torch.int32, "cu_win"),
                                int(n_seqs), _ptr(accept_len, torch.int32, "accept_len"),
                                _ptr(next_token, torch.int32, "next_token"),
                                _ptr(argmax_ids, torch.int32, "argmax_ids"),
                                _ptr(workspace, None, "workspace"), ws_bytes, _stream(stream)))
    return accept_len, next_token


def vc_accept_sample_workspace_bytes(total_rows: int, total_win: int, n_seqs: int, vocab: int) -> int:
    n = C.c_size_t()
    _check(load().vc_accept_sample_workspace_bytes(int(total_rows), int(total_win), int(n_seqs), int(vocab), C.byref(n)))
    return n.value


def vc_accept_sample(ctx: Context, target_logits, draft_logits, cu_rows, draft_ids, cu_win, temperature, u_accept,
                     u_resample, accept_len, next_token, workspace=None, stream=None):
    total_rows, vocab = target_logits.shape
    total_win = draft_logits.shape[0]
    n_seqs = cu_rows.numel() - 1
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().vc_accept_sample(ctx.handle, _ptr(target_logits, torch.float32, "target_logits"),
                                   _ptr(draft_logits, torch.float32, "draft_logits"), int(vocab),
                                   _ptr(cu_rows, torch.int32, "cu_rows"), int(total_rows),
                                   _ptr(draft_ids, torch.int32, "draft_ids"), _ptr(cu_win, torch.int32, "cu_win"),
                                   int(total_win), int(n_seqs), float(temperature),
                                   _ptr(u_accept, torch.float32, "u_accept"), _ptr(u_resample, torch.float32, "u_resample"),
                                   _ptr(accept_len, torch.int32, "accept_len"), _ptr(next_token, torch.int32, "next_token"),
                                   _ptr(workspace, None, "workspace"), ws_bytes, _stream(stream)))
    return accept_len, next_token


def vc_swap_in(ctx: Context, host_src, dev_dst, chunks) -> int:
    """chunks: list of (src_off, dst_off, bytes).  Returns the first ticket."""
    arr = (vc_chunk * max(1, len(chunks)))()
    for i, (s, d, n) in enumerate(chunks):
        arr[i].src_off, arr[i].dst_off, arr[i].bytes = int(s), int(d), int(n)
    first = C.c_int64()
    _check(load().vc_swap_in(ctx.handle, C.c_void_p(host_src.data_ptr()), C.c_void_p(dev_dst.data_ptr()),
                             arr, len(chunks), C.byref(first)))
    return first.value


def vc_swap_in_rows(ctx: Context, host_packed_k, host_packed_v, stage_k, stage_v, dev_k, dev_v, dropped, cu_drop,
                    cu_drop_host, cu_ctx, n_kv_heads, seq_begin, seq_end) -> int:
    """Reload only the dropped rows of sequences [seq_begin, seq_end) from packed pinned buffers.
    cu_drop_host: CPU int32 tensor (a copy of cu_drop).  Returns the first ticket."""
    if cu_drop_host.device.type != "cpu" or cu_drop_host.dtype != torch.int32:
        raise TypeError("cu_drop_host: expected a CPU int32 tensor")
    first = C.c_int64()
    stage_rows = min(stage_k.numel(), stage_v.numel()) // 128
    _check(load().vc_swap_in_rows(ctx.handle, C.c_void_p(host_packed_k.data_ptr()), C.c_void_p(host_packed_v.data_ptr()),
                                  _ptr(stage_k, torch.bfloat16, "stage_k"), _ptr(stage_v, torch.bfloat16, "stage_v"),
                                  stage_rows, _ptr(dev_k, torch.bfloat16, "dev_k"), _ptr(dev_v, torch.bfloat16, "dev_v"),
                                  _ptr(dropped, torch.int32, "dropped"), _ptr(cu_drop, torch.int32, "cu_drop"),
                                  C.c_void_p(cu_drop_host.data_ptr()), _ptr(cu_ctx, torch.int32, "cu_ctx"), n_kv_heads,
                                  seq_begin, seq_end, C.byref(first)))
    return first.value


def vc_pack_rows(ctx: Context, k, v, idx, cu_idx, cu_ctx, n_kv_heads, max_idx, packed_k, packed_v, stream=None):
    n_seqs = cu_ctx.numel() - 1
    _check(load().vc_pack_rows(ctx.handle, _ptr(k, torch.bfloat16, "k"), _ptr(v, torch.bfloat16, "v"),
                               _ptr(idx, torch.int32, "idx"), _ptr(cu_idx, torch.int32, "cu_idx"),
                               _ptr(cu_ctx, torch.int32, "cu_ctx"), n_seqs, n_kv_heads, max_idx,
                               _ptr(packed_k, torch.bfloat16, "packed_k"), _ptr(packed_v, torch.bfloat16, "packed_v"),
                               _stream(stream)))


def vc_swap_wait(ctx: Context, ticket: int, stream=None):
    _check(load().vc_swap_wait(ctx.handle, int(ticket), _stream(stream)))


def vc_mark(ctx: Context, stream=None) -> int:
    """Marks the work enqueued on `stream` so far; returns the mark's number."""
    m = C.c_int64()
    _check(load().vc_mark(ctx.handle, _stream(stream), C.byref(m)))
    return m.value


def vc_swap_after(ctx: Context, mark: int):
    """Later reloads start only after the marked work has finished (device-side ordering)."""
    _check(load().vc_swap_after(ctx.handle, int(mark)))


def vc_swap_query(ctx: Context, ticket: int) -> bool:
    st = load().vc_swap_query(ctx.handle, int(ticket))
    if st == VC_ERR_NOT_READY:
        return False
    _check(st)
    return True


def vc_time_main_kernel(ctx: Context, begin_event=None, end_event=None):
    """Arm two torch.cuda.Event(enable_timing=True) objects (already recorded once, so that their
    handles exist) around the main kernel(s) of the next attention call; None, None disarms."""
    b = None if begin_event is None else C.c_void_p(begin_event.cuda_event)
    e = None if end_event is None else C.c_void_p(end_event.cuda_event)
    _check(load().vc_time_main_kernel(ctx.handle, b, e))


def vc_swap_sync(ctx: Context):
    _check(load().vc_swap_sync(ctx.handle))


def vc_keep_from_dropped(ctx: Context, dropped, cu_drop, cu_ctx, n_kv_heads, max_ctx, keep_idx, cu_keep, stream=None):
    n_seqs = cu_ctx.numel() - 1
    _check(load().vc_keep_from_dropped(ctx.handle, _ptr(dropped, torch.int32, "dropped"),
                                       _ptr(cu_drop, torch.int32, "cu_drop"), _ptr(cu_ctx, torch.int32, "cu_ctx"),
                                       int(n_seqs), int(n_kv_heads), int(max_ctx),
                                       _ptr(keep_idx, torch.int32, "keep_idx"), _ptr(cu_keep, torch.int32, "cu_keep"),
                                       _stream(stream)))
    return keep_idx, cu_keep


def vc_compress_quant(ctx: Context, k, v, cu_ctx, cu_blk, bits, max_blk, blocks, stream=None):
    n_seqs = cu_ctx.numel() - 1
    _check(load().vc_compress_quant(ctx.handle, _ptr(k, torch.bfloat16, "k"), _ptr(v, torch.bfloat16, "v"),
                                    _ptr(cu_ctx, torch.int32, "cu_ctx"), _ptr(cu_blk, torch.int32, "cu_blk"), n_seqs,
                                    k.shape[1], bits, max_blk, _ptr(blocks, torch.uint8, "blocks"), _stream(stream)))


def vc_decompress_quant(ctx: Context, blocks, cu_blk, cu_ctx, bits, max_blk, k_out, v_out, stream=None):
    n_seqs = cu_ctx.numel() - 1
    _check(load().vc_decompress_quant(ctx.handle, _ptr(blocks, torch.uint8, "blocks"), _ptr(cu_blk, torch.int32, "cu_blk"),
                                      _ptr(cu_ctx, torch.int32, "cu_ctx"), n_seqs, k_out.shape[1], bits, max_blk,
                                      _ptr(k_out, torch.bfloat16, "k_out"), _ptr(v_out, torch.bfloat16, "v_out"),
                                      _stream(stream)))


def vc_topk_keep(ctx: Context, scores, cu_ctx, cu_keep, n_kv_heads, keep_idx, forced_first=None, forced_last=None,
                 stream=None):
    n_seqs = cu_ctx.numel() - 1
    _check(load().vc_topk_keep(ctx.handle, _ptr(scores, torch.float32, "scores"), _ptr(cu_ctx, torch.int32, "cu_ctx"),
                               _ptr(cu_keep, torch.int32, "cu_keep"), _ptr(forced_first, torch.int32, "forced_first"),
                               _ptr(forced_last, torch.int32, "forced_last"), n_seqs, n_kv_heads,
                               _ptr(keep_idx, torch.int32, "keep_idx"), _stream(stream)))


def vc_iter_time_model(model_bytes, batch, kv_full_bytes, c, x, bw_hbm, bw_inter):
    """Eq. 3 of the paper: returns (t_iter, t_gpu, t_xfer) in seconds."""
    ti, tg, tx = C.c_double(), C.c_double(), C.c_double()
    _check(load().vc_iter_time_model(model_bytes, batch, kv_full_bytes, c, x, bw_hbm, bw_inter,
                                     C.byref(ti), C.byref(tg), C.byref(tx)))
    return ti.value, tg.value, tx.value


class Sched:
    """vc_sched: the reserve rings, Admit and the execution loop (host side only)."""

    def __init__(self, windows, t_iter, bw, hbm_bytes, model_bytes, resident_bytes=0.0, capacity=1024):
        self._h = C.c_void_p()
        _check(load().vc_sched_create(int(windows), t_iter, bw, hbm_bytes, model_bytes, resident_bytes,
                                      C.byref(self._h)))
        self.windows = int(windows)
        self._cap = int(capacity)
        self._kick = (C.c_int64 * self._cap)()
        self._ver = (C.c_int64 * self._cap)()

    def close(self):
        if self._h:
            load().vc_sched_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_resident(self, resident_bytes):
        _check(load().vc_sched_set_resident(self._h, resident_bytes))

    def span(self, kv_full_bytes) -> int:
        n = C.c_int32()
        _check(load().vc_sched_span(self._h, kv_full_bytes, C.byref(n)))
        return n.value

    def admit(self, req, kv_full_bytes, x) -> int:
        d = C.c_int32()
        _check(load().vc_sched_admit(self._h, int(req), kv_full_bytes, int(x), C.byref(d)))
        return d.value

    def cancel(self, req):
        _check(load().vc_sched_cancel(self._h, int(req)))

    def step(self):
        nk, nv = C.c_int32(), C.c_int32()
        _check(load().vc_sched_step(self._h, self._kick, C.byref(nk), self._ver, C.byref(nv), self._cap))
        return list(self._kick[:nk.value]), list(self._ver[:nv.value])

    def rings(self):
        t = (C.c_double * self.windows)()
        b = (C.c_double * self.windows)()
        now = C.c_int64()
        _check(load().vc_sched_rings(self._h, t, b, C.byref(now)))
        return list(t), list(b), now.value
