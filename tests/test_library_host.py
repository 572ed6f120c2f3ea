"""CPU-only checks of the built library: it loads, exports every symbol the header declares, and
its host-side argument validation and split planning behave (no kernel is launched here)."""
import ctypes as C
import os
import re

import pytest

import paper_2605_17613_amd as vc
from paper_2605_17613_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "vericache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vc_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = vc.load()
    names = header_functions()
    assert len(names) >= 14
    for name in names:
        assert hasattr(lib, name), f"{name} declared in the header but not exported"
    assert sorted(B.EXPORTS) == names
    assert vc.vc_version() == "0.1"


def desc(**kw):
    d = B.vc_comp_kv()
    d.n_seqs, d.n_q_heads, d.n_kv_heads, d.head_dim, d.bits = 2, 8, 2, 128, 4
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def ws_bytes(d):
    n = C.c_size_t()
    st = vc.load().vc_draft_workspace_bytes(C.byref(d), C.byref(n))
    return st, n.value


def test_draft_descriptor_validation():
    assert ws_bytes(desc())[0] == B.VC_OK
    assert ws_bytes(desc(head_dim=64))[0] == B.VC_ERR_UNSUPPORTED
    assert ws_bytes(desc(n_q_heads=7))[0] == B.VC_ERR_INVALID_ARG
    assert ws_bytes(desc(n_q_heads=68, n_kv_heads=2))[0] == B.VC_ERR_UNSUPPORTED
    assert ws_bytes(desc(max_blk=-1))[0] == B.VC_ERR_INVALID_ARG
    assert ws_bytes(desc(pool_k=0x1000))[0] == B.VC_ERR_INVALID_ARG            # pool_v / cu_ctx missing
    assert ws_bytes(desc(pool_k=0x1008, pool_v=0x1000, cu_ctx=0x2000))[0] == B.VC_ERR_INVALID_ARG  # misaligned
    assert ws_bytes(desc(blocks=0x1000, cu_blk=0x2000, bits=3))[0] == B.VC_ERR_UNSUPPORTED
    assert b"bits 3" in vc.load().vc_last_error()
    st = vc.load().vc_draft_workspace_bytes(None, None)
    assert st == B.VC_ERR_INVALID_ARG


def test_draft_workspace_grows_with_work_and_covers_every_split():
    small = ws_bytes(desc(blocks=0x1000, cu_blk=0x2000, max_blk=64))[1]
    big = ws_bytes(desc(blocks=0x1000, cu_blk=0x2000, max_blk=1 << 16))[1]
    both = ws_bytes(desc(blocks=0x1000, cu_blk=0x2000, max_blk=64, pool_k=0x3000, pool_v=0x4000, cu_ctx=0x5000,
                         max_keep=1000))[1]
    assert small >= 2 * 8 * 130 * 4 and big > small and both > small
    assert small % (130 * 4) == 0
    # a launch this small finishes inside its split kernel, tail included: the tail needs no partial slot
    tail = ws_bytes(desc(blocks=0x1000, cu_blk=0x2000, max_blk=64, tail_k=0x3000, tail_v=0x4000, cu_tail=0x5000,
                         max_tail=63))[1]
    assert tail == small
    # with a merge launch, the tail is one more partial per (sequence, query head), made by workgroups of the
    # split launch - unless VC_DRAFT_TAIL_SPLIT = 0 leaves it to the merge
    big_tail = ws_bytes(desc(blocks=0x1000, cu_blk=0x2000, max_blk=1 << 16, tail_k=0x3000, tail_v=0x4000, cu_tail=0x5000,
                             max_tail=63))[1]
    assert big_tail == big + 2 * 8 * 130 * 4
    # (its workgroups sit in grid slices behind the sequences': beyond 32767 sequences the merge keeps the tail)
    many = dict(blocks=0x1000, cu_blk=0x2000, max_blk=64, n_seqs=40000)
    assert ws_bytes(desc(tail_k=0x3000, tail_v=0x4000, cu_tail=0x5000, max_tail=63, **many))[1] == ws_bytes(desc(**many))[1]
    try:
        vc.vc_set_tunable("VC_DRAFT_TAIL_SPLIT", 0)
        assert ws_bytes(desc(blocks=0x1000, cu_blk=0x2000, max_blk=1 << 16, tail_k=0x3000, tail_v=0x4000, cu_tail=0x5000,
                             max_tail=63))[1] == big
    finally:
        vc.vc_set_tunable("VC_DRAFT_TAIL_SPLIT", -1)
    # the sum hint changes the chunking (load balance), never below one slot per list
    hinted = ws_bytes(desc(blocks=0x1000, cu_blk=0x2000, max_blk=1 << 16, sum_blk=1 << 16))[1]
    assert hinted >= big


def test_verify_and_accept_host_validation():
    lib = vc.load()
    d = B.vc_full_kv()
    d.n_seqs, d.n_q_heads, d.n_kv_heads, d.head_dim, d.max_ctx, d.max_win = 2, 8, 2, 128, 1000, 1025
    d.k, d.v, d.cu_ctx = 0x1000, 0x2000, 0x3000
    n = C.c_size_t()
    assert lib.vc_verify_workspace_bytes(C.byref(d), 10, C.byref(n)) == B.VC_ERR_UNSUPPORTED   # more than 4096 rows per KV head
    d.max_win = 64
    assert lib.vc_verify_workspace_bytes(C.byref(d), 10, C.byref(n)) == B.VC_OK and n.value >= 10 * 8 * 130 * 4
    d.cu_ctx = None
    assert lib.vc_verify_workspace_bytes(C.byref(d), 10, C.byref(n)) == B.VC_ERR_INVALID_ARG
    assert lib.vc_accept_workspace_bytes(64, 128256, C.byref(n)) == B.VC_OK and n.value == 64 * 16 * 8   # one key per row and 8192-logit segment
    assert lib.vc_accept_workspace_bytes(64, 0, C.byref(n)) == B.VC_ERR_INVALID_ARG
    # calls that need a context reject a NULL one without touching the device
    assert lib.vc_swap_sync(None) == B.VC_ERR_INVALID_ARG
    assert lib.vc_swap_query(None, 0) == B.VC_ERR_INVALID_ARG
    assert lib.vc_destroy(None) == B.VC_OK


def test_verify_plan_of_a_ragged_batch():
    """Host logic of the verify plan: a batch whose sum of lengths is well below n_seqs x max_ctx gets
    shorter chunks, and a large one also room for the work list behind its partials."""
    lib = vc.load()
    d = B.vc_full_kv()
    d.n_seqs, d.n_q_heads, d.n_kv_heads, d.head_dim, d.max_ctx, d.max_win = 32, 32, 8, 128, 131072, 64
    d.k, d.v, d.cu_ctx = 0x1000, 0x2000, 0x3000
    chunk, nchunk, n = C.c_int32(), C.c_int32(), C.c_size_t()

    def plan(sum_ctx):
        d.sum_ctx = sum_ctx
        assert lib.vc_verify_plan(C.byref(d), C.byref(chunk), C.byref(nchunk)) == B.VC_OK
        assert lib.vc_verify_workspace_bytes(C.byref(d), 1000, C.byref(n)) == B.VC_OK
        partials = 1000 * 32 * nchunk.value * 130 * 4
        return chunk.value, nchunk.value, n.value - partials

    uniform = plan(0)                        # unknown sum: planned as 32 sequences of max_ctx, one round of 256 workgroups
    assert uniform[2] == 0 and uniform[0] * uniform[1] >= 131072 + 64
    ragged = plan(949359)                    # the mixed batch of 32 sequences, 2048 ... 131072 tokens
    assert ragged[0] < uniform[0] and ragged[0] % 512 == 0      # shorter chunks, whole tiles after two halvings
    assert ragged[2] > 0 and ragged[2] % 4 == 0                 # the list area
    small = plan(40000)                      # ragged but small: the plain grid, no list
    assert small[2] == 0
    d.n_seqs = 600                           # more sequences than a list ranks
    assert plan(600 * 20000)[2] == 0


def test_binding_rejects_wrong_dtypes_before_calling_the_library():
    import torch
    with pytest.raises(TypeError):
        B._ptr(torch.zeros(4, dtype=torch.float32), torch.bfloat16, "q")
    with pytest.raises(ValueError):
        B._ptr(torch.zeros(4, 4, dtype=torch.bfloat16).t(), torch.bfloat16, "q")


def test_tunables_are_a_process_table_not_the_environment(monkeypatch):
    """The plan reads tunables from the library's own table: set and restored through the C ABI, and
    an environment change after the first use has no effect on the query (so a query and its call
    cannot disagree because the environment moved between them)."""
    lib = vc.load()
    d = B.vc_full_kv()
    d.n_seqs, d.n_q_heads, d.n_kv_heads, d.head_dim, d.max_ctx, d.max_win = 16, 32, 8, 128, 65536, 32
    d.k, d.v, d.cu_ctx = 0x1000, 0x2000, 0x3000
    chunk, nchunk = C.c_int32(), C.c_int32()
    assert lib.vc_verify_plan(C.byref(d), C.byref(chunk), C.byref(nchunk)) == B.VC_OK
    base = chunk.value
    monkeypatch.setenv("VC_VERIFY_WGS", "1024")
    assert lib.vc_verify_plan(C.byref(d), C.byref(chunk), C.byref(nchunk)) == B.VC_OK and chunk.value == base
    assert vc.vc_get_tunable("VC_VERIFY_WGS") is None
    vc.vc_set_tunable("VC_VERIFY_WGS", 1024)
    assert vc.vc_get_tunable("VC_VERIFY_WGS") == 1024
    assert lib.vc_verify_plan(C.byref(d), C.byref(chunk), C.byref(nchunk)) == B.VC_OK and chunk.value < base
    vc.vc_set_tunable("VC_VERIFY_WGS", -1)
    assert lib.vc_verify_plan(C.byref(d), C.byref(chunk), C.byref(nchunk)) == B.VC_OK and chunk.value == base
    with pytest.raises(vc.VcError):
        vc.vc_set_tunable("VC_NO_SUCH_THING", 1)
    assert lib.vc_stream_status(None, None) == B.VC_ERR_INVALID_ARG
    assert lib.vc_validate_comp_kv(None, None, None, None) == B.VC_ERR_INVALID_ARG


def test_every_documented_tunable_is_known_and_the_reverse():
    """The header's tunable list and the library's name table are the same set: every VC_* name in the
    header's tunable comment can be set and read back, and no other VC_DRAFT_ / VC_VERIFY_ / VC_ACCEPT_
    name is accepted."""
    import re
    text = open(os.path.join(ROOT, "include", "vericache.h")).read()
    block = text[text.index("Launch-shape tunables"):text.index("vc_status vc_set_tunable")]
    names = sorted(set(re.findall(r"VC_(?:DRAFT|VERIFY|ACCEPT)_[A-Z0-9_]+", block)))
    assert len(names) >= 14, names
    for n in names:
        assert vc.vc_get_tunable(n) is None, n
        vc.vc_set_tunable(n, 3)
        assert vc.vc_get_tunable(n) == 3, n
        vc.vc_set_tunable(n, -1)
        assert vc.vc_get_tunable(n) is None, n
    for bogus in ("VC_DRAFT_TAPER", "VC_DRAFT_", "VC_VERIFY_WGS2", "vc_draft_flat", ""):
        with pytest.raises(vc.VcError):
            vc.vc_set_tunable(bogus, 1)


def test_draft_plan_reacts_to_its_launch_shape_tunables():
    """The workspace of a draft call holds one partial per split: cutting a launch for more workgroups,
    or allowing shorter splits, must grow it, and the defaults must come back afterwards."""
    def ws(**kw):
        d = B.vc_comp_kv()
        d.n_seqs, d.n_q_heads, d.n_kv_heads, d.head_dim = 16, 32, 8, 128
        d.bits, d.blocks, d.cu_blk, d.max_blk, d.sum_blk = 4, 0x1000, 0x2000, 2048, 16 * 2048
        n = C.c_size_t()
        assert vc.load().vc_draft_workspace_bytes(C.byref(d), C.byref(n)) == B.VC_OK
        return n.value
    base = ws()
    try:
        vc.vc_set_tunable("VC_DRAFT_QUANT_WGS", 3072)
        assert ws() > base
        vc.vc_set_tunable("VC_DRAFT_QUANT_WGS", 128)
        assert ws() < base
    finally:
        vc.vc_set_tunable("VC_DRAFT_QUANT_WGS", -1)
    assert ws() == base
