"""GPU parity: every entry point of the C ABI against the fp64 oracle on the same seeded inputs.
Attention outputs: max|gpu - oracle| / max|oracle| <= 1e-2 (bf16 outputs).  accept_len, next_token,
arg-max ids and kept-index lists: bit-exact."""
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


@pytest.fixture(params=[(100000, 1), (0, 1), (0, 0)], ids=["finish-in-kernel", "merge-launch", "merge-attends-tail"])
def draft_finish(request, tunables):
    """Tiny single-source launches finish inside the split kernel (by default up to 64 workgroups); here
    VC_DRAFT_FUSED makes every single-source launch do so, or none.  With a merge launch, the bf16 tail is
    attended to by workgroups of the split launch (one more partial; the default) or by the merge itself
    (VC_DRAFT_TAIL_SPLIT = 0).  The draft cases run all three ways."""
    tunables.set("VC_DRAFT_FUSED", request.param[0])
    tunables.set("VC_DRAFT_TAIL_SPLIT", request.param[1])
    return request.param[0]


def check_draft(lib, ctx, lay, tag, lse_tol=H.LSE_TOL, hints=None, **sel):
    kw = H.draft_kwargs(lay, **sel)
    kw.update(hints or {})      # sum_keep / sum_blk: they steer the launch shape only
    print(f"[draft] {tag} {sel}", flush=True)
    out, lse = H.gpu_draft(lib, ctx, lay, **kw)
    ref, ref_lse = H.oracle_draft(lay, kw)
    err = H.rel_err(out, ref)
    assert err <= H.TOL, f"{tag}: rel err {err}"
    fin = np.isfinite(ref_lse)
    assert np.abs(lse.cpu().numpy()[fin] - ref_lse[fin]).max() <= lse_tol
    assert np.array_equal(np.isneginf(lse.cpu().numpy()), np.isneginf(ref_lse))
    return out


# ------------------------------------------------------------------ draft, bf16 rows
@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (8, 4), (16, 2), (16, 1)])
def test_draft_bf16_contiguous_gqa(lib, ctx, hq, hkv, draft_finish):
    lay = synth.make_layer(11, DEV, ctx_len=[700, 1, 333], n_q_heads=hq, n_kv_heads=hkv)
    check_draft(lib, ctx, lay, f"bf16 g={hq // hkv}", use_pool=True)


def test_draft_bf16_gather_ragged_with_tail_and_empty(lib, ctx, draft_finish):
    lay = synth.make_layer(12, DEV, ctx_len=[900, 70, 2000, 64], n_q_heads=8, n_kv_heads=2,
                           keep=[257, 70, 0, 5], keep_first=[4, 2, 0, 1], keep_last=[9, 3, 0, 2],
                           tail_len=[3, 0, 17, 0])
    check_draft(lib, ctx, lay, "gather+tail", use_pool=True, use_keep=True, use_tail=True)
    check_draft(lib, ctx, lay, "gather", use_pool=True, use_keep=True)
    # sequence 2 keeps nothing and has no tail in the second call: out = 0, lse = -inf there


def test_draft_bf16_many_splits(lib, ctx, draft_finish):
    lay = synth.make_layer(13, DEV, ctx_len=[5000], n_q_heads=8, n_kv_heads=2, keep=[3001], keep_first=64, keep_last=256)
    check_draft(lib, ctx, lay, "gather splits", use_pool=True, use_keep=True)


def test_draft_bf16_two_wave_workgroups(lib, ctx, tunables, draft_finish):
    """The row kernel's form for ragged batches (two waves per workgroup), forced on small inputs:
    contiguous pool, gathered rows, 16 heads per KV head."""
    tunables.set("VC_DRAFT_ROW_WAVES", 2)
    tunables.set("VC_DRAFT_MIN_TOK", 128)
    lay = synth.make_layer(14, DEV, ctx_len=[700, 1, 333, 64, 65], n_q_heads=16, n_kv_heads=1)
    check_draft(lib, ctx, lay, "two waves, contiguous", use_pool=True)
    lay = synth.make_layer(15, DEV, ctx_len=[5000, 90], n_q_heads=8, n_kv_heads=2, keep=[3001, 33], keep_first=[64, 2],
                           keep_last=[256, 3], tail_len=[5, 0])
    check_draft(lib, ctx, lay, "two waves, gather", use_pool=True, use_keep=True, use_tail=True)


# ------------------------------------------------------------------ draft, block records
@pytest.mark.parametrize("bits", [4, 2])
@pytest.mark.parametrize("hq,hkv", [(8, 2), (2, 2), (16, 2), (6, 2), (10, 2), (32, 2), (14, 2)])
def test_draft_quant(lib, ctx, bits, hq, hkv, draft_finish):
    tb = synth.tokens_per_block(bits)
    lay = synth.make_layer(20 + bits, DEV, ctx_len=[tb * 37, tb, tb * 8 + 5], n_q_heads=hq, n_kv_heads=hkv,
                           quant_bits=(bits,), outlier_channels=3)
    check_draft(lib, ctx, lay, f"int{bits} g={hq // hkv}", bits=bits, use_tail=True)


@pytest.mark.parametrize("bits", [4, 2])
def test_draft_quant_long_with_tail(lib, ctx, bits, draft_finish):
    lay = synth.make_layer(30 + bits, DEV, ctx_len=[20000 + 13, 4096], n_q_heads=8, n_kv_heads=2, quant_bits=(bits,),
                           tail_len=[63, 1])
    check_draft(lib, ctx, lay, f"int{bits} long", bits=bits, use_tail=True)


@pytest.mark.parametrize("nseq", [2, 32])
def test_draft_long_tails_in_both_merge_variants(lib, ctx, nseq, draft_finish):
    """Tails beyond 128 tokens take the merge kernel's chunk loop; a small batch runs its four-group
    variant, a batch of 256 (sequence, head) pairs the one-group variant."""
    rng = np.random.default_rng(nseq)
    lens = [int(x) * 32 for x in rng.integers(1, 9, nseq)]
    tails = [200, 130] if nseq == 2 else [int(x) for x in rng.integers(0, 150, nseq)]
    lay = synth.make_layer(60 + nseq, DEV, ctx_len=lens, n_q_heads=8, n_kv_heads=2, quant_bits=(4,), tail_len=tails)
    check_draft(lib, ctx, lay, f"long tails, {nseq} sequences", bits=4, use_tail=True)
    lay = synth.make_layer(70 + nseq, DEV, ctx_len=lens, n_q_heads=8, n_kv_heads=2, tail_len=tails)
    check_draft(lib, ctx, lay, f"tail only, {nseq} sequences", use_tail=True)     # no split at all: the merge does everything


@pytest.mark.parametrize("nseq", [5, 64, 65])
def test_draft_ragged_mixed_batch_with_length_hints(lib, ctx, tunables, nseq):
    """A ragged batch whose descriptor carries the sums of its list lengths: up to 64 sequences both
    split kernels are launched over the splits that exist (every wave finds its sequence from the
    prefix arrays), beyond that over a grid sized by the longest sequence.  The splits are the same
    either way, so the two launches must agree bit for bit, and both with the oracle."""
    rng = np.random.default_rng(900 + nseq)
    lens = [int(x) for x in rng.integers(1, 1500, nseq)]
    lens[nseq // 2] = 6000                       # one long sequence makes the batch ragged
    lens[0] = 40
    keep = [int(rng.integers(0, n + 1)) if i % 3 else 0 for i, n in enumerate(lens)]
    keep[nseq // 2] = 2500
    first = [min(k, 2) for k in keep]
    last = [min(k - f, 3) for k, f in zip(keep, first)]
    lay = synth.make_layer(90 + nseq, DEV, ctx_len=lens, n_q_heads=8, n_kv_heads=2, keep=keep, keep_first=first,
                           keep_last=last, quant_bits=(4,), tail_len=[int(x) for x in rng.integers(0, 20, nseq)])
    outs = []
    tunables.set("VC_DRAFT_FUSED", 0)            # (a launch that finishes in the kernel is never flat)
    for flat in (1, 0):
        tunables.set("VC_DRAFT_FLAT", flat)
        # small splits so that even these short lists are cut several times
        tunables.set("VC_DRAFT_MIN_TOK", 128)
        tunables.set("VC_DRAFT_MIN_BLK", 4)
        tunables.set("VC_DRAFT_BF16_WGS", 300)
        tunables.set("VC_DRAFT_QUANT_WGS", 500)
        o1 = check_draft(lib, ctx, lay, f"hints rows, {nseq} sequences, flat {flat}", use_pool=True, use_keep=True,
                         use_tail=True, hints=dict(sum_keep=int(lay.cu_keep[-1])))
        o2 = check_draft(lib, ctx, lay, f"hints records, {nseq} sequences, flat {flat}", bits=4, use_tail=True,
                         hints=dict(sum_blk=int(lay.cu_blk[4][-1])))
        outs.append((o1.clone(), o2.clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


@pytest.mark.parametrize("bits", [4, 2])
def test_draft_flat_launch_with_two_head_passes_and_tails(lib, ctx, tunables, bits):
    """Sixteen query heads per KV head take two passes of the record kernel; in a flat launch of a ragged
    batch the workgroups behind the last split attend to the tails, once per (sequence, KV head) - not once per
    pass - and a sequence without records still gets its tail."""
    tb = synth.tokens_per_block(bits)
    lens = [tb * 50 + 3, tb * 2, 7, tb * 9 + 1, tb * 160]          # sequence 2 has no full block: tail only
    lay = synth.make_layer(120 + bits, DEV, ctx_len=lens, n_q_heads=32, n_kv_heads=2, quant_bits=(bits,),
                           tail_len=[5, 0, 0, 40, 70])
    tunables.set("VC_DRAFT_FUSED", 0)
    tunables.set("VC_DRAFT_MIN_BLK", 4)
    tunables.set("VC_DRAFT_QUANT_WGS", 200)
    outs = []
    for flat in (1, 0):
        tunables.set("VC_DRAFT_FLAT", flat)
        outs.append(check_draft(lib, ctx, lay, f"int{bits}, 16 heads per KV head, flat {flat}", bits=bits, use_tail=True,
                                hints=dict(sum_blk=int(lay.cu_blk[bits][-1]))).clone())
    assert torch.equal(outs[0], outs[1])


def test_draft_rows_flat_launch_sixteen_heads_with_tails(lib, ctx, tunables):
    """The row kernel's tail workgroups with more query heads than waves: two-wave workgroups of a ragged
    batch take eight heads of a KV head each, tails of 0, 1, 33 and 100 tokens (one and four chunks)."""
    lens = [3000, 40, 900, 5, 260]
    keep = [1500, 40, 0, 5, 130]
    lay = synth.make_layer(130, DEV, ctx_len=lens, n_q_heads=16, n_kv_heads=1, keep=keep, keep_first=[8, 2, 0, 1, 4],
                           keep_last=[16, 3, 0, 2, 8], tail_len=[33, 0, 100, 1, 64])
    tunables.set("VC_DRAFT_FUSED", 0)
    tunables.set("VC_DRAFT_MIN_TOK", 128)
    tunables.set("VC_DRAFT_BF16_WGS", 64)
    outs = []
    for flat in (1, 0):
        tunables.set("VC_DRAFT_FLAT", flat)
        outs.append(check_draft(lib, ctx, lay, f"rows, 16 heads per KV head, flat {flat}", use_pool=True, use_keep=True,
                                use_tail=True, hints=dict(sum_keep=int(lay.cu_keep[-1]))).clone())
    assert torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("bits", [4, 2])
def test_draft_quant_just_inside_the_fp16_range_limits(lib, ctx, bits):
    """The header's number range for block records: value scale and |value zero| up to 4094, key
    metadata times the scaled query inside fp16.  Key outlier channels x100 (key zero points of
    several hundred) and values of +-4000 (value scales 533 for int4, 2667 for int2) sit just inside."""
    tb = synth.tokens_per_block(bits)
    lens = [tb * 21, tb * 5]
    lay = synth.make_layer(81, DEV, ctx_len=lens, n_q_heads=8, n_kv_heads=2)
    k = lay.k_full.float()
    k[:, :, [7, 64, 101]] *= 100.0
    v = (lay.v_full.float() * 1300.0).clamp_(-4000.0, 4000.0)
    v[3::tb, :, 0] = 4000.0; v[3::tb, :, 1] = -4000.0            # groups that span the whole range
    lay.k_full, lay.v_full = k.to(torch.bfloat16).contiguous(), v.to(torch.bfloat16).contiguous()
    recs, lo = [], 0
    for n in lens:
        recs.append(synth.quantize_records(lay.k_full[lo:lo + n], lay.v_full[lo:lo + n], bits).reshape(-1, 5120))
        lo += n
    lay.blocks[bits] = torch.cat(recs).contiguous()
    lay.cu_blk[bits] = torch.tensor([0, lens[0] // tb, sum(lens) // tb], dtype=torch.int32, device=DEV)
    lay.max_blk[bits] = lens[0] // tb
    meta = lay.blocks[bits][:, 4608:5120].contiguous().view(torch.float16).float()
    assert meta.abs().max().item() <= 4094.0 and meta[:, :128].max().item() >= (500.0 if bits == 4 else 2600.0)
    # scores reach +-60 here (x100 key channels), and an fp16 operand carries 2^-11 relative rounding: the
    # log-sum-exp is held to 1e-3 of its magnitude instead of the absolute bound used at N(0,1) scale
    out = check_draft(lib, ctx, lay, f"int{bits} range limits", lse_tol=0.06, bits=bits)
    assert torch.isfinite(out.float()).all()


@pytest.mark.parametrize("bits", [4, 2])
def test_draft_lossless_grid_equals_bf16_path(lib, ctx, bits):
    """Cross-kernel: records built from exact grid values dequantise to the bf16 values, so the
    record kernel and the bf16 kernel must agree (both are also checked against the oracle)."""
    tb = synth.tokens_per_block(bits)
    g = synth.gen(77, DEV)
    lv = 1 << bits
    n_tok = 6 * tb
    codes = torch.randint(0, lv, (n_tok, 2, 128), generator=g, device=DEV)
    codes[0::tb] = 0
    codes[1::tb] = lv - 1
    codes[:, :, 0::tb] = 0
    codes[:, :, 1::tb] = lv - 1
    k = (codes.float() / 8.0 - 1.0).to(torch.bfloat16)
    codes2 = codes.flip(0)
    v = (codes2.float() / 8.0 + 0.5).to(torch.bfloat16)
    lay = synth.make_layer(5, DEV, ctx_len=[n_tok], n_q_heads=8, n_kv_heads=2)
    lay.k_full, lay.v_full = k.contiguous(), v.contiguous()
    lay.blocks[bits] = synth.quantize_records(lay.k_full, lay.v_full, bits).reshape(-1, 5120).contiguous()
    lay.cu_blk[bits] = torch.tensor([0, 6], dtype=torch.int32, device=DEV)
    lay.max_blk[bits] = 6
    a = check_draft(lib, ctx, lay, "grid bf16", use_pool=True)
    b = check_draft(lib, ctx, lay, "grid quant", bits=bits)
    assert (a.float() - b.float()).abs().max().item() <= 2e-2 * a.float().abs().max().item()


# ------------------------------------------------------------------ verify
@pytest.mark.parametrize("win", [[1], [3, 8], [16, 5, 1], [33], [64, 2]])
@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (16, 2)])
def test_verify_windows(lib, ctx, win, hq, hkv):
    ctx_len = [1000 + 37 * i for i in range(len(win))]
    lay = synth.make_layer(40 + len(win), DEV, ctx_len=ctx_len, n_q_heads=hq, n_kv_heads=hkv, win=win)
    print(f"[verify] win={win} hq={hq} hkv={hkv}", flush=True)
    out, lse = H.gpu_verify(lib, ctx, lay)
    ref, ref_lse = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= H.LSE_TOL


@pytest.mark.parametrize("hq,hkv,wins", [(16, 2, [40, 3, 33]), (8, 2, [100, 64, 65]), (32, 2, [17])])
def test_verify_more_than_256_rows_per_kv_head(lib, ctx, hq, hkv, wins):
    """Windows whose rows (window x GQA ratio) exceed one 256-row block: 320, 400 and 272 rows."""
    lens = [700 + 130 * i for i in range(len(wins))]
    lay = synth.make_layer(44 + hq, DEV, ctx_len=lens, n_q_heads=hq, n_kv_heads=hkv, win=wins)
    out, lse = H.gpu_verify(lib, ctx, lay)
    ref, ref_lse = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= H.LSE_TOL


def test_verify_short_context_and_zero_window(lib, ctx):
    lay = synth.make_layer(45, DEV, ctx_len=[5, 31, 32, 0 + 1], n_q_heads=8, n_kv_heads=2, win=[4, 0, 7, 2])
    out, lse = H.gpu_verify(lib, ctx, lay)
    ref, ref_lse = H.oracle_verify(lay)
    assert H.rel_err(out, ref) <= H.TOL


def test_verify_window_of_one_equals_draft(lib, ctx):
    lay = synth.make_layer(46, DEV, ctx_len=[777, 100], n_q_heads=8, n_kv_heads=2, win=[1, 1])
    out, _ = H.gpu_verify(lib, ctx, lay)
    lay.q = lay.q_win
    kw = dict(pool_k=lay.k_full, pool_v=lay.v_full, cu_ctx=lay.cu_ctx, max_keep=777,
              tail_k=lay.k_win, tail_v=lay.v_win, cu_tail=lay.cu_win, max_tail=1)
    d_out, _ = H.gpu_draft(lib, ctx, lay, **kw)
    assert (out.float() - d_out.float()).abs().max().item() <= 2e-2 * out.float().abs().max().item()


# ------------------------------------------------------------------ accept / keep
@pytest.fixture(params=[1, 0], ids=["one-launch", "two-launches"])
def accept_launches(request, tunables):
    """Short scans finish inside the scan launch; VC_ACCEPT_FUSED 0 forces the second launch that
    long scans take.  Every accept case runs both ways."""
    tunables.set("VC_ACCEPT_FUSED", request.param)
    return request.param


def test_accept_planted_ties_bonus(lib, ctx, accept_launches):
    lay = synth.make_layer(50, DEV, ctx_len=[8] * 6, n_q_heads=4, n_kv_heads=2, win=[5, 5, 3, 1, 64, 7], vocab=32000,
                           bonus_row=True, prefix_len=[0, 5, 2, 1, 64, 3])
    lay.logits[3, 100] = 10.0; lay.logits[3, 31999] = 10.0       # ties: lowest index must win
    lay.logits[7, :] = float("-inf"); lay.logits[7, 17] = -5.0
    lay.logits[9, :] = 0.25
    a, n, am = H.gpu_accept(lib, ctx, lay)
    ra, rn, ram = H.oracle_accept(lay)
    assert np.array_equal(am, ram) and np.array_equal(a, ra) and np.array_equal(n, rn)


def test_accept_signed_zero_ties_across_segments(lib, ctx, accept_launches):
    """Row maximum 0 held by -0.0 at a low index and +0.0 in another thread / another 8192-logit
    segment (and the other way round): the lower index wins, as in the oracle."""
    lay = synth.make_layer(52, DEV, ctx_len=[8] * 2, n_q_heads=4, n_kv_heads=2, win=[3, 2], vocab=32000)
    lay.logits.clamp_(max=-0.5)
    lay.logits[0, 5] = -0.0; lay.logits[0, 20000] = 0.0          # different segments
    lay.logits[1, 5] = 0.0; lay.logits[1, 20000] = -0.0
    lay.logits[2, 40] = -0.0; lay.logits[2, 41] = 0.0            # same segment, neighbouring threads
    lay.logits[3, 9000] = -0.0; lay.logits[3, 9000 + 4 * 256] = 0.0   # same thread's next vector
    lay.logits[4, :] = -0.0; lay.logits[4, 31999] = 0.0
    a, n, am = H.gpu_accept(lib, ctx, lay)
    ra, rn, ram = H.oracle_accept(lay)
    assert ram.tolist() == [5, 5, 40, 9000, 0]
    assert np.array_equal(am, ram) and np.array_equal(a, ra) and np.array_equal(n, rn)


@pytest.mark.parametrize("vocab", [128256, 32000, 1001, 7])
def test_accept_vocab_sizes(lib, ctx, vocab, accept_launches):
    lay = synth.make_layer(51, DEV, ctx_len=[8] * 5, n_q_heads=4, n_kv_heads=2, win=[4, 9, 1, 0, 33], vocab=vocab)
    a, n, am = H.gpu_accept(lib, ctx, lay)
    ra, rn, ram = H.oracle_accept(lay)
    assert np.array_equal(am, ram) and np.array_equal(a, ra) and np.array_equal(n, rn)
    assert a.tolist() == lay.prefix_len or vocab == 7


def test_accept_many_calls_reuse_the_contexts_counters(lib, ctx):
    """The one-launch form counts workgroups on counters the context owns, 16 sets used in turn and
    left at zero by the call that used them: 40 calls in a row over batches of different shapes, each
    checked against the oracle."""
    lays = [synth.make_layer(53 + i, DEV, ctx_len=[8] * n, n_q_heads=4, n_kv_heads=2, win=win, vocab=vocab, bonus_row=bonus)
            for i, (n, win, vocab, bonus) in enumerate([(3, [4, 1, 7], 32000, True), (1, [2], 128256, False),
                                                        (6, [1, 0, 3, 5, 2, 64], 9000, True)])]
    refs = [H.oracle_accept(lay) for lay in lays]
    for i in range(40):
        lay, (ra, rn, ram) = lays[i % 3], refs[i % 3]
        a, n, am = H.gpu_accept(lib, ctx, lay)
        assert np.array_equal(am, ram) and np.array_equal(a, ra) and np.array_equal(n, rn), f"call {i}"


def test_keep_from_dropped(lib, ctx):
    lay = synth.make_layer(60, DEV, ctx_len=[5000, 33, 20, 777], n_q_heads=8, n_kv_heads=4, keep=[500, 33, 0, 78],
                           keep_first=[64, 2, 0, 8], keep_last=[256, 3, 0, 16])
    ref_keep, ref_cu = O.keep_from_dropped(H.npi(lay.dropped_idx), H.npi(lay.cu_drop), lay.ctx_len, 4)
    keep = torch.full((len(ref_keep),), -1, dtype=torch.int32, device=DEV)
    cu = torch.full((5,), -1, dtype=torch.int32, device=DEV)
    lib.vc_keep_from_dropped(ctx, lay.dropped_idx, lay.cu_drop, lay.cu_ctx, 4, max(lay.ctx_len), keep, cu)
    torch.cuda.synchronize()
    assert np.array_equal(cu.cpu().numpy(), ref_cu)
    assert np.array_equal(keep.cpu().numpy(), ref_keep)


def test_keep_from_dropped_gap_shapes(lib, ctx):
    """The kernel writes the gaps between neighbouring dropped entries: lists with nothing dropped (one gap that
    is the whole sequence), everything dropped, one position, long kept runs in the middle, lengths at and around
    the 1024 gaps a workgroup takes, a different list per head."""
    rng = np.random.default_rng(77)
    hkv = 3
    lens = [4096, 1, 1, 1023, 1024, 1025, 3000, 2048, 10000, 0, 517]
    ndrop = [0, 0, 1, 1023, 1000, 1024, 1500, 2047, 9000, 0, 200]
    lists, cu_drop = [], [0]
    for n, nd in zip(lens, ndrop):
        for h in range(hkv):
            if n == 3000:        # two long kept runs: positions 100..899 and 2000..2699 are never dropped
                pool = np.array([p for p in range(n) if not (100 <= p < 900 or 2000 <= p < 2700)])
            else:
                pool = np.arange(n)
            lists.append(np.sort(rng.choice(pool, size=nd, replace=False)).astype(np.int32))
        cu_drop.append(cu_drop[-1] + nd)
    dropped = np.concatenate(lists) if lists else np.zeros(0, np.int32)
    cu_ctx = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cu_drop = np.array(cu_drop, dtype=np.int32)
    ref_keep, ref_cu = O.keep_from_dropped(dropped, cu_drop, lens, hkv)
    keep = torch.full((len(ref_keep) + 8,), -1, dtype=torch.int32, device=DEV)     # 8 guard entries behind the lists
    cu = torch.full((len(lens) + 1,), -1, dtype=torch.int32, device=DEV)
    lib.vc_keep_from_dropped(ctx, torch.from_numpy(np.concatenate([dropped, np.zeros(4, np.int32)])).to(DEV),
                             torch.from_numpy(cu_drop).to(DEV), torch.from_numpy(cu_ctx).to(DEV), hkv, max(lens), keep, cu)
    torch.cuda.synchronize()
    assert np.array_equal(cu.cpu().numpy(), ref_cu)
    got = keep.cpu().numpy()
    assert np.array_equal(got[:len(ref_keep)], ref_keep)
    assert (got[len(ref_keep):] == -1).all(), "stores behind the last list"


# ------------------------------------------------------------------ swap-in
def test_swap_in_bytes_tickets_and_wait(lib, ctx):
    n = 8 << 20
    src = torch.randint(0, 255, (n,), dtype=torch.uint8).pin_memory()
    dst = torch.zeros(n, dtype=torch.uint8, device=DEV)
    chunk = 1 << 20
    chunks = [(i * chunk, i * chunk, chunk) for i in range(8)]
    first = lib.vc_swap_in(ctx, src, dst, chunks)
    lib.vc_swap_wait(ctx, first + 7)                          # current stream waits on the last chunk
    total = dst.to(torch.int64).sum()
    torch.cuda.synchronize()
    assert lib.vc_swap_query(ctx, first + 7) and lib.vc_swap_query(ctx, first)
    assert int(total) == int(src.to(torch.int64).sum())
    assert torch.equal(dst.cpu(), src)
    first2 = lib.vc_swap_in(ctx, src, dst, [(0, chunk, 16)])
    assert first2 == first + 8
    lib.vc_swap_sync(ctx)
    assert torch.equal(dst[chunk:chunk + 16].cpu(), src[:16])


def test_swap_in_rejects_pageable_and_bad_ticket(lib, ctx):
    src = torch.zeros(1024, dtype=torch.uint8)
    dst = torch.zeros(1024, dtype=torch.uint8, device=DEV)
    with pytest.raises(lib.VcError) as e:
        lib.vc_swap_in(ctx, src, dst, [(0, 0, 1024)])
    assert e.value.status == 1
    with pytest.raises(lib.VcError):
        lib.vc_swap_wait(ctx, 1 << 40)
    # the context still works afterwards
    pin = src.pin_memory()
    t = lib.vc_swap_in(ctx, pin, dst, [(0, 0, 1024)])
    lib.vc_swap_sync(ctx)
    assert lib.vc_swap_query(ctx, t)


# ------------------------------------------------------------------ error paths that need a context
def test_workspace_too_small_and_null(lib, ctx):
    lay = synth.make_layer(70, DEV, ctx_len=[128], n_q_heads=8, n_kv_heads=2)
    out = torch.empty_like(lay.q)
    kw = H.draft_kwargs(lay, use_pool=True)
    with pytest.raises(lib.VcError) as e:
        lib.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=2, workspace=torch.empty(16, dtype=torch.uint8, device=DEV), **kw)
    assert e.value.status == 3
    with pytest.raises(lib.VcError) as e:
        lib.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=2, workspace=None, **kw)
    assert e.value.status == 3


def test_main_kernel_timing_events(lib, ctx):
    """vc_time_main_kernel brackets the main kernel inside the call: 0 < kernel time <= call time,
    and the hook disarms itself (a second call leaves the events alone)."""
    lay = synth.config(0, DEV)
    kw = H.draft_kwargs(lay, bits=4)
    out = torch.empty_like(lay.q)
    ws = torch.empty(max(lib.vc_draft_workspace_bytes(lay.n_q_heads, lay.n_kv_heads, 1, **kw), 16), dtype=torch.uint8, device=DEV)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for e in ev:
        e.record()
    lib.vc_time_main_kernel(ctx, ev[1], ev[2])
    ev[0].record()
    lib.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=lay.n_kv_heads, workspace=ws, **kw)
    ev[3].record()
    torch.cuda.synchronize()
    inner, outer = ev[1].elapsed_time(ev[2]), ev[0].elapsed_time(ev[3])
    assert 0.0 < inner <= outer
    lib.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=lay.n_kv_heads, workspace=ws, **kw)
    torch.cuda.synchronize()
    assert ev[1].elapsed_time(ev[2]) == inner
    with pytest.raises(lib.VcError):
        lib.vc_time_main_kernel(ctx, ev[0], None)


# ------------------------------------------------------------------ optional data validation
def _report(lib, ctx, fn):
    rep = torch.full((2,), 7, dtype=torch.int64, device=DEV)
    fn(rep)
    torch.cuda.synchronize()
    count, key = rep.tolist()
    return count, (None if key == -1 else (key >> 56, (key >> 32) & 0xFFFFFF, key & 0xFFFFFFFF))


def test_validate_comp_and_full_descriptors(lib, ctx):
    lay = synth.make_layer(90, DEV, ctx_len=[900, 70, 2000], n_q_heads=8, n_kv_heads=2, keep=[257, 70, 5],
                           keep_first=[4, 2, 1], keep_last=[9, 3, 2], quant_bits=(4,), tail_len=[3, 0, 17], win=[4, 0, 9])
    kw = H.draft_kwargs(lay, bits=4, use_pool=True, use_keep=True, use_tail=True)
    geo = dict(n_q_heads=8, n_kv_heads=2, n_seqs=3)
    assert _report(lib, ctx, lambda r: lib.vc_validate_comp_kv(ctx, r, **geo, **kw)) == (0, None)
    # a kept position out of range, in list (sequence 0, head 1), entry 256
    bad = dict(kw); bad["keep_idx"] = lay.keep_idx.clone(); bad["keep_idx"][257 + 256] = 900
    assert _report(lib, ctx, lambda r: lib.vc_validate_comp_kv(ctx, r, **geo, **bad)) == (1, (4, 0, 256))
    # two entries swapped in list (sequence 2, head 0): positions 1 and 2 out of order (one violation at entry 2 or two)
    bad["keep_idx"] = lay.keep_idx.clone()
    base = (257 + 70) * 2
    bad["keep_idx"][base + 1], bad["keep_idx"][base + 2] = lay.keep_idx[base + 2].item(), lay.keep_idx[base + 1].item()
    count, first = _report(lib, ctx, lambda r: lib.vc_validate_comp_kv(ctx, r, **geo, **bad))
    assert count >= 1 and first[0] == 5 and first[1] == 2
    # a host-side maximum that under-estimates, and a decreasing prefix array
    low = dict(kw); low["max_blk"] = lay.max_blk[4] - 1
    assert _report(lib, ctx, lambda r: lib.vc_validate_comp_kv(ctx, r, **geo, **low)) == (1, (2, 2, 2))
    dec = dict(kw); dec["cu_tail"] = torch.tensor([0, 3, 2, 20], dtype=torch.int32, device=DEV)
    count, first = _report(lib, ctx, lambda r: lib.vc_validate_comp_kv(ctx, r, **geo, **dec))
    assert first == (1, 1, 3)
    # a kept list longer than its sequence
    long = dict(kw); long["cu_ctx"] = torch.tensor([0, 900, 960, 2960], dtype=torch.int32, device=DEV)
    count, first = _report(lib, ctx, lambda r: lib.vc_validate_comp_kv(ctx, r, **geo, **long))
    assert first[0] == 3 and first[1] == 1
    full = dict(k=lay.k_full, v=lay.v_full, cu_ctx=lay.cu_ctx, max_ctx=2000, max_win=9)
    assert _report(lib, ctx, lambda r: lib.vc_validate_full_kv(ctx, r, lay.cu_win, 13, **geo, **full)) == (0, None)
    full["max_win"] = 8
    assert _report(lib, ctx, lambda r: lib.vc_validate_full_kv(ctx, r, lay.cu_win, 13, **geo, **full)) == (1, (2, 2, 4))
    assert lib.vc_stream_status(ctx) is True
