"""Seeded synthetic inputs for the draft / verify / accept / swap path.

This module only *makes inputs*: random tensors, the stand-in compressors (a min/max group
quantiser that writes block records, a top-k token dropper) and planted logits.  None of the
method's own arithmetic (dequantisation, attention, arg-max, index complement) lives here; the
GPU library and the CPU oracle each implement that on their own and both are fed from the
tensors made here.  Everything is plain torch ops, so the same code runs on the CPU for small
cases and on the GPU for the full-size ones; a (seed, device) pair fixes the values.

The shapes follow the paper's long-context setting (8B-class GQA attention layer, 32k-131k
context, 10-25 % token budgets, 4- and 2-bit caches, draft lengths of a few tens); they stand in
for its datasets, which are not available.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import torch

HEAD_DIM = 128
RECORD_BYTES = 5120


def gen(seed: int, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def randn_bf16(shape, g: torch.Generator) -> torch.Tensor:
    """N(0,1) drawn in fp32, rounded to bf16 (round to nearest even)."""
    return torch.randn(shape, generator=g, device=g.device, dtype=torch.float32).to(torch.bfloat16)


def tokens_per_block(bits: int) -> int:
    return {4: 32, 2: 64}[bits]


# ------------------------------------------------------------------------------------------------
# stand-in quantising compressor: asymmetric min/max per group, fp16 scale and zero
# ------------------------------------------------------------------------------------------------
def _minmax_codes(x: torch.Tensor, dim: int, levels: int):
    """x fp32; groups reduce over `dim`.  zero = fp16(min), scale = fp16((max-min)/levels),
    code = clamp(rne((x - zero) * (1/scale)), 0, levels) with the stored fp16 values, every step
    one fp32 operation; a constant group gets scale 0 and code 0."""
    mn = x.amin(dim=dim, keepdim=True)
    mx = x.amax(dim=dim, keepdim=True)
    zero = (mn + 0.0).to(torch.float16)
    scale = ((mx - mn) / levels).to(torch.float16)
    zf, sf = zero.float(), scale.float()
    safe = torch.where(sf > 0, sf, torch.ones_like(sf))
    code = torch.round((x - zf) * (1.0 / safe)).clamp_(0, levels)
    code = torch.where(sf > 0, code, torch.zeros_like(code))
    return code.to(torch.int64), scale, zero


def _bytes_of_words(words: torch.Tensor) -> torch.Tensor:
    """int64 holding unsigned 32-bit values [..., n] -> uint8 [..., 4n], little endian."""
    parts = [((words >> (8 * k)) & 0xFF) for k in range(4)]
    return torch.stack(parts, dim=-1).to(torch.uint8).flatten(-2)


def _bytes_of_halves(h: torch.Tensor) -> torch.Tensor:
    """fp16 [..., n] -> uint8 [..., 2n] (native little endian)."""
    return h.contiguous().view(torch.uint8).reshape(*h.shape[:-1], h.shape[-1] * 2)


def quantize_records(k: torch.Tensor, v: torch.Tensor, bits: int) -> torch.Tensor:
    """Compress one sequence's bf16 K, V [T, Hkv, 128] (T a multiple of the block length) into
    block records, uint8 [Hkv, T/TB, 5120], in the layout the library header describes: keys are
    quantised per channel over the TB tokens of a block, values per token over groups of TB
    channels."""
    tb = tokens_per_block(bits)
    levels = (1 << bits) - 1
    t, hkv, d = k.shape
    assert d == HEAD_DIM and t % tb == 0 and v.shape == k.shape
    nb = t // tb
    dev = k.device
    # [H, nb, tb, 128]
    kf = k.float().view(nb, tb, hkv, d).permute(2, 0, 1, 3)
    vf = v.float().view(nb, tb, hkv, d).permute(2, 0, 1, 3)

    per_word = 32 // bits
    # element e of a 32-bit word sits at bit 16*(e % 2) + bits*(e // 2)
    e = torch.arange(per_word, device=dev)
    sh = 16 * (e % 2) + bits * (e // 2)

    kc, ks, kz = _minmax_codes(kf, 2, levels)                       # scale/zero [H, nb, 1, 128]
    kc = kc.reshape(hkv, nb, tb, d // per_word, per_word)
    k_words = (kc << sh.view(1, 1, 1, 1, per_word)).sum(-1).reshape(hkv, nb, tb * d // per_word)
    k_bytes = _bytes_of_words(k_words)

    ngrp = d // tb
    vg = vf.reshape(hkv, nb, tb, ngrp, tb)
    vc, vs, vz = _minmax_codes(vg, 4, levels)                       # scale/zero [H, nb, tb, ngrp, 1]
    vc = vc.reshape(hkv, nb, tb, d)
    # token t = per_word*j + e ; channel d = 64*c + 16*q + n  ->  word order [c][j][n][q]
    vc = vc.view(hkv, nb, 4, per_word, 2, 4, 16).permute(0, 1, 4, 2, 6, 5, 3)   # H nb c j n q e
    words = (vc << sh.view(1, 1, 1, 1, 1, 1, per_word)).sum(-1).reshape(hkv, nb, 512)
    v_bytes = _bytes_of_words(words)

    k_meta = torch.cat([_bytes_of_halves(ks.reshape(hkv, nb, d)),
                        _bytes_of_halves(kz.reshape(hkv, nb, d))], dim=-1)
    vs_gt = vs.reshape(hkv, nb, tb, ngrp).transpose(2, 3).reshape(hkv, nb, d)
    vz_gt = vz.reshape(hkv, nb, tb, ngrp).transpose(2, 3).reshape(hkv, nb, d)
    v_meta = torch.cat([_bytes_of_halves(vs_gt), _bytes_of_halves(vz_gt)], dim=-1)

    rec = torch.cat([k_bytes, v_bytes, k_meta, v_meta], dim=-1).contiguous()
    assert rec.shape == (hkv, nb, RECORD_BYTES)
    return rec


# ------------------------------------------------------------------------------------------------
# stand-in token-dropping compressor
# ------------------------------------------------------------------------------------------------
def topk_keep(n_ctx: int, n_keep: int, n_first: int, n_last: int, n_lists: int,
              g: torch.Generator, return_scores: bool = False):
    """Kept positions for `n_lists` (sequence, KV head) lists over a context of n_ctx tokens:
    always the first n_first and last n_last positions, the remaining slots by the highest
    seeded N(0,1) score (ties to the lower position); ascending int32 [n_lists, n_keep]."""
    n_keep = min(n_keep, n_ctx)
    n_first = min(n_first, n_keep)
    n_last = min(n_last, n_keep - n_first)
    score = torch.randn((n_lists, n_ctx), generator=g, device=g.device, dtype=torch.float32)
    raw = score.clone() if return_scores else None
    score[:, :n_first] = float("inf")
    if n_last:
        score[:, n_ctx - n_last:] = float("inf")
    order = torch.sort(score, dim=1, descending=True, stable=True).indices[:, :n_keep]
    keep = torch.sort(order, dim=1).values.to(torch.int32).contiguous()
    return (keep, raw) if return_scores else keep


def dropped_from_keep(keep: torch.Tensor, n_ctx: int) -> torch.Tensor:
    """The compressor's own view (positions it evicted): ascending int32 [n_lists, n_ctx-n_keep].
    Built by masking, as a compressor would; the library turns it back into kept lists."""
    n_lists, _ = keep.shape
    gone = torch.ones((n_lists, n_ctx), dtype=torch.bool, device=keep.device)
    gone.scatter_(1, keep.long(), False)
    return gone.nonzero()[:, 1].view(n_lists, -1).to(torch.int32).contiguous()


# ------------------------------------------------------------------------------------------------
# verify logits with a known arg-max
# ------------------------------------------------------------------------------------------------
def planted_logits(n_rows: int, vocab: int, g: torch.Generator, peak: float = 10.0):
    """fp32 N(0,1) logits [n_rows, vocab] with one entry per row raised to `peak` (far above the
    largest of `vocab` normals), so the arg-max is known by construction.  Returns (logits, ids)."""
    logits = torch.randn((n_rows, vocab), generator=g, device=g.device, dtype=torch.float32)
    ids = torch.randint(0, vocab, (n_rows,), generator=g, device=g.device, dtype=torch.int64)
    logits[torch.arange(n_rows, device=g.device), ids] = peak
    return logits, ids.to(torch.int32)


def drafts_with_prefix(ids: torch.Tensor, cu_win, prefix_len, vocab: int) -> torch.Tensor:
    """Draft ids that agree with `ids` for prefix_len[b] positions of sequence b, then differ."""
    draft = ids.clone()
    for b in range(len(cu_win) - 1):
        w0, w1 = int(cu_win[b]), int(cu_win[b + 1])
        p = int(prefix_len[b])
        if p < w1 - w0:
            draft[w0 + p:w1] = (ids[w0 + p:w1] + 1 + 7 * b) % vocab
            same = draft[w0 + p] == ids[w0 + p]
            if bool(same):
                draft[w0 + p] = (ids[w0 + p] + 1) % vocab
    return draft


# ------------------------------------------------------------------------------------------------
# one layer's workload
# ------------------------------------------------------------------------------------------------
@dataclass
class Layer:
    """Everything one pass of the hot path over one attention layer needs (torch tensors on one
    device unless named *_host).  Entries that a mode does not use stay None."""
    n_q_heads: int
    n_kv_heads: int
    scale: float
    ctx_len: list                      # tokens per sequence (full context)
    q: torch.Tensor                    # bf16 [B, Hq, 128] draft queries
    k_full: torch.Tensor               # bf16 [sum ctx, Hkv, 128]
    v_full: torch.Tensor
    cu_ctx: torch.Tensor               # int32 [B+1]
    keep_idx: torch.Tensor = None      # int32, lists (b, h) back to back
    dropped_idx: torch.Tensor = None
    cu_keep: torch.Tensor = None       # int32 [B+1] (per-head counts, prefix summed)
    cu_drop: torch.Tensor = None
    max_keep: int = 0
    blocks: dict = field(default_factory=dict)      # bits -> uint8 [records, 5120]
    cu_blk: dict = field(default_factory=dict)      # bits -> int32 [B+1]
    max_blk: dict = field(default_factory=dict)
    tail_k: torch.Tensor = None        # bf16 [sum tail, Hkv, 128]
    tail_v: torch.Tensor = None
    cu_tail: torch.Tensor = None
    max_tail: int = 0
    win: list = None                   # window length per sequence
    q_win: torch.Tensor = None         # bf16 [sum w, Hq, 128]
    k_win: torch.Tensor = None
    v_win: torch.Tensor = None
    cu_win: torch.Tensor = None
    logits: torch.Tensor = None        # fp32 [sum rows, vocab]
    cu_rows: torch.Tensor = None
    ids_star: torch.Tensor = None      # planted arg-max ids [sum rows]
    draft_ids: torch.Tensor = None     # int32 [sum w]
    prefix_len: list = None            # planted accept lengths


def _cu(counts, device) -> torch.Tensor:
    c = [0]
    for n in counts:
        c.append(c[-1] + int(n))
    return torch.tensor(c, dtype=torch.int32, device=device)


def make_layer(seed: int, device, *, ctx_len, n_q_heads=32, n_kv_heads=8,
               outlier_channels: int = 0, keep=None, keep_first=64, keep_last=256,
               quant_bits=(), quant_seqs=None, tail_len=None, win=None,
               vocab: int = 0, bonus_row: bool = False, prefix_len=None) -> Layer:
    """Build one layer's inputs.

    ctx_len     list of context lengths
    keep        None, or per-sequence kept-token counts (0 = this sequence is not token-dropped)
    quant_bits  tuple of bit widths to make block records for; quant_seqs = which sequences are
                quantised (default all).  A quantised sequence compresses floor(len/TB)*TB tokens;
                the remainder is prepended to its bf16 tail.
    tail_len    None or per-sequence number of extra recent tokens kept in bf16
    win         None or per-sequence verify window
    """
    g = gen(seed, device)
    nseq = len(ctx_len)
    total = int(sum(ctx_len))
    k_full = randn_bf16((total, n_kv_heads, HEAD_DIM), g)
    v_full = randn_bf16((total, n_kv_heads, HEAD_DIM), g)
    if outlier_channels:
        kf = k_full.float()
        for h in range(n_kv_heads):
            ch = torch.randperm(HEAD_DIM, generator=g, device=g.device)[:outlier_channels]
            kf[:, h, ch] *= 10.0
        k_full = kf.to(torch.bfloat16)
    q = randn_bf16((nseq, n_q_heads, HEAD_DIM), g)
    cu_ctx = _cu(ctx_len, device)
    lay = Layer(n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, scale=1.0 / math.sqrt(HEAD_DIM),
                ctx_len=[int(n) for n in ctx_len], q=q, k_full=k_full, v_full=v_full, cu_ctx=cu_ctx)

    if keep is not None:
        lists, drops = [], []
        for b in range(nseq):
            nk = int(keep[b])
            if nk == 0:
                lists.append(torch.zeros((n_kv_heads, 0), dtype=torch.int32, device=device))
                drops.append(torch.zeros((n_kv_heads, 0), dtype=torch.int32, device=device))
                continue
            kp = topk_keep(lay.ctx_len[b], nk, keep_first[b] if isinstance(keep_first, (list, tuple)) else keep_first,
                           keep_last[b] if isinstance(keep_last, (list, tuple)) else keep_last, n_kv_heads, g)
            lists.append(kp)
            drops.append(dropped_from_keep(kp, lay.ctx_len[b]))
        lay.keep_idx = torch.cat([x.reshape(-1) for x in lists]).contiguous()
        lay.dropped_idx = torch.cat([x.reshape(-1) for x in drops]).contiguous()
        lay.cu_keep = _cu([x.shape[1] for x in lists], device)
        lay.cu_drop = _cu([x.shape[1] for x in drops], device)
        lay.max_keep = max(x.shape[1] for x in lists)

    extra_tail = [0] * nseq
    if quant_bits:
        qs = set(range(nseq)) if quant_seqs is None else set(quant_seqs)
        for bits in quant_bits:
            tb = tokens_per_block(bits)
            recs, nblk = [], []
            for b in range(nseq):
                if b not in qs:
                    nblk.append(0)
                    continue
                lo = int(cu_ctx[b])
                nb = lay.ctx_len[b] // tb
                nblk.append(nb)
                if nb:
                    r = quantize_records(k_full[lo:lo + nb * tb], v_full[lo:lo + nb * tb], bits)
                    recs.append(r.reshape(-1, RECORD_BYTES))
                extra_tail[b] = max(extra_tail[b], lay.ctx_len[b] - nb * tb) if len(quant_bits) == 1 else 0
            lay.blocks[bits] = (torch.cat(recs) if recs else
                                torch.zeros((0, RECORD_BYTES), dtype=torch.uint8, device=device)).contiguous()
            lay.cu_blk[bits] = _cu(nblk, device)
            lay.max_blk[bits] = max(nblk) if nblk else 0

    if tail_len is not None or any(extra_tail):
        tl = [0] * nseq if tail_len is None else [int(x) for x in tail_len]
        ks, vs, counts = [], [], []
        for b in range(nseq):
            hi = int(cu_ctx[b + 1])
            rem = extra_tail[b]
            fresh_k = randn_bf16((tl[b], n_kv_heads, HEAD_DIM), g)
            fresh_v = randn_bf16((tl[b], n_kv_heads, HEAD_DIM), g)
            ks += [k_full[hi - rem:hi], fresh_k]
            vs += [v_full[hi - rem:hi], fresh_v]
            counts.append(rem + tl[b])
        lay.tail_k = torch.cat(ks).contiguous()
        lay.tail_v = torch.cat(vs).contiguous()
        lay.cu_tail = _cu(counts, device)
        lay.max_tail = max(counts)

    if win is not None:
        lay.win = [int(w) for w in win]
        tw = sum(lay.win)
        lay.q_win = randn_bf16((tw, n_q_heads, HEAD_DIM), g)
        lay.k_win = randn_bf16((tw, n_kv_heads, HEAD_DIM), g)
        lay.v_win = randn_bf16((tw, n_kv_heads, HEAD_DIM), g)
        lay.cu_win = _cu(lay.win, device)
        if vocab:
            rows = [w + (1 if bonus_row else 0) for w in lay.win]
            lay.cu_rows = _cu(rows, device)
            lay.logits, lay.ids_star = planted_logits(sum(rows), vocab, g)
            if prefix_len is None:
                prefix_len = [int(torch.randint(0, w + 1, (1,), generator=g, device=g.device)) for w in lay.win]
            lay.prefix_len = [int(p) for p in prefix_len]
            # ids aligned with the window rows (skip the bonus rows)
            sel = torch.cat([torch.arange(int(lay.cu_rows[b]), int(lay.cu_rows[b]) + lay.win[b], device=device)
                             for b in range(nseq)]) if tw else torch.zeros(0, dtype=torch.long, device=device)
            lay.draft_ids = drafts_with_prefix(lay.ids_star[sel].clone(), lay.cu_win.tolist(),
                                               lay.prefix_len, vocab).to(torch.int32).contiguous()
    return lay


# ------------------------------------------------------------------------------------------------
# the five workloads; `shrink` divides context lengths so the CPU oracle can do a whole case
# ------------------------------------------------------------------------------------------------
SEED_BASE = 0x5EED0000


def config(idx: int, device, shrink: int = 1, layer: int = 0) -> Layer:
    seed = SEED_BASE + idx + 1000 * layer
    if idx == 0:      # tiny GQA layer, int4, outlier key channels
        return make_layer(seed, device, ctx_len=[4096 // shrink], n_q_heads=8, n_kv_heads=2,
                          outlier_channels=4, quant_bits=(4,), win=[8], vocab=32000)
    if idx == 1:      # token dropping, 8 sequences of 32768, keep 2048
        n = 32768 // shrink
        return make_layer(seed, device, ctx_len=[n] * 8, keep=[2048 // shrink] * 8,
                          keep_first=64 // shrink, keep_last=256 // shrink, win=[16] * 8, vocab=32000)
    if idx == 2:      # quantised, 16 sequences of 65536, int4 and int2, window 32
        n = 65536 // shrink
        return make_layer(seed, device, ctx_len=[n] * 16, quant_bits=(4, 2), win=[32] * 16, vocab=32000)
    if idx == 3:      # one layer of the 32-layer round: 1 sequence of 131072, int4, tail, window 64
        n = 131072 // shrink
        return make_layer(seed, device, ctx_len=[n], quant_bits=(4,), tail_len=[63], win=[64],
                          vocab=128256 if layer == 0 else 0)
    if idx == 4:      # ragged mixed batch
        g = gen(seed ^ 0xABCDEF, "cpu")
        u = torch.rand(32, generator=g)
        lens = [max(64, int(2048 * (64.0 ** float(x))) // shrink) for x in u]
        quant = [bool(x) for x in (torch.rand(32, generator=g) < 0.5)]
        wins = [int(x) for x in torch.randint(4, 65, (32,), generator=g)]
        keep, kf, kl = [], [], []
        for b in range(32):
            if quant[b]:
                keep.append(0); kf.append(0); kl.append(0)
            else:
                nk = -(-lens[b] // 10)
                keep.append(nk); kf.append(min(64, nk // 4)); kl.append(min(256, nk // 2))
        return make_layer(seed, device, ctx_len=lens, keep=keep, keep_first=kf, keep_last=kl,
                          quant_bits=(4,), quant_seqs=[b for b in range(32) if quant[b]],
                          win=wins, vocab=128256 // (shrink if shrink > 1 else 1))
    raise ValueError("config index 0..4")
