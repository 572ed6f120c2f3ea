"""Plain fp64 CPU oracle of the VeriCache hot path (TEST INFRASTRUCTURE, not a product path).

What it computes, step by step, in IEEE double precision (paper section 4.1, core loop):

  draft   (step 1) - one query token attends, with exact softmax attention, to whatever the
                     compressed cache holds for its sequence: retained bf16 rows picked by a
                     kept-index list (compressor interface, section 6: positions dropped per
                     (layer, head), bit scheme 16), group-quantised int4 / int2 block records
                     (bit scheme 4 / 2, keys per channel, values per token), and a bf16 tail of
                     recent tokens.
  verify  (step 2) - every drafted position i attends to the full KV plus drafted positions 0..i.
  accept  (step 3) - greedy: first position whose draft id differs from the arg-max of the
                     verify logits; the correction (or bonus) token follows.
  keep    (section 6, CompressedKV.dropped_indices) - complement of the dropped positions.
  compress / decompress (section 6, Compressor interface, quantising methods) - min/max group
                     quantiser into block records (decisions in float32, spelled out at
                     quantise_groups) and its inverse, rounded once to bf16.
  topk_keep (section 6, what update() decides) - kept positions from importance scores.
  pack_rows / swap_in_rows (appendix B.1, the (1 - c) * KV_full transfer) - the dropped rows kept
                     on the host, and their placement back into the pool.

Every input is taken in the byte layout that the C header of the library describes in prose
(bf16 / fp16 bit patterns, packed codes); the unpacking below is written from that prose and
shares no code with the GPU library.  bf16, fp16 and the small integer codes convert to double
exactly, so the only rounding in here is double-precision arithmetic itself.

Pins (tests, "-m 'not gpu'"): softmax rows sum to one and are shift invariant; identical keys
give the mean of the values; a dominant key returns its value row; brute force with Python loops
on tiny shapes; split/merge invariance; zero dropping equals full attention; lossless quantisation
grids equal bf16 attention; hand-packed records (written element by element from the layout
prose) unpack to the planted codes; causal rows do not see later rows; planted arg-max logits,
planted ties, brute-force set difference; for the compressor side: hand-computed groups and
rounding ties, closed-form records against a byte-by-byte hand packer, error bound and extreme
codes per group, key/value group axes, a second vectorised packer, grid data surviving a round
trip, single rounding to bf16, brute-force top-k with exact ties and forced positions.
No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

HEAD_DIM = 128
RECORD_BYTES = 5120
_K_CODES, _V_CODES, _K_META, _V_META = 0, 2048, 4096, 4608


# --------------------------------------------------------------------------------------------
# exact widening of 16-bit floating point bit patterns
# --------------------------------------------------------------------------------------------
def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exact (bf16 is the top half of an IEEE float32)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f16_to_f64(bits: np.ndarray) -> np.ndarray:
    """IEEE fp16 bit patterns (uint16) -> float64, exact."""
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def tokens_per_block(bits: int) -> int:
    """Quantisation group: 32 tokens / 32 channels for 4 bit, 64 / 64 for 2 bit."""
    if bits == 4:
        return 32
    if bits == 2:
        return 64
    raise ValueError("bits must be 4 or 2")


# --------------------------------------------------------------------------------------------
# block records -> dequantised K, V   (KIVI-style axes: keys per channel, values per token)
# --------------------------------------------------------------------------------------------
def unpack_records(records: np.ndarray, bits: int):
    """Dequantise block records.

    records: uint8 [n_heads, n_blocks, 5120].  One record holds TB = 32 (int4) or 64 (int2)
    consecutive tokens of one KV head.  Codes sit in little-endian 32-bit words of E = 32/bits
    elements; element e of a word is the field at bit 16*(e mod 2) + bits*(e // 2):
      bytes    0..2047  key codes, token-major: token t owns words 4*bits*t ...; word wi of a
                        token holds channels E*wi .. E*wi+E-1
      bytes 2048..4095  value codes in 128 slots of 16 bytes; slot L = 64*c + 16*j + n
                        (c<2, j<4, n<16) holds words q<4; word q belongs to channel
                        d = 64*c + 16*q + n and holds tokens E*j .. E*j+E-1
      bytes 4096..4607  key scale[128] then key zero[128], fp16, one pair per channel
      bytes 4608..5119  value scale[g][t] then value zero[g][t], fp16, g = channel group
                        (d // TB), t = token in block
    x_hat = scale * code + zero, evaluated in double (no intermediate rounding).

    Returns (K_hat, V_hat) float64 [n_heads, n_blocks*TB, 128].
    """
    tb = tokens_per_block(bits)
    rec = np.ascontiguousarray(records, dtype=np.uint8)
    if rec.ndim != 3 or rec.shape[2] != RECORD_BYTES:
        raise ValueError("records must be [heads, blocks, 5120] uint8")
    nh, nb, _ = rec.shape
    cmask = (1 << bits) - 1
    per_word = 32 // bits
    words_per_token = HEAD_DIM // per_word

    def field(word, e):
        return (word >> np.uint32(16 * (e % 2) + bits * (e // 2))) & np.uint32(cmask)

    kwords = rec[:, :, _K_CODES:_K_CODES + 2048].copy().view("<u4")  # [nh, nb, 512]
    k_code = np.empty((nh, nb, tb, HEAD_DIM), dtype=np.float64)
    for t in range(tb):
        for d in range(HEAD_DIM):
            word = kwords[:, :, words_per_token * t + d // per_word]
            k_code[:, :, t, d] = field(word, d % per_word)

    vwords = rec[:, :, _V_CODES:_V_CODES + 2048].copy().view("<u4")  # [nh, nb, 512]
    v_code = np.empty((nh, nb, tb, HEAD_DIM), dtype=np.float64)
    for c in range(2):
        for j in range(4):
            for n in range(16):
                slot = 64 * c + 16 * j + n
                for q in range(4):
                    d = 64 * c + 16 * q + n
                    word = vwords[:, :, 4 * slot + q]
                    for e in range(per_word):
                        v_code[:, :, per_word * j + e, d] = field(word, e)

    kmeta = rec[:, :, _K_META:_K_META + 512].copy().view("<u2")       # [nh, nb, 256]
    k_scale = f16_to_f64(kmeta[:, :, 0:128])
    k_zero = f16_to_f64(kmeta[:, :, 128:256])
    k_hat = k_scale[:, :, None, :] * k_code + k_zero[:, :, None, :]

    ngrp = HEAD_DIM // tb
    vmeta = rec[:, :, _V_META:_V_META + 512].copy().view("<u2")
    v_scale = f16_to_f64(vmeta[:, :, 0:128]).reshape(nh, nb, ngrp, tb)
    v_zero = f16_to_f64(vmeta[:, :, 128:256]).reshape(nh, nb, ngrp, tb)
    v_hat = np.empty_like(v_code)
    for d in range(HEAD_DIM):
        g = d // tb
        v_hat[:, :, :, d] = v_scale[:, :, g, :] * v_code[:, :, :, d] + v_zero[:, :, g, :]

    return k_hat.reshape(nh, nb * tb, HEAD_DIM), v_hat.reshape(nh, nb * tb, HEAD_DIM)


# --------------------------------------------------------------------------------------------
# the attention definition
# --------------------------------------------------------------------------------------------
def attend(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float):
    """Softmax attention of one query vector over n keys, textbook definition in double.

    q [128], k [n,128], v [n,128] float64.  s_j = scale * <q, k_j>;  p = softmax(s);
    o = sum_j p_j v_j;  lse = log sum_j exp(s_j).  Returns (o, lse, p).
    An empty key set gives o = 0, lse = -inf.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64).reshape(-1, q.shape[0])
    v = np.asarray(v, dtype=np.float64).reshape(-1, q.shape[0])
    if k.shape[0] == 0:
        return np.zeros_like(q), -np.inf, np.zeros(0)
    s = float(scale) * (k @ q)
    m = s.max()
    e = np.exp(s - m)
    l = e.sum()
    p = e / l
    return p @ v, m + np.log(l), p


def _rows(a, lo, hi, head):
    """bf16 pool [T, Hkv, 128] (uint16 bits) -> float64 rows lo..hi of one head."""
    return bf16_to_f64(np.asarray(a)[lo:hi, head, :])


def draft_keys(b: int, kvh: int, *, n_kv_heads: int,
               pool_k=None, pool_v=None, cu_ctx=None, keep_idx=None, cu_keep=None,
               blocks=None, cu_blk=None, bits: int = 16,
               tail_k=None, tail_v=None, cu_tail=None):
    """Key/value rows sequence b's drafted token sees on KV head kvh (paper section 4.1 step 1).

    Three sources, each optional, concatenated (order does not matter to the result):
      bf16 pool  [T, Hkv, 128] bf16 bits; sequence b owns rows cu_ctx[b]..cu_ctx[b+1]; with
                 keep_idx the retained rows are cu_ctx[b] + keep_idx[(cu_keep[b]*Hkv +
                 kvh*nk) + i], i < nk = cu_keep[b+1]-cu_keep[b] (same count for every head,
                 section 6 scope (i)); without keep_idx every row of the sequence
      blocks     uint8 [*, 5120] block records; sequence b, head kvh owns records
                 cu_blk[b]*Hkv + kvh*nb + i, i < nb = cu_blk[b+1]-cu_blk[b]
      tail       bf16 [Ttail, Hkv, 128] recent tokens, rows cu_tail[b]..cu_tail[b+1]
    """
    ks, vs = [], []
    if pool_k is not None:
        base = int(cu_ctx[b])
        if keep_idx is not None:
            nk = int(cu_keep[b + 1]) - int(cu_keep[b])
            start = int(cu_keep[b]) * n_kv_heads + kvh * nk
            idx = base + np.asarray(keep_idx[start:start + nk], dtype=np.int64)
        else:
            idx = np.arange(base, int(cu_ctx[b + 1]), dtype=np.int64)
        ks.append(bf16_to_f64(np.asarray(pool_k)[idx, kvh, :]))
        vs.append(bf16_to_f64(np.asarray(pool_v)[idx, kvh, :]))
    if blocks is not None:
        nb = int(cu_blk[b + 1]) - int(cu_blk[b])
        start = int(cu_blk[b]) * n_kv_heads + kvh * nb
        rec = np.asarray(blocks).reshape(-1, RECORD_BYTES)[start:start + nb]
        if nb > 0:
            kh, vh = unpack_records(rec[None], bits)
            ks.append(kh[0])
            vs.append(vh[0])
    if tail_k is not None:
        lo, hi = int(cu_tail[b]), int(cu_tail[b + 1])
        ks.append(_rows(tail_k, lo, hi, kvh))
        vs.append(_rows(tail_v, lo, hi, kvh))
    if not ks:
        return np.zeros((0, HEAD_DIM)), np.zeros((0, HEAD_DIM))
    return np.concatenate(ks, axis=0), np.concatenate(vs, axis=0)


def draft_attn_one(q_bits, b: int, h: int, scale: float, *, n_q_heads: int, n_kv_heads: int, **kv):
    """Draft attention output (o [128], lse) of sequence b, query head h (GQA: KV head h // g)."""
    g = n_q_heads // n_kv_heads
    k, v = draft_keys(b, h // g, n_kv_heads=n_kv_heads, **kv)
    q = bf16_to_f64(np.asarray(q_bits)[b, h, :])
    o, lse, _ = attend(q, k, v, scale)
    return o, lse


def draft_attn(q_bits, scale: float, *, n_q_heads: int, n_kv_heads: int, **kv):
    """All sequences and heads: q bf16 bits [B, Hq, 128] -> (out [B,Hq,128], lse [B,Hq]) float64."""
    q_bits = np.asarray(q_bits)
    nseq = q_bits.shape[0]
    out = np.zeros((nseq, n_q_heads, HEAD_DIM))
    lse = np.zeros((nseq, n_q_heads))
    g = n_q_heads // n_kv_heads
    for b in range(nseq):
        for kvh in range(n_kv_heads):
            k, v = draft_keys(b, kvh, n_kv_heads=n_kv_heads, **kv)
            for h in range(kvh * g, (kvh + 1) * g):
                o, s, _ = attend(bf16_to_f64(q_bits[b, h, :]), k, v, scale)
                out[b, h] = o
                lse[b, h] = s
    return out, lse


# --------------------------------------------------------------------------------------------
# verify: causal window over the full KV  (paper section 4.1 step 2)
# --------------------------------------------------------------------------------------------
def verify_attn_one(q_win, k_full, v_full, k_win, v_win, cu_ctx, cu_win,
                    b: int, i: int, h: int, scale: float, *, n_q_heads: int, n_kv_heads: int):
    """Window row i of sequence b, query head h: keys are the sequence's full-KV rows followed by
    window rows 0..i (its own position included).  All arrays are bf16 bit patterns:
    q_win [W, Hq, 128], k_full/v_full [T, Hkv, 128], k_win/v_win [W, Hkv, 128]."""
    g = n_q_heads // n_kv_heads
    kvh = h // g
    lo, hi = int(cu_ctx[b]), int(cu_ctx[b + 1])
    w0 = int(cu_win[b])
    if not 0 <= i < int(cu_win[b + 1]) - w0:
        raise IndexError("window row out of range")
    k = np.concatenate([_rows(k_full, lo, hi, kvh), _rows(k_win, w0, w0 + i + 1, kvh)], axis=0)
    v = np.concatenate([_rows(v_full, lo, hi, kvh), _rows(v_win, w0, w0 + i + 1, kvh)], axis=0)
    q = bf16_to_f64(np.asarray(q_win)[w0 + i, h, :])
    o, lse, _ = attend(q, k, v, scale)
    return o, lse


def verify_attn(q_win, k_full, v_full, k_win, v_win, cu_ctx, cu_win, scale: float,
                *, n_q_heads: int, n_kv_heads: int):
    """All window rows: returns (out [W, Hq, 128], lse [W, Hq]) float64."""
    q_win = np.asarray(q_win)
    nseq = len(cu_win) - 1
    g = n_q_heads // n_kv_heads
    out = np.zeros((q_win.shape[0], n_q_heads, HEAD_DIM))
    lse = np.zeros((q_win.shape[0], n_q_heads))
    for b in range(nseq):
        lo, hi = int(cu_ctx[b]), int(cu_ctx[b + 1])
        w0, w1 = int(cu_win[b]), int(cu_win[b + 1])
        for kvh in range(n_kv_heads):
            # same key order as verify_attn_one: full-KV rows, then the window rows
            k = np.concatenate([_rows(k_full, lo, hi, kvh), _rows(k_win, w0, w1, kvh)], axis=0)
            v = np.concatenate([_rows(v_full, lo, hi, kvh), _rows(v_win, w0, w1, kvh)], axis=0)
            n = hi - lo
            for i in range(w1 - w0):
                for h in range(kvh * g, (kvh + 1) * g):
                    q = bf16_to_f64(q_win[w0 + i, h, :])
                    o, s, _ = attend(q, k[:n + i + 1], v[:n + i + 1], scale)
                    out[w0 + i, h] = o
                    lse[w0 + i, h] = s
    return out, lse


# --------------------------------------------------------------------------------------------
# accept: greedy first mismatch  (paper section 4.1 step 3)
# --------------------------------------------------------------------------------------------
def argmax_row(row: np.ndarray) -> int:
    """Index of the largest logit; the lowest index wins a tie.  Logits are finite or -inf."""
    row = np.asarray(row)
    best = row.max()
    return int(np.flatnonzero(row == best)[0])


def accept(logits, cu_rows, draft_ids, cu_win):
    """Greedy acceptance.

    logits fp32 [R, V]; sequence b owns logits rows cu_rows[b]..cu_rows[b+1] (w_b rows, or
    w_b + 1 when the bonus row is supplied) and draft ids cu_win[b]..cu_win[b+1] (w_b ids).
    Row j is the full-KV prediction for drafted position j.
      a_b    = first j < w_b with draft[j] != argmax(row j), else w_b
      next_b = argmax(row a_b) if that row exists, else -1
    Returns (accept_len [B] int32, next_token [B] int32, argmax_ids [R] int32).
    """
    logits = np.asarray(logits, dtype=np.float32)
    nseq = len(cu_rows) - 1
    amax = np.array([argmax_row(logits[r]) for r in range(logits.shape[0])], dtype=np.int32)
    acc = np.zeros(nseq, dtype=np.int32)
    nxt = np.zeros(nseq, dtype=np.int32)
    for b in range(nseq):
        r0, r1 = int(cu_rows[b]), int(cu_rows[b + 1])
        w0, w1 = int(cu_win[b]), int(cu_win[b + 1])
        w = w1 - w0
        a = w
        for j in range(w):
            if int(draft_ids[w0 + j]) != int(amax[r0 + j]):
                a = j
                break
        acc[b] = a
        nxt[b] = amax[r0 + a] if r0 + a < r1 else -1
    return acc, nxt, amax


# --------------------------------------------------------------------------------------------
# kept-index lists from dropped-index lists  (section 6, CompressedKV.dropped_indices)
# --------------------------------------------------------------------------------------------
def keep_from_dropped(dropped, cu_drop, ctx_len, n_kv_heads: int):
    """Complement of the dropped positions, ascending.

    dropped int32: list (b, h) is dropped[(cu_drop[b]*Hkv + h*nd) + i], i < nd = cu_drop[b+1] -
    cu_drop[b], positions in [0, ctx_len[b]).  The kept lists use the same scheme with
    nk = ctx_len[b] - nd and cu_keep[b] = sum_{b' < b} nk.  Returns (keep_idx, cu_keep) int32.
    """
    dropped = np.asarray(dropped, dtype=np.int64)
    nseq = len(ctx_len)
    cu_keep = np.zeros(nseq + 1, dtype=np.int32)
    pieces = []
    for b in range(nseq):
        nd = int(cu_drop[b + 1]) - int(cu_drop[b])
        n = int(ctx_len[b])
        cu_keep[b + 1] = cu_keep[b] + (n - nd)
        for h in range(n_kv_heads):
            start = int(cu_drop[b]) * n_kv_heads + h * nd
            gone = np.zeros(n, dtype=bool)
            gone[dropped[start:start + nd]] = True
            pieces.append(np.flatnonzero(~gone).astype(np.int32))
    keep = np.concatenate(pieces) if pieces else np.zeros(0, dtype=np.int32)
    return keep, cu_keep


# --------------------------------------------------------------------------------------------
# quantising compressor and its inverse  (section 6: Compressor.compress / decompress for the
# quantisation methods; section 2: keys per channel, values per token)
# --------------------------------------------------------------------------------------------
def quantise_groups(x32: np.ndarray, levels: int):
    """Asymmetric min/max quantisation of groups along the last axis.

    The decisions are integers taken from floating point, so the precision is part of the
    definition: everything below is IEEE float32 (one rounding per operation), the stored scale and
    zero point are fp16 (round to nearest even), and the code is computed from the STORED values:
        zero  = fp16(min)  (-0 stored as +0)    scale = fp16((max - min) / levels)
        code  = clamp(rne((x - zero) * (1 / scale)), 0, levels)      (scale = 0: code 0)
    Returns (code int64 [..., G], scale fp16 [...], zero fp16 [...]).
    """
    x32 = np.asarray(x32, dtype=np.float32)
    mn = x32.min(axis=-1)
    mx = x32.max(axis=-1)
    zero = (mn + np.float32(0.0)).astype(np.float16)
    scale = ((mx - mn) / np.float32(levels)).astype(np.float16)
    zf = zero.astype(np.float32)[..., None]
    sf = scale.astype(np.float32)[..., None]
    pos = sf > 0
    inv = np.float32(1.0) / np.where(pos, sf, np.float32(1.0))
    code = np.rint((x32 - zf) * inv)
    code = np.clip(code, 0, levels)
    code = np.where(pos, code, 0.0).astype(np.int64)
    return code, scale, zero


def _put_field(words, index, e, bits, code):
    """OR `code` into element e of words[..., index] (element e sits at bit 16*(e%2)+bits*(e//2))."""
    words[..., index] |= (code.astype(np.uint32) << np.uint32(16 * (e % 2) + bits * (e // 2)))


def quantize_records(k_bits: np.ndarray, v_bits: np.ndarray, bits: int) -> np.ndarray:
    """bf16 K, V bit patterns [T, n_heads, 128] of one sequence -> block records
    uint8 [n_heads, T // TB, 5120] over its first (T // TB) * TB tokens (the layout is the one
    unpack_records documents).  Keys: one group per channel over the TB tokens of a block;
    values: one group per token over TB consecutive channels."""
    tb = tokens_per_block(bits)
    levels = (1 << bits) - 1
    per_word = 32 // bits
    words_per_token = HEAD_DIM // per_word
    ngrp = HEAD_DIM // tb
    t_all, nh, d = np.asarray(k_bits).shape
    if d != HEAD_DIM:
        raise ValueError("head dim must be 128")
    nb = t_all // tb
    widen = lambda a: (np.ascontiguousarray(a, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    k32 = widen(k_bits)[:nb * tb].reshape(nb, tb, nh, HEAD_DIM)
    v32 = widen(v_bits)[:nb * tb].reshape(nb, tb, nh, HEAD_DIM)
    rec = np.zeros((nh, nb, RECORD_BYTES), dtype=np.uint8)
    for h in range(nh):
        # keys: groups over tokens -> move the token axis last
        kc, ks, kz = quantise_groups(np.transpose(k32[:, :, h, :], (0, 2, 1)), levels)   # [nb, 128, tb]
        kwords = np.zeros((nb, 512), dtype=np.uint32)
        for t in range(tb):
            for ch in range(HEAD_DIM):
                _put_field(kwords, words_per_token * t + ch // per_word, ch % per_word, bits, kc[:, ch, t])
        # values: groups of tb channels of one token
        vc, vs, vz = quantise_groups(v32[:, :, h, :].reshape(nb, tb, ngrp, tb), levels)   # [nb, tb, ngrp, tb]
        vc = vc.reshape(nb, tb, HEAD_DIM)
        vwords = np.zeros((nb, 512), dtype=np.uint32)
        for c in range(2):
            for j in range(4):
                for n in range(16):
                    slot = 64 * c + 16 * j + n
                    for q in range(4):
                        ch = 64 * c + 16 * q + n
                        for e in range(per_word):
                            _put_field(vwords, 4 * slot + q, e, bits, vc[:, per_word * j + e, ch])
        rec[h, :, _K_CODES:_K_CODES + 2048] = kwords.astype("<u4").view(np.uint8).reshape(nb, 2048)
        rec[h, :, _V_CODES:_V_CODES + 2048] = vwords.astype("<u4").view(np.uint8).reshape(nb, 2048)
        kmeta = np.concatenate([ks.view(np.uint16), kz.view(np.uint16)], axis=-1)            # [nb, 256]
        rec[h, :, _K_META:_K_META + 512] = kmeta.astype("<u2").view(np.uint8).reshape(nb, 512)
        vs_gt = np.transpose(vs, (0, 2, 1)).reshape(nb, HEAD_DIM)                             # [g][t]
        vz_gt = np.transpose(vz, (0, 2, 1)).reshape(nb, HEAD_DIM)
        vmeta = np.concatenate([vs_gt.view(np.uint16), vz_gt.view(np.uint16)], axis=-1)
        rec[h, :, _V_META:_V_META + 512] = vmeta.astype("<u2").view(np.uint8).reshape(nb, 512)
    return rec


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round doubles to bf16 (8 significant bits, round to nearest even) in ONE rounding step and
    return the bit patterns.  For values in bf16's normal range (and zero)."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                      # x = m * 2^e, 0.5 <= |m| < 1
    r = np.ldexp(np.rint(np.ldexp(m, 8)), e - 8)   # rint is round-half-to-even; r has <= 8 bits
    f32 = r.astype(np.float32)              # exact: 8 significant bits fit
    return (f32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def dequantize_records(records: np.ndarray, bits: int):
    """Inverse of the quantising compressor: x_hat = scale * code + zero exactly (the sum is exact
    in double), then ONE rounding to bf16.  Returns (k_bits, v_bits) uint16 [T, n_heads, 128]."""
    k_hat, v_hat = unpack_records(records, bits)        # [nh, T, 128] float64
    return (np.ascontiguousarray(np.transpose(f64_to_bf16_bits(k_hat), (1, 0, 2))),
            np.ascontiguousarray(np.transpose(f64_to_bf16_bits(v_hat), (1, 0, 2))))


# --------------------------------------------------------------------------------------------
# kept-index lists from importance scores  (section 6: what an online compressor's update()
# decides per request and head; every head of a layer keeps the same number of positions)
# --------------------------------------------------------------------------------------------
def topk_keep(scores, ctx_len, keep_len, n_kv_heads: int, forced_first=None, forced_last=None):
    """Per (sequence b, head h) list: keep the first F_b and the last L_b positions, fill the
    remaining keep_len[b] - F_b - L_b slots with the highest-scoring other positions (equal
    scores: the lower position wins), and return the kept positions in ascending order.

    scores float32: list (b, h) is scores[(cu_ctx[b]*Hkv + h*N_b) + t], t < N_b = ctx_len[b].
    F_b = min(forced_first[b], keep_len[b]); L_b = min(forced_last[b], keep_len[b] - F_b).
    Returns (keep_idx int32, cu_keep int32) in the list layout of keep_from_dropped.
    """
    scores = np.asarray(scores, dtype=np.float32)
    nseq = len(ctx_len)
    cu_keep = np.zeros(nseq + 1, dtype=np.int32)
    pieces = []
    off = 0
    for b in range(nseq):
        n = int(ctx_len[b])
        k = min(int(keep_len[b]), n)
        cu_keep[b + 1] = cu_keep[b] + k
        f = min(int(forced_first[b]) if forced_first is not None else 0, k)
        l = min(int(forced_last[b]) if forced_last is not None else 0, k - f)
        for h in range(n_kv_heads):
            s = scores[off:off + n]
            off += n
            forced = np.zeros(n, dtype=bool)
            forced[:f] = True
            forced[n - l:n] = l > 0
            free = np.flatnonzero(~forced)
            # stable sort of the negated scores: descending score, ascending position among equals
            order = free[np.argsort(-s[free].astype(np.float64), kind="stable")]
            chosen = np.concatenate([np.flatnonzero(forced), order[:k - f - l]])
            pieces.append(np.sort(chosen).astype(np.int32))
    keep = np.concatenate(pieces) if pieces else np.zeros(0, dtype=np.int32)
    return keep, cu_keep


# --------------------------------------------------------------------------------------------
# reload of the dropped rows only  (appendix B.1: a verify after token dropping needs only the
# extra (1 - c) * KV_full, the kept rows are already resident)
# --------------------------------------------------------------------------------------------
def pack_rows(k, v, idx, cu_idx, cu_ctx, n_kv_heads: int):
    """Rows named by the index lists, list after list: packed row (cu_idx[b]*Hkv + h*n_b + i) is
    row (cu_ctx[b] + idx_list(b, h)[i], h) of the pools [tokens, n_kv_heads, 128] (16-bit patterns).
    This is what the host keeps of a token-dropped sequence: its dropped rows only."""
    idx = np.asarray(idx, dtype=np.int64)
    nseq = len(cu_idx) - 1
    total = int(cu_idx[-1]) * n_kv_heads
    pk = np.zeros((total, k.shape[2]), dtype=k.dtype)
    pv = np.zeros((total, v.shape[2]), dtype=v.dtype)
    for b in range(nseq):
        n = int(cu_idx[b + 1]) - int(cu_idx[b])
        for h in range(n_kv_heads):
            start = int(cu_idx[b]) * n_kv_heads + h * n
            for i in range(n):
                row = int(cu_ctx[b]) + int(idx[start + i])
                pk[start + i] = k[row, h]
                pv[start + i] = v[row, h]
    return pk, pv


def swap_in_rows(packed_k, packed_v, dev_k, dev_v, dropped, cu_drop, cu_ctx, n_kv_heads: int, seqs):
    """The inverse placement for the sequences in `seqs`: packed row (cu_drop[b]*Hkv + h*nd + i)
    goes to row (cu_ctx[b] + dropped_list(b, h)[i], h) of the device pools.  Returns new
    (dev_k, dev_v); every other row is untouched."""
    dk, dv = np.array(dev_k, copy=True), np.array(dev_v, copy=True)
    dropped = np.asarray(dropped, dtype=np.int64)
    for b in seqs:
        nd = int(cu_drop[b + 1]) - int(cu_drop[b])
        for h in range(n_kv_heads):
            start = int(cu_drop[b]) * n_kv_heads + h * nd
            for i in range(nd):
                row = int(cu_ctx[b]) + int(dropped[start + i])
                dk[row, h] = packed_k[start + i]
                dv[row, h] = packed_v[start + i]
    return dk, dv
