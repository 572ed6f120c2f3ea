"""Pins of the fp64 oracle against what the mathematics fixes (closed forms, invariants, brute
force, hand-packed records).  CPU only.  Each test is chosen so that a plausible slip in the
oracle (dropped term, wrong sign or index, transposed operand, wrong GQA map, off-by-one in the
causal mask, wrong nibble order) fails it."""
import math

import numpy as np
import pytest
import torch

from oracle import vc_oracle as O
from tests import synth

D = 128


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float array -> bf16 bit patterns (round to nearest even) via torch."""
    t = torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def tbits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


# ------------------------------------------------------------------ widening
def test_bf16_and_f16_widening_exact():
    vals = np.array([0.0, 1.0, -2.5, 3.140625, 65280.0, 2.0 ** -20], dtype=np.float32)
    assert np.array_equal(O.bf16_to_f64(bf16_bits(vals)), vals.astype(np.float64))
    # known patterns: 0x3F80 = 1.0, 0xC020 = -2.5 (bf16); 0x3C00 = 1.0, 0x3555 ~ 1/3 (fp16)
    assert O.bf16_to_f64(np.array([0x3F80, 0xC020], dtype=np.uint16)).tolist() == [1.0, -2.5]
    h = O.f16_to_f64(np.array([0x3C00, 0x3555, 0xC400], dtype=np.uint16))
    assert h[0] == 1.0 and abs(h[1] - 1 / 3) < 2.5e-4 and h[2] == -4.0


# ------------------------------------------------------------------ softmax / attention
def test_softmax_rows_sum_to_one_and_shift_invariance():
    q, k, v = rnd(1, D), rnd(2, 50, D), rnd(3, 50, D)
    o, lse, p = O.attend(q, k, v, 0.3)
    assert abs(p.sum() - 1.0) <= 1e-12
    # adding c*q/|q|^2/scale to every key adds the constant c to every score
    c = 7.5
    k2 = k + (c / 0.3) * q / (q @ q)
    o2, lse2, p2 = O.attend(q, k2, v, 0.3)
    assert np.allclose(p, p2, atol=1e-12) and np.allclose(o, o2, atol=1e-11)
    assert abs((lse2 - lse) - c) < 1e-9


def test_two_key_closed_form():
    # scores (0, ln 3) -> p = (1/4, 3/4); lse = ln 4
    q = np.zeros(D); q[5] = 2.0
    k = np.zeros((2, D)); k[1, 5] = math.log(3.0)       # scale 0.5 * 2 * ln3 = ln3
    v = rnd(4, 2, D)
    o, lse, p = O.attend(q, k, v, 0.5)
    assert np.allclose(p, [0.25, 0.75], atol=1e-15)
    assert np.allclose(o, 0.25 * v[0] + 0.75 * v[1], atol=1e-14)
    assert abs(lse - math.log(4.0)) < 1e-14


def test_uniform_keys_give_mean_of_values():
    q = rnd(5, D)
    k = np.tile(rnd(6, 1, D), (37, 1))
    v = rnd(7, 37, D)
    o, lse, _ = O.attend(q, k, v, 1 / math.sqrt(D))
    assert np.allclose(o, v.mean(axis=0), atol=1e-13)


def test_dominant_key_returns_its_value_row():
    q = rnd(8, D)
    k = np.zeros((20, D)); k[13] = 50.0 * q / (q @ q)    # score 50 against 0
    v = rnd(9, 20, D)
    o, _, _ = O.attend(q, k, v, 1.0)
    assert np.allclose(o, v[13], atol=1e-12 * 20 * 10 + 20 * math.exp(-50) * 10)


def test_transposed_operand_would_fail():
    # scores must come from K (not V) and the output from V (not K)
    q = rnd(10, D); k = rnd(11, 9, D); v = rnd(12, 9, D)
    o, _, p = O.attend(q, k, v, 0.2)
    s = np.array([0.2 * sum(q[d] * k[j, d] for d in range(D)) for j in range(9)])
    e = np.exp(s - s.max()); pp = e / e.sum()
    assert np.allclose(p, pp, atol=1e-14)
    assert np.allclose(o, sum(pp[j] * v[j] for j in range(9)), atol=1e-13)


def brute_attention(q, keys, vals, scale):
    """Second, differently written routine: Python loops, math.exp, no max subtraction trick
    beyond a plain two-pass softmax."""
    n = len(keys)
    s = [scale * sum(q[d] * keys[j][d] for d in range(len(q))) for j in range(n)]
    mx = max(s)
    e = [math.exp(x - mx) for x in s]
    tot = sum(e)
    out = [sum(e[j] * vals[j][d] for j in range(n)) / tot for d in range(len(q))]
    return out, mx + math.log(tot)


def small_layer(seed=3, **kw):
    base = dict(ctx_len=[7, 5], n_q_heads=4, n_kv_heads=2)
    base.update(kw)
    return synth.make_layer(seed, "cpu", **base)


def test_draft_brute_force_gqa_and_gather():
    lay = small_layer(keep=[3, 2], keep_first=1, keep_last=1, tail_len=[2, 0])
    out, lse = O.draft_attn(tbits(lay.q), lay.scale, n_q_heads=4, n_kv_heads=2,
                            pool_k=tbits(lay.k_full), pool_v=tbits(lay.v_full),
                            cu_ctx=lay.cu_ctx.numpy(), keep_idx=lay.keep_idx.numpy(),
                            cu_keep=lay.cu_keep.numpy(), tail_k=tbits(lay.tail_k),
                            tail_v=tbits(lay.tail_v), cu_tail=lay.cu_tail.numpy())
    kf, vf = lay.k_full.double().numpy(), lay.v_full.double().numpy()
    tk, tv = lay.tail_k.double().numpy(), lay.tail_v.double().numpy()
    qf = lay.q.double().numpy()
    keep = lay.keep_idx.numpy()
    cu, cuk, cut = lay.cu_ctx.tolist(), lay.cu_keep.tolist(), lay.cu_tail.tolist()
    for b in range(2):
        nk = cuk[b + 1] - cuk[b]
        for h in range(4):
            kvh = h // 2
            pos = [cu[b] + int(keep[cuk[b] * 2 + kvh * nk + i]) for i in range(nk)]
            keys = [kf[p, kvh] for p in pos] + [tk[t, kvh] for t in range(cut[b], cut[b + 1])]
            vals = [vf[p, kvh] for p in pos] + [tv[t, kvh] for t in range(cut[b], cut[b + 1])]
            ref, ref_lse = brute_attention(qf[b, h], keys, vals, lay.scale)
            assert np.allclose(out[b, h], ref, atol=1e-12)
            assert abs(lse[b, h] - ref_lse) < 1e-12


def test_verify_brute_force_causal():
    lay = small_layer(win=[3, 2])
    out, lse = O.verify_attn(tbits(lay.q_win), tbits(lay.k_full), tbits(lay.v_full),
                             tbits(lay.k_win), tbits(lay.v_win), lay.cu_ctx.numpy(),
                             lay.cu_win.numpy(), lay.scale, n_q_heads=4, n_kv_heads=2)
    kf, vf = lay.k_full.double().numpy(), lay.v_full.double().numpy()
    kw, vw = lay.k_win.double().numpy(), lay.v_win.double().numpy()
    qw = lay.q_win.double().numpy()
    cu, cw = lay.cu_ctx.tolist(), lay.cu_win.tolist()
    for b in range(2):
        for i in range(cw[b + 1] - cw[b]):
            for h in range(4):
                kvh = h // 2
                keys = [kf[t, kvh] for t in range(cu[b], cu[b + 1])] + [kw[cw[b] + r, kvh] for r in range(i + 1)]
                vals = [vf[t, kvh] for t in range(cu[b], cu[b + 1])] + [vw[cw[b] + r, kvh] for r in range(i + 1)]
                ref, ref_lse = brute_attention(qw[cw[b] + i, h], keys, vals, lay.scale)
                assert np.allclose(out[cw[b] + i, h], ref, atol=1e-12)
                assert abs(lse[cw[b] + i, h] - ref_lse) < 1e-12


def test_verify_rows_do_not_see_later_rows_and_see_themselves():
    lay = small_layer(win=[4, 1])
    args = lambda kw, vw: (tbits(lay.q_win), tbits(lay.k_full), tbits(lay.v_full), tbits(kw), tbits(vw),
                           lay.cu_ctx.numpy(), lay.cu_win.numpy(), lay.scale)
    base, _ = O.verify_attn(*args(lay.k_win, lay.v_win), n_q_heads=4, n_kv_heads=2)
    k2, v2 = lay.k_win.clone(), lay.v_win.clone()
    k2[2:4] += 3.0; v2[2:4] -= 5.0                      # rows 2, 3 of sequence 0
    pert, _ = O.verify_attn(*args(k2, v2), n_q_heads=4, n_kv_heads=2)
    assert np.array_equal(base[0:2], pert[0:2])          # rows 0, 1 bit-identical
    assert not np.allclose(base[2], pert[2])             # row 2 sees its own position
    assert np.array_equal(base[4], pert[4])              # other sequence untouched


def test_verify_uniform_keys_mean_over_n_plus_i_plus_one():
    lay = small_layer(win=[3, 2])
    kf = lay.k_full.clone(); kw = lay.k_win.clone()
    kf[:] = kf[0, 0]; kw[:] = kf[0, 0]
    out, _ = O.verify_attn(tbits(lay.q_win), tbits(kf), tbits(lay.v_full), tbits(kw), tbits(lay.v_win),
                           lay.cu_ctx.numpy(), lay.cu_win.numpy(), lay.scale, n_q_heads=4, n_kv_heads=2)
    vf, vw = lay.v_full.double().numpy(), lay.v_win.double().numpy()
    for i in range(3):
        for h in range(4):
            rows = np.concatenate([vf[0:7, h // 2], vw[0:i + 1, h // 2]])
            assert rows.shape[0] == 7 + i + 1
            assert np.allclose(out[i, h], rows.mean(axis=0), atol=1e-13)


def test_verify_window_of_one_equals_decode_over_full_plus_self():
    lay = small_layer(win=[1, 1])
    out, lse = O.verify_attn(tbits(lay.q_win), tbits(lay.k_full), tbits(lay.v_full), tbits(lay.k_win),
                             tbits(lay.v_win), lay.cu_ctx.numpy(), lay.cu_win.numpy(), lay.scale,
                             n_q_heads=4, n_kv_heads=2)
    d_out, d_lse = O.draft_attn(tbits(lay.q_win), lay.scale, n_q_heads=4, n_kv_heads=2,
                                pool_k=tbits(lay.k_full), pool_v=tbits(lay.v_full), cu_ctx=lay.cu_ctx.numpy(),
                                tail_k=tbits(lay.k_win), tail_v=tbits(lay.v_win), cu_tail=lay.cu_win.numpy())
    assert np.allclose(out, d_out, atol=1e-13) and np.allclose(lse, d_lse, atol=1e-13)


def test_split_merge_invariance():
    q, k, v = rnd(20, D), rnd(21, 60, D), rnd(22, 60, D)
    o, lse, _ = O.attend(q, k, v, 0.09)
    oa, la, _ = O.attend(q, k[:23], v[:23], 0.09)
    ob, lb, _ = O.attend(q, k[23:], v[23:], 0.09)
    m = max(la, lb)
    wa, wb = math.exp(la - m), math.exp(lb - m)
    assert np.allclose(o, (wa * oa + wb * ob) / (wa + wb), atol=1e-13)
    assert abs(lse - (m + math.log(wa + wb))) < 1e-13


def test_permutation_invariance_and_zero_dropping():
    lay = small_layer(ctx_len=[40], keep=[40], keep_first=0, keep_last=0)
    assert lay.keep_idx.view(2, 40).tolist() == [list(range(40))] * 2
    kw = dict(n_q_heads=4, n_kv_heads=2, pool_k=tbits(lay.k_full), pool_v=tbits(lay.v_full),
              cu_ctx=lay.cu_ctx.numpy())
    full, _ = O.draft_attn(tbits(lay.q), lay.scale, **kw)
    kept, _ = O.draft_attn(tbits(lay.q), lay.scale, keep_idx=lay.keep_idx.numpy(),
                           cu_keep=lay.cu_keep.numpy(), **kw)
    assert np.allclose(full, kept, atol=1e-14)
    perm = np.random.default_rng(0).permutation(40).astype(np.int32)
    shuffled, _ = O.draft_attn(tbits(lay.q), lay.scale, keep_idx=np.concatenate([perm, perm[::-1]]),
                               cu_keep=lay.cu_keep.numpy(), **kw)
    assert np.allclose(full, shuffled, atol=1e-13)


def test_dropping_tokens_with_vanishing_weight_changes_nothing():
    lay = small_layer(ctx_len=[30], n_q_heads=2, n_kv_heads=1, keep=[20], keep_first=2, keep_last=2)
    keep = lay.keep_idx.numpy()
    kf = lay.k_full.clone().float()
    q = lay.q.float()
    dropped = sorted(set(range(30)) - set(keep.tolist()))
    for t in dropped:                                    # score about -1e4 / sqrt(128) * |q|... make it huge
        kf[t, 0] = -200.0 * q[0, 0] / (q[0, 0] @ q[0, 0]) * math.sqrt(D)
    kfb = kf.to(torch.bfloat16)
    kw = dict(n_q_heads=2, n_kv_heads=1, pool_k=tbits(kfb), pool_v=tbits(lay.v_full), cu_ctx=lay.cu_ctx.numpy())
    full, _ = O.draft_attn(tbits(lay.q)[:, :1], lay.scale, **dict(kw, n_q_heads=1))
    kept, _ = O.draft_attn(tbits(lay.q)[:, :1], lay.scale, keep_idx=keep, cu_keep=lay.cu_keep.numpy(),
                           **dict(kw, n_q_heads=1))
    assert np.allclose(full, kept, atol=1e-12)


def test_gqa_head_mapping():
    lay = small_layer(ctx_len=[16], n_q_heads=8, n_kv_heads=2)
    q = lay.q.clone(); q[0, :] = q[0, 0]                 # identical queries
    kw = dict(n_q_heads=8, n_kv_heads=2, pool_k=tbits(lay.k_full), pool_v=tbits(lay.v_full),
              cu_ctx=lay.cu_ctx.numpy())
    out, _ = O.draft_attn(tbits(q), lay.scale, **kw)
    for h in (1, 2, 3):
        assert np.array_equal(out[0, 0], out[0, h])
    for h in (5, 6, 7):
        assert np.array_equal(out[0, 4], out[0, h])
    assert not np.allclose(out[0, 0], out[0, 4])
    v2 = lay.v_full.clone(); v2[:, 1] *= 2.0             # change KV head 1 only (exact in bf16)
    out2, _ = O.draft_attn(tbits(q), lay.scale, **dict(kw, pool_v=tbits(v2)))
    assert np.array_equal(out[0, :4], out2[0, :4]) and np.allclose(out2[0, 4:], out[0, 4:] * 2.0, atol=1e-12)


# ------------------------------------------------------------------ block records
def hand_pack_record(bits, kcode, vcode, kscale, kzero, vscale, vzero):
    """Write one record byte by byte from the layout prose of the header (independent of both the
    generator's vectorised packer and the oracle's unpacker).  kcode/vcode [TB][128] ints."""
    tb = 32 if bits == 4 else 64
    rec = bytearray(5120)
    per_word = 32 // bits
    mask = (1 << bits) - 1

    def put(word_byte_offset, e, code):
        bit = 16 * (e % 2) + bits * (e // 2)               # even elements low half-word, odd high
        rec[word_byte_offset + bit // 8] |= (code & mask) << (bit % 8)

    for t in range(tb):
        for d in range(128):
            put(4 * ((128 // per_word) * t + d // per_word), d % per_word, kcode[t][d])
    for t in range(tb):
        for d in range(128):
            c, rem = divmod(d, 64)
            q, n = divmod(rem, 16)
            j, e = divmod(t, per_word)
            slot = 64 * c + 16 * j + n
            put(2048 + 16 * slot + 4 * q, e, vcode[t][d])
    f16 = lambda x: int(np.array([x], dtype=np.float16).view(np.uint16)[0])
    for d in range(128):
        s, z = f16(kscale[d]), f16(kzero[d])
        rec[4096 + 2 * d] = s & 0xFF; rec[4097 + 2 * d] = s >> 8
        rec[4352 + 2 * d] = z & 0xFF; rec[4353 + 2 * d] = z >> 8
    for g in range(128 // tb):
        for t in range(tb):
            s, z = f16(vscale[g][t]), f16(vzero[g][t])
            o = 4608 + 2 * (g * tb + t)
            rec[o] = s & 0xFF; rec[o + 1] = s >> 8
            rec[o + 256] = z & 0xFF; rec[o + 257] = z >> 8
    return np.frombuffer(bytes(rec), dtype=np.uint8)


@pytest.mark.parametrize("bits", [4, 2])
def test_unpack_hand_packed_record(bits):
    tb = 32 if bits == 4 else 64
    rng = np.random.default_rng(bits)
    kc = rng.integers(0, 1 << bits, (tb, 128))
    vc = rng.integers(0, 1 << bits, (tb, 128))
    ks = np.float16(rng.uniform(0.1, 1.0, 128)); kz = np.float16(rng.uniform(-3, 0, 128))
    vs = np.float16(rng.uniform(0.1, 1.0, (128 // tb, tb))); vz = np.float16(rng.uniform(-3, 0, (128 // tb, tb)))
    rec = hand_pack_record(bits, kc.tolist(), vc.tolist(), ks, kz, vs, vz)
    kh, vh = O.unpack_records(rec.reshape(1, 1, 5120), bits)
    k_ref = ks.astype(np.float64)[None, :] * kc + kz.astype(np.float64)[None, :]
    v_ref = np.empty((tb, 128))
    for t in range(tb):
        for d in range(128):
            v_ref[t, d] = float(vs[d // tb, t]) * vc[t, d] + float(vz[d // tb, t])
    assert np.array_equal(kh[0], k_ref)
    assert np.array_equal(vh[0], v_ref)


@pytest.mark.parametrize("bits", [4, 2])
def test_generator_packer_matches_hand_packer(bits):
    # the input generator's vectorised packer must write the same bytes as the hand packer
    tb = synth.tokens_per_block(bits)
    g = synth.gen(11, "cpu")
    k = synth.randn_bf16((tb, 1, 128), g); v = synth.randn_bf16((tb, 1, 128), g)
    rec = synth.quantize_records(k, v, bits)[0, 0].numpy()
    kh, vh = O.unpack_records(rec.reshape(1, 1, 5120), bits)
    # recover codes through the oracle and re-pack by hand
    meta = rec[4096:].view(np.uint16)
    ks, kz = meta[0:128].view(np.float16), meta[128:256].view(np.float16)
    vs, vz = meta[256:384].view(np.float16).reshape(128 // tb, tb), meta[384:512].view(np.float16).reshape(128 // tb, tb)
    kc = np.rint((kh[0] - kz.astype(np.float64)) / np.where(ks > 0, ks, 1).astype(np.float64)).astype(int)
    vc = np.empty((tb, 128), dtype=int)
    for t in range(tb):
        for d in range(128):
            s = float(vs[d // tb, t])
            vc[t, d] = int(round((vh[0][t, d] - float(vz[d // tb, t])) / (s if s > 0 else 1.0)))
    rec2 = hand_pack_record(bits, kc.tolist(), vc.tolist(), ks, kz, vs, vz)
    assert np.array_equal(rec, rec2)


@pytest.mark.parametrize("bits", [4, 2])
def test_quantisation_error_bound_and_constant_group(bits):
    tb = synth.tokens_per_block(bits)
    g = synth.gen(5, "cpu")
    k = synth.randn_bf16((3 * tb, 2, 128), g); v = synth.randn_bf16((3 * tb, 2, 128), g)
    k[0:tb, 0, 7] = 1.5                                   # a constant key group -> exact
    rec = synth.quantize_records(k, v, bits).numpy()
    kh, vh = O.unpack_records(rec, bits)
    kd = k.double().numpy().transpose(1, 0, 2); vd = v.double().numpy().transpose(1, 0, 2)
    meta = rec[:, :, 4096:].copy().view(np.uint16)
    ks = O.f16_to_f64(meta[:, :, 0:128])                  # [H, nb, 128]
    kerr = np.abs(kh - kd).reshape(2, 3, tb, 128)
    # |x_hat - x| <= scale/2 plus fp16 rounding of zero (half ulp of |min| <= 8 -> 2^-8) and of scale*code
    assert (kerr <= ks[:, :, None, :] / 2 + 2.0 ** -8 + 2.0 ** -11 * ks[:, :, None, :] * (1 << bits)).all()
    assert np.array_equal(kh[0, 0:tb, 7], np.full(tb, 1.5))
    vs = O.f16_to_f64(meta[:, :, 256:384]).reshape(2, 3, 128 // tb, tb)
    verr = np.abs(vh - vd).reshape(2, 3, tb, 128 // tb, tb)
    bound = vs.transpose(0, 1, 3, 2)[..., None] / 2 + 2.0 ** -8 + 2.0 ** -11 * vs.transpose(0, 1, 3, 2)[..., None] * (1 << bits)
    assert (verr <= bound).all()


@pytest.mark.parametrize("bits", [4, 2])
def test_lossless_grid_quantised_draft_equals_bf16_draft(bits):
    """Groups built from grid values zero + j/8 (j = 0..2^b-1, both ends present) survive
    quantise -> dequantise exactly, so attention over the records equals attention over bf16."""
    tb = synth.tokens_per_block(bits)
    lv = 1 << bits
    rng = np.random.default_rng(bits + 40)
    n_tok, hkv = 2 * tb, 2
    k = np.empty((n_tok, hkv, 128)); v = np.empty((n_tok, hkv, 128))
    for h in range(hkv):
        for blk in range(2):
            for d in range(128):                          # key groups: one channel, tb tokens
                z = rng.integers(-16, 16) / 4.0
                j = rng.integers(0, lv, tb); j[0], j[1] = 0, lv - 1
                k[blk * tb:(blk + 1) * tb, h, d] = z + rng.permutation(j) / 8.0
            for t in range(tb):                           # value groups: one token, tb channels
                for gidx in range(128 // tb):
                    z = rng.integers(-16, 16) / 4.0
                    j = rng.integers(0, lv, tb); j[0], j[1] = 0, lv - 1
                    v[blk * tb + t, h, gidx * tb:(gidx + 1) * tb] = z + rng.permutation(j) / 8.0
    kt = torch.from_numpy(k).to(torch.bfloat16); vt = torch.from_numpy(v).to(torch.bfloat16)
    assert np.array_equal(kt.double().numpy(), k) and np.array_equal(vt.double().numpy(), v)
    rec = synth.quantize_records(kt, vt, bits)
    kh, vh = O.unpack_records(rec.numpy(), bits)
    assert np.array_equal(kh, k.transpose(1, 0, 2)) and np.array_equal(vh, v.transpose(1, 0, 2))
    q = synth.randn_bf16((1, 4, 128), synth.gen(2, "cpu"))
    cu = np.array([0, n_tok], dtype=np.int32)
    a, la = O.draft_attn(tbits(q), 0.1, n_q_heads=4, n_kv_heads=2, pool_k=tbits(kt), pool_v=tbits(vt), cu_ctx=cu)
    b, lb = O.draft_attn(tbits(q), 0.1, n_q_heads=4, n_kv_heads=2, bits=bits,
                         blocks=rec.reshape(-1, 5120).numpy(), cu_blk=np.array([0, 2], dtype=np.int32))
    assert np.allclose(a, b, atol=1e-13) and np.allclose(la, lb, atol=1e-13)


def test_record_ownership_over_sequences_and_heads():
    # sequence 1, head 1 must read records cu_blk[1]*Hkv + 1*nb ... (wrong stride would mix heads)
    lay = synth.make_layer(9, "cpu", ctx_len=[64, 96], n_q_heads=4, n_kv_heads=2, quant_bits=(4,))
    rec = lay.blocks[4].numpy()
    cu = lay.cu_blk[4].numpy()
    assert cu.tolist() == [0, 2, 5]
    k, v = O.draft_keys(1, 1, n_kv_heads=2, blocks=rec, cu_blk=cu, bits=4)
    ref = lay.k_full[64:160, 1].double().numpy()
    assert k.shape == (96, 128) and np.abs(k - ref).max() < 0.6       # int4 of N(0,1): step ~0.4
    wrong = lay.k_full[64:160, 0].double().numpy()
    assert np.abs(k - wrong).max() > 1.5


# ------------------------------------------------------------------ accept
def test_accept_planted_prefix_and_token_count():
    lay = synth.make_layer(4, "cpu", ctx_len=[8, 8, 8, 8], n_q_heads=4, n_kv_heads=2, win=[5, 5, 3, 1],
                           vocab=997, prefix_len=[0, 5, 2, 1])
    a, nxt, amax = O.accept(lay.logits.numpy(), lay.cu_rows.numpy(), lay.draft_ids.numpy(), lay.cu_win.numpy())
    assert amax.tolist() == lay.ids_star.tolist()          # planted 10.0 beats N(0,1) by construction
    assert a.tolist() == [0, 5, 2, 1]
    ids = lay.ids_star.tolist(); cr = lay.cu_rows.tolist()
    assert nxt.tolist() == [ids[cr[0] + 0], -1, ids[cr[2] + 2], -1]   # no bonus rows supplied
    for b in range(4):                                      # 1 .. x+1 tokens per round (with a bonus row)
        assert 0 <= a[b] <= lay.win[b]


def test_accept_bonus_row_and_ties_and_neg_inf():
    v = 6
    logits = np.full((5, v), -np.inf, dtype=np.float32)
    logits[0, [2, 4]] = 1.0                                 # tie -> lowest index 2
    logits[1, 5] = -3.0                                     # only finite entry
    logits[2, :] = 0.5                                      # all equal -> 0
    logits[3, 3] = 2.0; logits[3, 1] = 2.0                  # tie -> 1
    logits[4, 0] = -1.0; logits[4, 4] = 7.0
    cu_rows = np.array([0, 3, 5]); cu_win = np.array([0, 2, 4])      # seq0: w=2 + bonus; seq1: w=2, no bonus
    draft = np.array([2, 5, 1, 4], dtype=np.int32)
    a, nxt, amax = O.accept(logits, cu_rows, draft, cu_win)
    assert amax.tolist() == [2, 5, 0, 1, 4]
    assert a.tolist() == [2, 2] and nxt.tolist() == [0, -1]          # seq0 all matched -> bonus row argmax
    draft2 = np.array([4, 5, 1, 0], dtype=np.int32)                   # seq0 mismatch at 0 (tie resolved to 2)
    a, nxt, _ = O.accept(logits, cu_rows, draft2, cu_win)
    assert a.tolist() == [0, 1] and nxt.tolist() == [2, 4]


def test_argmax_signed_zero_tie_goes_to_the_lower_index():
    """-0.0 and +0.0 are the same logit value: the tie rule (lowest index) applies between them in
    either order (section 4.1 step 3 compares token ids, so the arg-max must be unique)."""
    row = np.full(20000, -1.0, dtype=np.float32)
    row[3] = -0.0; row[15000] = 0.0
    assert O.argmax_row(row) == 3
    row[3] = 0.0; row[15000] = -0.0
    assert O.argmax_row(row) == 3
    row[:] = -0.0; row[19999] = 0.0
    assert O.argmax_row(row) == 0


def test_accept_brute_force_tiny_vocab():
    rng = np.random.default_rng(3)
    for trial in range(30):
        w = [int(x) for x in rng.integers(0, 5, 3)]
        bonus = [int(x) for x in rng.integers(0, 2, 3)]
        rows = [w[b] + bonus[b] for b in range(3)]
        cu_rows = np.concatenate([[0], np.cumsum(rows)]); cu_win = np.concatenate([[0], np.cumsum(w)])
        logits = rng.integers(0, 3, (max(1, sum(rows)), 4)).astype(np.float32)[:sum(rows)]
        draft = rng.integers(0, 4, sum(w)).astype(np.int32)
        a, nxt, _ = O.accept(logits.reshape(sum(rows), 4), cu_rows, draft, cu_win)
        for b in range(3):
            am = []
            for r in range(cu_rows[b], cu_rows[b + 1]):
                best, bi = -1e30, -1
                for x in range(4):
                    if logits[r, x] > best:
                        best, bi = logits[r, x], x
                am.append(bi)
            j = 0
            while j < w[b] and draft[cu_win[b] + j] == am[j]:
                j += 1
            assert a[b] == j
            assert nxt[b] == (am[j] if j < rows[b] else -1)


# ------------------------------------------------------------------ kept index
def test_keep_from_dropped_brute_force():
    lay = synth.make_layer(6, "cpu", ctx_len=[50, 33, 20], n_q_heads=4, n_kv_heads=2, keep=[10, 33, 0],
                           keep_first=2, keep_last=3)
    keep, cu_keep = O.keep_from_dropped(lay.dropped_idx.numpy(), lay.cu_drop.numpy(), lay.ctx_len, 2)
    # sequence 2 keeps nothing in the generator (count 0 means "not token-dropped"): its dropped list is empty,
    # so the complement is everything
    assert cu_keep.tolist() == [0, 10, 43, 63]
    drop = lay.dropped_idx.numpy(); cud = lay.cu_drop.tolist()
    for b, n in enumerate([50, 33, 20]):
        nd = cud[b + 1] - cud[b]; nk = n - nd
        for h in range(2):
            gone = set(drop[cud[b] * 2 + h * nd: cud[b] * 2 + (h + 1) * nd].tolist())
            ref = [p for p in range(n) if p not in gone]
            got = keep[cu_keep[b] * 2 + h * nk: cu_keep[b] * 2 + (h + 1) * nk].tolist()
            assert got == ref and len(got) + len(gone) == n
    assert np.array_equal(keep[:cu_keep[2] * 2], lay.keep_idx.numpy()[:cu_keep[2] * 2])


def test_topk_keep_rule():
    kp = synth.topk_keep(1000, 100, 8, 16, 3, synth.gen(1, "cpu"))
    assert kp.shape == (3, 100)
    for row in kp.tolist():
        assert row == sorted(set(row)) and row[:8] == list(range(8)) and row[-16:] == list(range(984, 1000))
