"""CPU pins of the oracle's compressor-side functions (section 6 of the paper: compress /
decompress for quantising methods, kept positions chosen from scores): hand-computed records,
closed forms, invariants, brute force, and a second independently written routine."""
import numpy as np
import pytest
import torch

from oracle import vc_oracle as O
from tests import synth
from tests.test_oracle_pins import hand_pack_record


def b16(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def bf16_bits_of(x) -> np.ndarray:
    """bf16-representable floats -> bit patterns."""
    return b16(torch.tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16))


# ------------------------------------------------------------------ quantiser
def test_quantise_groups_hand_values_and_ties():
    # min 0, max 15 -> zero 0, scale 1: codes are the values; 0.5 and 2.5 are ties -> even (0, 2)
    x = np.array([[0, 0.5, 1.5, 2.5, 3.0, 15.0, 7.25, 7.75]], dtype=np.float32)
    code, scale, zero = O.quantise_groups(x, 15)
    assert float(scale[0]) == 1.0 and float(zero[0]) == 0.0
    assert code[0].tolist() == [0, 0, 2, 2, 3, 15, 7, 8]
    # offset and step: zero -2, step 0.25 over 4 levels
    y = np.array([[-2.0, -1.75, -1.5, -1.25]], dtype=np.float32)
    code, scale, zero = O.quantise_groups(y, 3)
    assert float(scale[0]) == 0.25 and float(zero[0]) == -2.0 and code[0].tolist() == [0, 1, 2, 3]
    # constant group: scale 0, codes 0, zero carries the value
    code, scale, zero = O.quantise_groups(np.full((1, 8), 1.5, dtype=np.float32), 15)
    assert float(scale[0]) == 0.0 and float(zero[0]) == 1.5 and not code.any()


def test_quantise_groups_uses_stored_fp16_values():
    # min = 0.1 is not an fp16 value: zero is fp16(0.1) and the codes come from that stored zero
    x = np.array([[0.1, 0.1 + 15 * 0.3, 1.0]], dtype=np.float32)
    code, scale, zero = O.quantise_groups(x, 15)
    assert zero[0] == np.float16(np.float32(0.1))
    assert scale[0] == np.float16((x[0, 1] - x[0, 0]) / np.float32(15))
    z, s = float(zero[0]), float(scale[0])
    assert code[0].tolist() == [0, 15, int(np.rint((1.0 - z) / s))]


def test_quantise_groups_stores_negative_zero_minimum_as_positive_zero():
    """Reading of the quantiser (the paper names only the axes, section 2 and section 6): a group whose
    minimum is -0.0 stores the zero point +0.0 (fp16 bits 0x0000, never 0x8000).  The two zeros compare
    equal, so a minimum taken in any order may come out as either; adding +0.0 makes the stored byte
    unique.  Dequantised values are unaffected: scale * code + (-0.0) and scale * code + 0.0 are the
    same number for every code."""
    neg0 = np.float32(-0.0)
    # -0.0 alone as the minimum; -0.0 before +0.0; +0.0 before -0.0
    for grp in ([neg0, 1.0, 2.0, 3.0], [neg0, 0.0, 1.5, 3.0], [0.0, neg0, 1.5, 3.0]):
        code, scale, zero = O.quantise_groups(np.array([grp], dtype=np.float32), 3)
        assert zero.view(np.uint16)[0] == 0x0000
        assert float(scale[0]) == 1.0 and code[0, 0] == 0 and code[0, -1] == 3
    # a constant group of -0.0: scale 0, zero +0, codes 0
    code, scale, zero = O.quantise_groups(np.full((1, 8), neg0, dtype=np.float32), 15)
    assert zero.view(np.uint16)[0] == 0x0000 and scale.view(np.uint16)[0] == 0x0000 and not code.any()


@pytest.mark.parametrize("bits", [4, 2])
def test_quantize_records_negative_zero_minimum_bytes(bits):
    """The same rule in the record: a key group (one channel over the block's tokens) and a value
    group (one token over TB channels) whose minimum is -0.0 store zero-point bytes 00 00."""
    tb = O.tokens_per_block(bits)
    levels = (1 << bits) - 1
    k = np.ones((tb, 1, 128), dtype=np.float32)
    v = np.ones((tb, 1, 128), dtype=np.float32)
    k[:, 0, 9] = np.arange(tb) % (levels + 1)          # channel 9: values 0..levels, minimum stored as -0.0
    k[0, 0, 9] = -0.0
    v[5, 0, tb:2 * tb] = np.arange(tb) % (levels + 1) if 2 * tb <= 128 else 0
    v[5, 0, 0:tb] = np.arange(tb) % (levels + 1)       # token 5, channel group 0
    v[5, 0, 0] = -0.0
    kb, vb = bf16_bits_of(k), bf16_bits_of(v)
    assert kb[0, 0, 9] == 0x8000 and vb[5, 0, 0] == 0x8000          # the inputs really are -0.0
    rec = O.quantize_records(kb, vb, bits)[0, 0]
    kzero = rec[4096 + 256:4096 + 512].view("<u2")                   # key zero[128]
    vzero = rec[4608 + 256:4608 + 512].view("<u2")                   # value zero[g][t]
    assert kzero[9] == 0x0000 and vzero[0 * tb + 5] == 0x0000
    kscale = rec[4096:4096 + 256].view("<u2").view(np.float16)
    assert float(kscale[9]) == 1.0


@pytest.mark.parametrize("bits", [4, 2])
def test_quantize_records_equals_hand_packed_closed_form(bits):
    """Keys: channel d of token t holds zero_d + step_d * ((t + d) mod L1); values: token t, channel
    d holds zero_t + step_g * ((t + d) mod L1) - every group spans 0..levels, so the codes, scales and
    zero points are known in closed form, and the record must equal the hand-packed bytes."""
    tb = O.tokens_per_block(bits)
    levels = (1 << bits) - 1
    t = np.arange(tb)[:, None]
    d = np.arange(128)[None, :]
    kcode = (t + d) % (levels + 1)
    kstep = 2.0 ** -(1 + d % 3)                       # per channel
    kzero = -1.0 - (d % 5) * 0.25
    k = kzero + kstep * kcode
    vcode = (3 * t + d) % (levels + 1)
    g = d // tb
    vstep = 2.0 ** -(1 + (t + g) % 3)                 # per (token, channel group)
    vzero = 0.5 * ((t + 2 * g) % 4) - 1.0
    v = vzero + vstep * vcode
    rec = O.quantize_records(bf16_bits_of(k)[:, None, :], bf16_bits_of(v)[:, None, :], bits)
    vs = np.array([[2.0 ** -(1 + (tt + gg) % 3) * 1.0 for tt in range(tb)] for gg in range(128 // tb)])
    vz = np.array([[0.5 * ((tt + 2 * gg) % 4) - 1.0 for tt in range(tb)] for gg in range(128 // tb)])
    hand = hand_pack_record(bits, kcode.tolist(), vcode.tolist(), kstep[0], kzero[0], vs, vz)
    assert np.array_equal(rec[0, 0], hand)


@pytest.mark.parametrize("bits", [4, 2])
def test_quantize_records_bounds_extremes_and_second_routine(bits):
    tb = O.tokens_per_block(bits)
    levels = (1 << bits) - 1
    gen = synth.gen(21, "cpu")
    k = synth.randn_bf16((3 * tb + 5, 2, 128), gen)     # 5 leftover tokens are not compressed
    v = synth.randn_bf16((3 * tb + 5, 2, 128), gen)
    k[:, 0, 3] *= 10.0                                   # an outlier channel
    rec = O.quantize_records(b16(k), b16(v), bits)
    assert rec.shape == (2, 3, 5120)
    # the input generator's packer is written differently (torch, vectorised): same bytes
    assert np.array_equal(rec, synth.quantize_records(k[:3 * tb], v[:3 * tb], bits).numpy())
    kh, vh = O.unpack_records(rec, bits)
    kd = k[:3 * tb].double().numpy().transpose(1, 0, 2)
    vd = v[:3 * tb].double().numpy().transpose(1, 0, 2)
    meta = rec[:, :, 4096:].copy().view(np.uint16)
    ks = O.f16_to_f64(meta[:, :, 0:128])[:, :, None, :]
    kz = O.f16_to_f64(meta[:, :, 128:256])[:, :, None, :]
    # |x_hat - x| <= scale/2 + what fp16 rounding of zero and scale can add
    kerr = np.abs(kh - kd).reshape(2, 3, tb, 128)
    assert (kerr <= ks / 2 + 2.0 ** -11 * np.abs(kz) + 2.0 ** -11 * ks * levels + 1e-12).all()
    vs = O.f16_to_f64(meta[:, :, 256:384]).reshape(2, 3, 128 // tb, tb).transpose(0, 1, 3, 2)[..., None]
    vz = O.f16_to_f64(meta[:, :, 384:512]).reshape(2, 3, 128 // tb, tb).transpose(0, 1, 3, 2)[..., None]
    verr = np.abs(vh - vd).reshape(2, 3, tb, 128 // tb, tb)
    assert (verr <= vs / 2 + 2.0 ** -11 * np.abs(vz) + 2.0 ** -11 * vs * levels + 1e-12).all()
    # the minimum of every group has code 0 and the maximum code `levels`
    kcode = np.rint((kh.reshape(2, 3, tb, 128) - kz) / ks)
    assert (kcode.min(axis=2) == 0).all() and (kcode.max(axis=2) == levels).all()
    vcode = np.rint((vh.reshape(2, 3, tb, 128 // tb, tb) - vz) / vs)
    assert (vcode.min(axis=4) == 0).all() and (vcode.max(axis=4) == levels).all()


def test_key_groups_run_over_tokens_and_value_groups_over_channels():
    """Swapping the two axes must fail: a key channel with a huge range inflates only that
    channel's scale; a value token with a huge range inflates only that token's scales."""
    tb = 32
    k = np.zeros((tb, 1, 128), dtype=np.float32); v = np.zeros((tb, 1, 128), dtype=np.float32)
    k[:, 0, :] = np.arange(tb)[:, None] % 2              # every channel spans 0..1
    k[5, 0, 9] = 150.0                                   # channel 9 spans 0..150
    v[:, 0, :] = np.arange(128)[None, :] % 2
    v[7, 0, 40] = 150.0                                  # token 7, channel group 1
    rec = O.quantize_records(bf16_bits_of(k), bf16_bits_of(v), 4)
    meta = rec[0, 0, 4096:].copy().view(np.uint16).view(np.float16).astype(np.float64)
    ks, vs = meta[0:128], meta[256:384].reshape(4, tb)
    assert ks[9] == 10.0 and (np.delete(ks, 9) == np.float16(1 / 15)).all()
    assert vs[1, 7] == 10.0 and (np.delete(vs.ravel(), 1 * tb + 7) == np.float16(1 / 15)).all()


# ------------------------------------------------------------------ decompress
def test_f64_to_bf16_single_rounding():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -30, -(1.0 + 2.0 ** -8 + 2.0 ** -40),
                  0.0, 3.0e-5, 1.0 - 2.0 ** -9, 255.5, 65280.0])
    got = O.bf16_to_f64(O.f64_to_bf16_bits(x))
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -(1.0 + 2.0 ** -7), 0.0,
                     float(torch.tensor(3.0e-5, dtype=torch.float32).to(torch.bfloat16)), 1.0, 256.0, 65280.0])
    assert np.array_equal(got, want)
    # fp32 inputs (exact in double): the library conversion of torch is a single rounding too
    r = torch.randn(20000, generator=synth.gen(3, "cpu")) * 37.0
    assert np.array_equal(O.f64_to_bf16_bits(r.double().numpy()), b16(r.to(torch.bfloat16)))


@pytest.mark.parametrize("bits", [4, 2])
def test_dequantize_is_identity_on_grid_data_and_rounds_once(bits):
    tb = O.tokens_per_block(bits)
    levels = (1 << bits) - 1
    rng = np.random.default_rng(bits)
    k = -2.0 + 0.125 * rng.integers(0, levels + 1, (2 * tb, 2, 128))
    v = 1.0 + 0.25 * rng.integers(0, levels + 1, (2 * tb, 2, 128))
    k[0::tb], k[1::tb] = -2.0, -2.0 + 0.125 * levels    # both ends in every key group
    v[:, :, 0::tb], v[:, :, 1::tb] = 1.0, 1.0 + 0.25 * levels
    kb, vb = bf16_bits_of(k), bf16_bits_of(v)
    rec = O.quantize_records(kb, vb, bits)
    k2, v2 = O.dequantize_records(rec, bits)
    assert np.array_equal(k2, kb) and np.array_equal(v2, vb)
    # random data: equals the bf16 rounding (by torch, from values that are exact in fp32) of the
    # pinned unpacker's doubles
    gen = synth.gen(8, "cpu")
    kr = synth.randn_bf16((tb, 1, 128), gen); vr = synth.randn_bf16((tb, 1, 128), gen)
    rec = O.quantize_records(b16(kr), b16(vr), bits)
    kh, vh = O.unpack_records(rec, bits)
    assert np.array_equal(kh, kh.astype(np.float32).astype(np.float64))
    k3, v3 = O.dequantize_records(rec, bits)
    assert np.array_equal(k3[:, 0], b16(torch.tensor(kh[0], dtype=torch.float32).to(torch.bfloat16)))
    assert np.array_equal(v3[:, 0], b16(torch.tensor(vh[0], dtype=torch.float32).to(torch.bfloat16)))


# ------------------------------------------------------------------ kept positions from scores
def brute_topk(scores, n, k, f, l):
    forced = set(range(f)) | set(range(n - l, n))
    rest = sorted((p for p in range(n) if p not in forced), key=lambda p: (-float(scores[p]), p))
    return sorted(forced | set(rest[:k - len(forced)]))


def test_topk_keep_brute_force_ties_and_forced():
    rng = np.random.default_rng(12)
    ctx_len, keep_len = [13, 40, 7, 1], [5, 17, 7, 1]
    first, last = [2, 4, 0, 3], [1, 6, 9, 0]
    hkv = 3
    scores = np.round(rng.normal(size=sum(ctx_len) * hkv) * 2).astype(np.float32) / 2     # many exact ties
    keep, cu = O.topk_keep(scores, ctx_len, keep_len, hkv, first, last)
    assert cu.tolist() == [0, 5, 22, 29, 30]
    off = 0
    for b, n in enumerate(ctx_len):
        k = keep_len[b]
        f = min(first[b], k); l = min(last[b], k - f)
        for h in range(hkv):
            got = keep[cu[b] * hkv + h * k: cu[b] * hkv + (h + 1) * k].tolist()
            assert got == brute_topk(scores[off:off + n], n, k, f, l)
            off += n


def test_topk_keep_planted_and_degenerate():
    s = np.zeros(10, dtype=np.float32)
    s[[7, 2, 5]] = [3.0, 2.0, 1.0]
    keep, _ = O.topk_keep(s, [10], [2], 1)
    assert keep.tolist() == [2, 7]
    keep, _ = O.topk_keep(s, [10], [5], 1)              # two ties at 0.0 -> positions 0, 1
    assert keep.tolist() == [0, 1, 2, 5, 7]
    keep, _ = O.topk_keep(np.concatenate([s, -s]), [10], [3], 2, [1], [1])
    assert keep.tolist() == [0, 7, 9] + [0, 1, 9]
    keep, cu = O.topk_keep(s, [10], [10], 1)
    assert keep.tolist() == list(range(10)) and cu.tolist() == [0, 10]
    keep, _ = O.topk_keep(s, [10], [0], 1)
    assert keep.size == 0
    # negative zero ties with zero
    z = np.array([0.0, -0.0, 0.0, -0.0], dtype=np.float32)
    assert O.topk_keep(z, [4], [2], 1)[0].tolist() == [0, 1]


def test_topk_keep_matches_generator_lists():
    g = synth.gen(1, "cpu")
    keep, scores = synth.topk_keep(1000, 100, 8, 16, 3, g, return_scores=True)
    got, _ = O.topk_keep(scores.numpy().ravel(), [1000], [100], 3, [8], [16])
    assert np.array_equal(got, keep.numpy().ravel())


# ------------------------------------------------------------------ reload of dropped rows
def test_swap_in_rows_completes_the_pool_and_touches_nothing_else():
    """kept rows (valid in the pool) + reloaded dropped rows = the full KV, for the chosen
    sequences only; rows of other sequences and kept rows keep their poison / their values."""
    rng = np.random.default_rng(0)
    ctx_len, hkv = [9, 5, 12], 2
    cu_ctx = np.concatenate([[0], np.cumsum(ctx_len)])
    total = int(cu_ctx[-1])
    host_k = rng.integers(0, 65536, (total, hkv, 128)).astype(np.uint16)
    host_v = rng.integers(0, 65536, (total, hkv, 128)).astype(np.uint16)
    nd = [4, 2, 7]
    cu_drop = np.concatenate([[0], np.cumsum(nd)])
    lists = []
    for b, n in enumerate(ctx_len):
        for h in range(hkv):
            lists.append(np.sort(rng.choice(n, nd[b], replace=False)))
    dropped = np.concatenate(lists)
    keep, cu_keep = O.keep_from_dropped(dropped, cu_drop, ctx_len, hkv)
    dev_k = np.full_like(host_k, 0xDEAD); dev_v = np.full_like(host_v, 0xBEEF)
    # the resident part: kept rows
    for b, n in enumerate(ctx_len):
        nk = n - nd[b]
        for h in range(hkv):
            for t in keep[cu_keep[b] * hkv + h * nk: cu_keep[b] * hkv + (h + 1) * nk]:
                dev_k[cu_ctx[b] + t, h] = host_k[cu_ctx[b] + t, h]
                dev_v[cu_ctx[b] + t, h] = host_v[cu_ctx[b] + t, h]
    pk, pv = O.pack_rows(host_k, host_v, dropped, cu_drop, cu_ctx, hkv)
    assert pk.shape == (int(cu_drop[-1]) * hkv, 128)
    # packed row order: list (b, h) after list, entries in list order (checked on one planted row)
    b, h, i = 2, 1, 3
    start = cu_drop[b] * hkv + h * nd[b]
    assert np.array_equal(pk[start + i], host_k[cu_ctx[b] + dropped[start + i], h])
    k2, v2 = O.swap_in_rows(pk, pv, dev_k, dev_v, dropped, cu_drop, cu_ctx, hkv, [0, 2])
    for b in (0, 2):
        lo, hi = cu_ctx[b], cu_ctx[b + 1]
        assert np.array_equal(k2[lo:hi], host_k[lo:hi]) and np.array_equal(v2[lo:hi], host_v[lo:hi])
    lo, hi = cu_ctx[1], cu_ctx[2]
    assert np.array_equal(k2[lo:hi], dev_k[lo:hi]) and np.array_equal(v2[lo:hi], dev_v[lo:hi])
    assert (k2[lo:hi] == 0xDEAD).sum() == nd[1] * hkv * 128
