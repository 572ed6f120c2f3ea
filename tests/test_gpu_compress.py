"""GPU parity of the compressor-side entry points (vc_compress_quant, vc_decompress_quant,
vc_topk_keep) against the oracle: records, bf16 rows and kept-index lists are integer / byte
results, so everything here is compared bit for bit."""
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


def i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


def make_ragged(bits, lens, hkv, seed):
    tb = synth.tokens_per_block(bits)
    g = synth.gen(seed, DEV)
    total = sum(lens)
    k = synth.randn_bf16((total, hkv, 128), g)
    v = synth.randn_bf16((total, hkv, 128), g)
    k[:, 0, 5] *= 10.0                                  # an outlier key channel
    if lens[0] >= tb:
        k[0:tb, hkv - 1, 17] = 0.75                     # a constant key group
        v[3, 0, 0:tb] = -1.25                           # a constant value group
        v[4, 0, tb:2 * tb] = 0.0                        # zeros
        k[0:tb, 0, 40] = k[0:tb, 0, 40].abs()           # a key group whose minimum is -0.0 (stored zero point: +0)
        k[tb // 2, 0, 40] = -0.0
        k[1, 0, 40] = 0.0
        v[6, 0, 0:tb] = v[6, 0, 0:tb].abs()             # a value group whose minimum is -0.0
        v[6, 0, tb - 1] = -0.0
    nb = [n // tb for n in lens]
    cu_ctx = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cu_blk = np.concatenate([[0], np.cumsum(nb)]).astype(np.int32)
    return k, v, nb, cu_ctx, cu_blk


def oracle_records(k, v, bits, lens, cu_ctx):
    pieces = []
    for b, n in enumerate(lens):
        lo = int(cu_ctx[b])
        r = O.quantize_records(H.bits16(k[lo:lo + n]), H.bits16(v[lo:lo + n]), bits)
        pieces.append(r.reshape(-1, 5120))
    return np.concatenate(pieces) if pieces else np.zeros((0, 5120), dtype=np.uint8)


@pytest.mark.parametrize("bits", [4, 2])
@pytest.mark.parametrize("lens,hkv", [([200, 64, 7, 333], 2), ([128], 1), ([1000, 129], 3)])
def test_compress_and_decompress_match_oracle(lib, ctx, bits, lens, hkv):
    print(f"[compress] bits {bits} lens {lens} hkv {hkv}", flush=True)
    tb = synth.tokens_per_block(bits)
    k, v, nb, cu_ctx, cu_blk = make_ragged(bits, lens, hkv, 100 + bits)
    nrec = int(cu_blk[-1]) * hkv
    blocks = torch.full((max(nrec, 1), 5120), 0xAB, dtype=torch.uint8, device=DEV)
    lib.vc_compress_quant(ctx, k, v, i32(cu_ctx), i32(cu_blk), bits, max(nb), blocks)
    torch.cuda.synchronize()
    ref = oracle_records(k, v, bits, lens, cu_ctx)
    got = blocks[:nrec].cpu().numpy()
    assert got.shape == ref.shape
    bad = np.argwhere(got != ref)
    assert bad.size == 0, f"first differing (record, byte): {bad[:5].tolist()}"
    # inverse: rows of compressed tokens equal the oracle's, rows beyond nb*TB are left alone
    k_out = torch.full_like(k, float("nan")); v_out = torch.full_like(v, float("nan"))
    lib.vc_decompress_quant(ctx, blocks, i32(cu_blk), i32(cu_ctx), bits, max(nb), k_out, v_out)
    torch.cuda.synchronize()
    ko, vo = H.bits16(k_out), H.bits16(v_out)
    nan_bits = H.bits16(torch.full((1,), float("nan"), dtype=torch.bfloat16))[0]
    r0 = 0
    for b, n in enumerate(lens):
        lo = int(cu_ctx[b])
        cnt = nb[b] * tb
        if cnt:
            rk, rv = O.dequantize_records(ref[r0:r0 + nb[b] * hkv].reshape(hkv, nb[b], 5120), bits)
            assert np.array_equal(ko[lo:lo + cnt], rk) and np.array_equal(vo[lo:lo + cnt], rv)
        assert (ko[lo + cnt:lo + n] == nan_bits).all() and (vo[lo + cnt:lo + n] == nan_bits).all()
        r0 += nb[b] * hkv


def test_compress_fewer_blocks_than_fit_and_empty(lib, ctx):
    """The caller may compress only a prefix of each sequence; n_seqs = 0 and max_blk = 0 are no-ops."""
    bits, hkv, lens = 4, 2, [160, 96]
    k, v, _, cu_ctx, _ = make_ragged(bits, lens, hkv, 7)
    nb = [2, 0]
    cu_blk = np.array([0, 2, 2], dtype=np.int32)
    blocks = torch.zeros((4, 5120), dtype=torch.uint8, device=DEV)
    lib.vc_compress_quant(ctx, k, v, i32(cu_ctx), i32(cu_blk), bits, 2, blocks)
    torch.cuda.synchronize()
    ref = O.quantize_records(H.bits16(k[:64]), H.bits16(v[:64]), bits).reshape(-1, 5120)
    assert np.array_equal(blocks.cpu().numpy(), ref)
    lib.vc_compress_quant(ctx, k, v, i32(cu_ctx), i32(cu_blk), bits, 0, blocks)
    lib.vc_compress_quant(ctx, k[:0], v[:0], i32([0]), i32([0]), bits, 0, blocks)
    with pytest.raises(lib.VcError):
        lib.vc_compress_quant(ctx, k, v, i32(cu_ctx), i32(cu_blk), 8, 2, blocks)


@pytest.mark.parametrize("bits", [4, 2])
def test_draft_over_gpu_compressed_records_matches_oracle(lib, ctx, bits):
    """compress -> draft on the GPU against the oracle's draft over the oracle's own records."""
    lay = synth.make_layer(77, DEV, ctx_len=[512, 320], n_q_heads=8, n_kv_heads=2, quant_bits=(bits,))
    tb = synth.tokens_per_block(bits)
    nb = [n // tb for n in lay.ctx_len]
    cu_blk = i32(np.concatenate([[0], np.cumsum(nb)]))
    blocks = torch.empty((sum(nb) * 2, 5120), dtype=torch.uint8, device=DEV)
    lib.vc_compress_quant(ctx, lay.k_full, lay.v_full, lay.cu_ctx, cu_blk, bits, max(nb), blocks)
    assert torch.equal(blocks, lay.blocks[bits].reshape(-1, 5120))
    kw = dict(blocks=blocks, cu_blk=cu_blk, max_blk=max(nb), bits=bits)
    out, lse = H.gpu_draft(lib, ctx, lay, **kw)
    ref, _ = H.oracle_draft(lay, kw)
    assert H.rel_err(out, ref) <= H.TOL


def topk_case(lib, ctx, ctx_len, keep_len, hkv, first, last, scores):
    cu_ctx = i32(np.concatenate([[0], np.cumsum(ctx_len)]))
    klen = [min(k, n) for k, n in zip(keep_len, ctx_len)]
    cu_keep = i32(np.concatenate([[0], np.cumsum(klen)]))
    out = torch.full((max(sum(klen) * hkv, 1),), -9, dtype=torch.int32, device=DEV)
    lib.vc_topk_keep(ctx, scores, cu_ctx, cu_keep, hkv, out,
                     forced_first=None if first is None else i32(first), forced_last=None if last is None else i32(last))
    torch.cuda.synchronize()
    ref, ref_cu = O.topk_keep(scores.cpu().numpy(), ctx_len, keep_len, hkv, first, last)
    assert np.array_equal(out[:sum(klen) * hkv].cpu().numpy(), ref)
    return out


def test_topk_keep_matches_oracle_with_ties_and_forced(lib, ctx):
    rng = np.random.default_rng(5)
    ctx_len = [13, 4000, 7, 1, 70000, 1024, 1025]
    keep_len = [5, 400, 7, 1, 7000, 1, 1100]
    first = [2, 64, 0, 3, 64, 0, 2000]
    last = [1, 256, 9, 0, 256, 0, 5]
    hkv = 3
    n = sum(ctx_len) * hkv
    s = np.round(rng.normal(size=n) * 8).astype(np.float32) / 8          # heavy exact ties
    s[::97] = -0.0
    topk_case(lib, ctx, ctx_len, keep_len, hkv, first, last, torch.tensor(s, device=DEV))
    s2 = rng.normal(size=n).astype(np.float32)                           # no ties
    topk_case(lib, ctx, ctx_len, keep_len, hkv, None, None, torch.tensor(s2, device=DEV))
    # all scores equal: the lowest free positions win
    topk_case(lib, ctx, ctx_len, keep_len, hkv, first, last, torch.zeros(n, device=DEV))
    # extreme magnitudes and infinities order correctly
    s3 = s2.copy(); s3[::5] *= 1e30; s3[3::11] = -np.inf; s3[4::13] = np.inf; s3[5::17] *= 1e-30
    topk_case(lib, ctx, ctx_len, keep_len, hkv, first, last, torch.tensor(s3, device=DEV))


def test_topk_keep_config1_size_reproduces_generator_lists(lib, ctx):
    """64 lists of 32768 positions, 2048 kept, first 64 / last 256 forced: the generator's own
    kept lists (torch sort) and the oracle agree with the library."""
    g = synth.gen(synth.SEED_BASE + 1, DEV)
    keep, scores = synth.topk_keep(32768, 2048, 64, 256, 64, g, return_scores=True)
    out = topk_case(lib, ctx, [32768] * 8, [2048] * 8, 8, [64] * 8, [256] * 8, scores.reshape(-1).contiguous())
    assert torch.equal(out.view(64, 2048), keep)
