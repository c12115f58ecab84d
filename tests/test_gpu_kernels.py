"""Kernel-level parity: each HIP kernel behind the C ABI against the CPU oracle on the same seeded
inputs.  Integer results (codes, {min,scale} bits, stored FP16 rows) must match bit for bit; FP16
activations within relative L2 2e-3 and max abs 1e-2."""
import math

import numpy as np
import pytest
import torch

from oracle import fg_oracle as O
from paper_2303_06865_amd import binding as B
from paper_2303_06865_amd import synth
from tests.util import assert_close, dev, host, rel_l2
from tests.weight_layout import tile_weights

pytestmark = pytest.mark.gpu


def _rand16(shape, std, seed):
    return (np.random.default_rng(seed).standard_normal(shape) * std).astype(np.float16)


# ------------------------------------------------------------------ quantizer
@pytest.mark.parametrize("rows,cols,std", [(1, 64, 1.0), (37, 576, 0.02), (513, 12288, 0.02), (7, 64 * 5, 30.0),
                                           (144, 768, 1.0), (3, 49152, 0.02)])
def test_quantize_bit_exact(rows, cols, std):
    x = _rand16((rows, cols), std, rows * 7 + cols)
    codes_ref, meta_ref = O.quantize_groupwise(x)
    codes, meta = B.fg_quantize_groupwise(dev(x))
    torch.cuda.synchronize()
    assert np.array_equal(host(codes), codes_ref)
    assert np.array_equal(host(meta).view(np.uint32), meta_ref.view(np.uint32))


def test_quantize_edge_groups_bit_exact():
    x = np.zeros((6, 128), np.float16)
    x[0, :64] = 0.37                                   # constant group
    x[0, 64:] = np.tile(np.arange(16), 4)              # integers 0..15: scale 1
    x[1, 1] = 15.0
    x[1, 2:6] = [0.5, 1.5, 2.5, 3.5]                   # exact ties -> even
    x[2] = _rand16(128, 1e-4, 1)                       # tiny values (FP16 subnormals present)
    x[3] = _rand16(128, 2000.0, 2)                     # large values
    x[4, :64] = -5.0
    x[4, 64:] = np.linspace(-3, 4.5, 64).astype(np.float16)
    x[5] = np.float16(65504.0) * np.sign(_rand16(128, 1.0, 3)).astype(np.float16)   # +-max finite
    codes_ref, meta_ref = O.quantize_groupwise(x)
    codes, meta = B.fg_quantize_groupwise(dev(x))
    torch.cuda.synchronize()
    assert np.array_equal(host(codes), codes_ref)
    assert np.array_equal(host(meta).view(np.uint32), meta_ref.view(np.uint32))
    assert list(O.unpack_codes(host(codes))[1, 2:6]) == [0, 2, 2, 4]


@pytest.mark.parametrize("rows,cols,std", [(1, 64, 1.0), (37, 576, 0.02), (257, 12288, 0.02), (7, 64 * 5, 30.0),
                                           (9, 256, 1e-4), (5, 128, 3000.0)])
def test_quantize_h16_variant_bit_exact(rows, cols, std):
    """FP16 {min, scale} pairs: same bit-exactness bar, including scales in the FP16 subnormal range."""
    x = _rand16((rows, cols), std, rows * 11 + cols)
    x[0, :64] = x[0, 0]                                  # a constant group
    codes_ref, meta_ref = O.quantize_groupwise_h16(x)
    codes, meta = B.fg_quantize_groupwise(dev(x), meta_f16=True)
    torch.cuda.synchronize()
    assert meta.dtype == torch.float16
    assert np.array_equal(host(meta).view(np.uint16), meta_ref.view(np.uint16))
    assert np.array_equal(host(codes), codes_ref)
    out = B.fg_dequantize_groupwise(dev(codes_ref), dev(meta_ref))
    torch.cuda.synchronize()
    ref = O.dequantize_groupwise(codes_ref, meta_ref)
    assert np.array_equal(host(out).view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("meta_f16", [False, True])
def test_quantize_arbitrary_finite_bit_patterns_bit_exact(meta_f16):
    """Every finite FP16 bit pattern can occur: subnormals, both zeros, the largest magnitudes, groups
    whose maximum is 0 (where min + 15*scale does not return the maximum exactly).  Codes, pairs and
    both dequantized forms (binary32 for the cache, FP16 for the weights) must equal the oracle's."""
    rng = np.random.default_rng(17)
    bits = rng.integers(0, 1 << 16, size=(64, 512), dtype=np.uint16)
    bits[(bits & 0x7C00) == 0x7C00] &= 0x83FF                    # no infinities or NaNs
    x = bits.view(np.float16).copy()
    x[0] = np.float16(-1.0)
    x[0, ::64] = 0.0                                             # maximum 0, minimum -1 in every group
    x[1, :64] = np.float16(5.96e-8)
    x[1, 0] = 0.0                                                # range of one FP16 subnormal unit
    if meta_f16:                                                 # keep the range within what an FP16 scale can express
        x = (x.astype(np.float32) * np.float32(2.0 ** -4)).astype(np.float16)
    quant = O.quantize_groupwise_h16 if meta_f16 else O.quantize_groupwise
    codes_ref, meta_ref = quant(x)
    codes, meta = B.fg_quantize_groupwise(dev(x), meta_f16=meta_f16)
    torch.cuda.synchronize()
    mb = np.uint16 if meta_f16 else np.uint32
    assert np.array_equal(host(codes), codes_ref)
    assert np.array_equal(host(meta).view(mb), meta_ref.view(mb))
    out = B.fg_dequantize_groupwise(codes, meta)
    torch.cuda.synchronize()
    assert np.array_equal(host(out).view(np.uint32), O.dequantize_groupwise(codes_ref, meta_ref).view(np.uint32))
    # the FP16 weight form, read out of the GEMM with one-hot activations (products with 1 and sums with
    # zeros are exact): rows of x as a [64, 512] weight matrix in the tiled layout
    wm = B.Mat(64, 512, B.FG_Q4G64_H16 if meta_f16 else B.FG_Q4G64, codes, meta).tiled()
    w_ref = O.dequantize_groupwise_f16(codes_ref, meta_ref)
    for k0 in (0, 64, 448):
        e = np.zeros((64, 512), np.float16)
        e[np.arange(64), k0 + np.arange(64)] = 1.0               # row i picks column k0 + i
        got = host(B.fg_linear(wm, None, dev(e)))                # got[i, n] = w[n, k0 + i]
        torch.cuda.synchronize()
        # compared as numbers: a weight of -0 comes out of the sum with zeros as +0
        assert np.array_equal(got.astype(np.float32), w_ref[:, k0:k0 + 64].T.astype(np.float32))


def test_quantize_empty_input_is_a_noop():
    x = torch.empty((0, 128), dtype=torch.float16, device="cuda")
    codes, meta = B.fg_quantize_groupwise(x)
    assert codes.shape == (0, 64) and meta.shape == (0, 2, 2)


def test_dequantize_bit_exact():
    x = _rand16((65, 640), 0.5, 5)
    codes_ref, meta_ref = O.quantize_groupwise(x)
    out = B.fg_dequantize_groupwise(dev(codes_ref), dev(meta_ref))
    torch.cuda.synchronize()
    ref = O.dequantize_groupwise(codes_ref, meta_ref)
    assert np.array_equal(host(out).view(np.uint32), ref.view(np.uint32))


# ------------------------------------------------------------------ LayerNorm
@pytest.mark.parametrize("rows,cols", [(1, 768), (5, 12288), (33, 4096), (2, 7168), (3, 64), (4, 4104), (2, 16384), (2, 16392),
                                       (1, 49152)])
def test_layernorm(rows, cols):
    x = (_rand16((rows, cols), 3.0, rows + cols).astype(np.float32) + 0.7).astype(np.float16)
    g = (1 + _rand16(cols, 0.1, 1).astype(np.float32)).astype(np.float16)
    b = _rand16(cols, 0.1, 2)
    ref = O.round_f16(O.layernorm(x, g, b, 1e-5))
    out = B.fg_layernorm(dev(x), dev(g), dev(b), 1e-5)
    torch.cuda.synchronize()
    assert_close(host(out), ref, "layernorm", rel=5e-4, mabs=4e-3)


# ------------------------------------------------------------------ fused dequant + GEMM
def _linear_case(m, n, k, quant, bias, relu, residual, seed, std_w=0.02, std_x=1.0, tiled=False, meta_f16=False):
    w16 = _rand16((n, k), std_w, seed)
    x16 = _rand16((m, k), std_x, seed + 1)
    b16 = _rand16(n, 0.5, seed + 2) if bias else None
    r16 = _rand16((m, n), 1.0, seed + 3) if residual else None
    om = O.Mat.from_f16(w16, quant, meta_f16)
    y = O.linear(x16.astype(np.float64), om, b16)
    if relu:
        y = np.maximum(y, 0.0)
    if residual:
        y = y + r16.astype(np.float64)
    ref = O.round_f16(y)
    wm = B.Mat.from_f16(dev(w16), quant, meta_f16=meta_f16)
    bits = np.uint16 if meta_f16 else np.uint32
    if quant:   # the device-made weights are the oracle's bits
        assert np.array_equal(host(wm.data), om.codes) and np.array_equal(host(wm.meta).view(bits), om.meta.view(bits))
    if tiled:
        wm = wm.tiled()
        tc, tmeta = tile_weights(om.codes, om.meta)
        assert np.array_equal(host(wm.data), tc) and np.array_equal(host(wm.meta).view(bits), tmeta.view(bits))
    out = B.fg_linear(wm, dev(b16), dev(x16), dev(r16), relu)
    torch.cuda.synchronize()
    return host(out), ref


SMALL_M_CASES = [
    # m, n, k, bias, relu, residual
    (1, 256, 128, False, False, False),
    (4, 768, 768, True, False, True),
    (4, 3072, 768, True, True, False),
    (4, 768, 3072, False, False, True),
    (17, 2304, 768, True, False, False),
    (36, 1000, 832, True, False, True),      # ragged N, K = 64 mod 128
    (48, 264, 192, False, True, False),
    (100, 520, 1024, True, False, False),
    (144, 1024, 12288, True, False, True),   # OPT-175B hidden size, one column slab
    (150, 768, 768, False, False, False),
    (200, 512, 256, True, True, True),       # two row blocks
    (300, 776, 448, True, False, True),
]


@pytest.mark.parametrize("quant", [True, False])
@pytest.mark.parametrize("m,n,k,bias,relu,residual", SMALL_M_CASES)
def test_linear_small_m(m, n, k, bias, relu, residual, quant):
    got, ref = _linear_case(m, n, k, quant, bias, relu, residual, seed=m + n + k)
    assert_close(got, ref, "linear m=%d n=%d k=%d q=%s" % (m, n, k, quant))


# Row-major FP16 weights with up to 128 rows take the narrow-tile weight streamer (csrc/fg_gemm_f16w.hip).
# `cols` fixes its tile width (16 * cols columns; 0 = the library's own choice), so that every width is run
# on whole tiles, on tiles split along K with the reduction pass, on more than one round of tiles, on
# contractions shorter and longer than the copy ring, and on every row-tile count.
F16W_CASES = [
    # m, n, k, bias, relu, residual
    (1, 192, 64, False, False, False),        # one K step, 3..12 tiles
    (128, 768, 256, True, False, True),       # fewer (tile, K step) units than workgroups: empty ranges
    (100, 1536, 1024, True, True, False),
    (128, 12288, 256, False, False, True),    # 256 whole tiles of 48 columns; 3 rounds of 16; 192 split tiles of 64
    (33, 3072, 2048, True, False, True),      # 32 K steps: longer than the 12-step weight ring
    (64, 6144, 192, True, False, False),
    (77, 6144, 448, False, True, True),       # three 32-row tiles, ragged
    (17, 16384, 128, True, False, False),     # 1024 tiles of 16: four whole rounds
]


@pytest.mark.parametrize("cols", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("m,n,k,bias,relu,residual", F16W_CASES)
def test_linear_f16_weights_narrow_tiles(m, n, k, bias, relu, residual, cols, monkeypatch):
    if cols:
        monkeypatch.setenv("FG_F16W_COLS", str(cols))
    else:
        monkeypatch.delenv("FG_F16W_COLS", raising=False)
    got, ref = _linear_case(m, n, k, False, bias, relu, residual, seed=m + n + k + cols)
    assert_close(got, ref, "linear f16w m=%d n=%d k=%d cols=%d" % (m, n, k, cols))


@pytest.mark.parametrize("quant", [True, False])
@pytest.mark.parametrize("m,n,k,bias,relu,residual", [
    (600, 768, 768, True, False, True),
    (1100, 520, 448, True, True, False),      # ragged M, N; K = 7 groups
    (2048, 3072, 768, False, False, False),
    (513, 256, 3072, True, False, True),
    (1100, 544, 448, True, True, False),      # FP16: 256 x 256 tiles with a ragged last column block (544 = 17 x 32)
    (4100, 4352, 128, True, False, True),     # 17 x 17 tiles: one whole round + 33 stream-K tiles, ragged last row block
    (2049, 8224, 192, True, False, False),    # 9 x 33 tiles, ragged rows and a ragged column block
    (600, 512, 64, True, False, True),        # a single K step: every look-ahead copy is a clamped one
])
def test_linear_large_m(m, n, k, bias, relu, residual, quant):
    got, ref = _linear_case(m, n, k, quant, bias, relu, residual, seed=m + n + k)
    assert_close(got, ref, "linear m=%d n=%d k=%d q=%s" % (m, n, k, quant))


TILED_CASES = [
    (1, 256, 128, False, False, False),
    (4, 768, 768, True, False, True),
    (4, 3072, 768, True, True, False),
    (17, 2304, 768, True, False, False),
    (36, 992, 832, True, False, True),       # ragged column block (992 = 31 tiles of 32)
    (48, 288, 192, False, True, False),
    (70, 512, 640, True, True, True),        # five 16-row tiles
    (96, 512, 640, True, False, True),       # six 16-row tiles (eight-wave kernel at an even count)
    (100, 544, 1024, True, False, False),
    (128, 1280, 512, False, True, False),    # eight 16-row tiles
    (250, 768, 256, True, False, True),      # two blocks of eight 16-row tiles, ragged
    (112, 36864, 256, False, False, True),   # 144 whole tiles of seven 16-row tiles: no reduction pass at all
    (144, 1024, 12288, True, False, True),   # 4 tiles over 256 workgroups: 64 contributors per tile in the reduction pass
    (288, 1280, 512, True, False, True),     # two row blocks of nine 16-row tiles
    (150, 768, 768, False, False, False),
    (200, 512, 256, True, True, True),       # two row blocks
    (300, 800, 448, True, False, True),
    (161, 320, 64, True, False, True),       # smallest prefill-shape launch: one ragged 256-row block, one K step
    (600, 768, 768, True, False, True),      # prefill shape (256-row blocks, 8 waves), stream-K pieces only
    (1100, 544, 448, True, True, False),
    (4100, 4352, 128, True, False, True),    # 17 x 17 tiles: one whole round + 33 stream-K tiles, ragged last block
    (2304, 15360, 64, False, True, False),   # 540 tiles: two whole rounds + 28
    (2049, 8224, 192, True, False, False),   # 9 x 33 tiles, ragged rows and a ragged column block
]


@pytest.mark.parametrize("m,n,k,bias,relu,residual", TILED_CASES)
def test_linear_tiled_weights(m, n, k, bias, relu, residual):
    got, ref = _linear_case(m, n, k, True, bias, relu, residual, seed=m + n + k, tiled=True)
    assert_close(got, ref, "tiled linear m=%d n=%d k=%d" % (m, n, k))


@pytest.mark.parametrize("m,n,k,bias,relu,residual", TILED_CASES)
def test_linear_tiled_weights_fp16_pairs(m, n, k, bias, relu, residual):
    """Tiled 4-bit weights whose {min, scale} pairs are FP16 (0.5625 bytes per weight)."""
    got, ref = _linear_case(m, n, k, True, bias, relu, residual, seed=m + n + k + 7, tiled=True, meta_f16=True)
    assert_close(got, ref, "tiled FP16-pair linear m=%d n=%d k=%d" % (m, n, k))


def test_linear_rejects_canonical_fp16_pair_weights():
    """Only the tiled form of an FP16-pair matrix can be multiplied."""
    wq = B.Mat.from_f16(dev(_rand16((64, 128), 0.02, 5)), True, meta_f16=True)
    with pytest.raises(RuntimeError):
        B.fg_linear(wq, None, dev(_rand16((4, 128), 1.0, 6)))


def test_linear_identity_and_onehot():
    """Special cases that fix the orientation of W ([out, in]) and the K order inside a group."""
    eye = np.eye(128, dtype=np.float16)
    x = _rand16((5, 128), 1.0, 3)
    out = B.fg_linear(B.Mat.from_f16(dev(eye), False), None, dev(x))
    assert np.array_equal(host(out), x)
    w = _rand16((64, 256), 0.5, 4)
    wq = B.Mat.from_f16(dev(w), True)
    what = O.Mat.from_f16(w, True).dense()
    for kk in (0, 1, 5, 63, 64, 130, 255):
        e = np.zeros((1, 256), np.float16)
        e[0, kk] = 1.0
        col = host(B.fg_linear(wq, None, dev(e)))[0]
        assert_close(col, O.round_f16(what[:, kk]), "one-hot k=%d" % kk, rel=1e-3, mabs=2e-3)


# ------------------------------------------------------------------ KV append
@pytest.mark.parametrize("quant", [True, False, "h16"])
@pytest.mark.parametrize("nh,dh", [(3, 128), (12, 64)])
def test_kv_append_bit_exact(nh, dh, quant):
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 1000, 64)
    b, s, cap, boff, pos0 = 3, 5, 16, 1, 4
    qkv = _rand16((b * s, 3 * h1), 1.0, nh + dh)
    h16 = quant == "h16"
    quant = bool(quant)
    okv = O.KVCache.empty(5, nh, cap, dh, quant, h16)
    okv.store(boff, pos0, qkv[:, h1:2 * h1].reshape(b, s, h1), qkv[:, 2 * h1:].reshape(b, s, h1))
    kv = B.KVCache(cfg, 5, cap, quant, meta_f16=h16)
    dq = dev(qkv)
    B.fg_kv_append(cfg, dq[:, h1:], dq[:, 2 * h1:], 3 * h1, b, s, kv, boff, pos0)
    torch.cuda.synchronize()
    if quant:
        assert np.array_equal(host(kv.k_codes), okv.k_codes) and np.array_equal(host(kv.v_codes), okv.v_codes)
        bits = np.uint16 if h16 else np.uint32
        assert np.array_equal(host(kv.k_meta).view(bits), okv.k_meta.view(bits))
        assert np.array_equal(host(kv.v_meta).view(bits), okv.v_meta.view(bits))
    else:
        assert np.array_equal(host(kv.k_codes), okv.k_f16) and np.array_equal(host(kv.v_codes), okv.v_f16)


# ------------------------------------------------------------------ decode attention
def _decode_attn_case(nh, dh, quant, rows, b=3, batch=4, boff=1, seed=0, kstd=1.0, meta_f16=False):
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 1000, 4096)
    cap = rows + 3
    k16 = _rand16((batch, rows, h1), kstd, seed)
    v16 = _rand16((batch, rows, h1), 1.0, seed + 1)
    q16 = _rand16((b, 3 * h1), 1.0, seed + 2)
    okv = O.KVCache.empty(batch, nh, cap, dh, quant, meta_f16)
    okv.store(0, 0, k16, v16)
    ref = np.empty((b, nh, dh))
    for i in range(b):
        for h in range(nh):
            kh, vh = okv.load(boff + i, h, rows)
            ref[i, h] = O.attn_decode(q16[i, h * dh:(h + 1) * dh].astype(np.float64), kh, vh)
    ref = O.round_f16(ref.reshape(b, h1))
    kv = B.KVCache(cfg, batch, cap, quant, meta_f16=meta_f16)
    if quant:   # upload the oracle's cache bytes: this test isolates the attention kernel
        kv.k_codes.copy_(dev(okv.k_codes)); kv.v_codes.copy_(dev(okv.v_codes))
        kv.k_meta.copy_(dev(okv.k_meta)); kv.v_meta.copy_(dev(okv.v_meta))
    else:
        kv.k_codes.copy_(dev(okv.k_f16)); kv.v_codes.copy_(dev(okv.v_f16))
    out = B.fg_decode_attention(cfg, dev(q16), 3 * h1, b, rows, kv, boff)
    torch.cuda.synchronize()
    return host(out), ref


@pytest.mark.parametrize("quant", [True, False])
@pytest.mark.parametrize("nh,dh", [(2, 128), (3, 64)])
@pytest.mark.parametrize("rows", [1, 2, 5, 63, 64, 65, 127, 128, 129, 255, 257, 600, 1100])
def test_decode_attention(rows, nh, dh, quant):
    got, ref = _decode_attn_case(nh, dh, quant, rows, seed=rows)
    assert_close(got, ref, "decode attention rows=%d dh=%d q=%s" % (rows, dh, quant))


@pytest.mark.parametrize("nh,dh", [(2, 128), (3, 64)])
@pytest.mark.parametrize("rows", [1, 63, 65, 129, 257, 600])
def test_decode_attention_fp16_pair_cache(rows, nh, dh):
    got, ref = _decode_attn_case(nh, dh, True, rows, seed=rows + 1, meta_f16=True)
    assert_close(got, ref, "decode attention, FP16 pairs, rows=%d dh=%d" % (rows, dh))


def test_decode_attention_fp16_pair_cache_many_heads():
    got, ref = _decode_attn_case(51, 128, True, 150, b=41, batch=42, boff=1, seed=8, meta_f16=True)
    assert_close(got, ref, "decode attention, FP16 pairs, one wave per head")


@pytest.mark.parametrize("quant", [True, False])
@pytest.mark.parametrize("b,nh,dh,rows", [
    (33, 33, 64, 200),     # 1089 heads: two waves per head, the last workgroup has one head only
    (41, 51, 128, 150),    # 2091 heads: one wave per head, one surplus wave in the last workgroup
    (40, 52, 64, 70),      # 2080 heads, a single chunk each (one wave per head, no second buffer)
])
def test_decode_attention_many_heads(b, nh, dh, rows, quant):
    """The kernel uses fewer waves per head when there are many heads: cover those launch shapes."""
    got, ref = _decode_attn_case(nh, dh, quant, rows, b=b, batch=b + 1, boff=1, seed=b + rows)
    assert_close(got, ref, "decode attention b=%d nh=%d dh=%d rows=%d q=%s" % (b, nh, dh, rows, quant))


@pytest.mark.parametrize("b,nh,dh,rows,meta_f16", [
    (51, 72, 64, 70, False),     # 3672 heads
    (57, 75, 64, 130, True),     # 4275 heads, the last workgroup has three of its four waves busy
    (33, 128, 128, 90, False),   # 4224 heads at head size 128
])
def test_decode_attention_more_heads_than_wave_slots(b, nh, dh, rows, meta_f16):
    """More heads than the chip holds waves at once (3072): the launch runs in several rounds."""
    got, ref = _decode_attn_case(nh, dh, True, rows, b=b, batch=b, boff=0, seed=b + nh, meta_f16=meta_f16)
    assert_close(got, ref, "decode attention, b=%d nh=%d dh=%d" % (b, nh, dh))


@pytest.mark.parametrize("quant", [True, False])
def test_decode_attention_peaked_softmax(quant):
    """Large key norm: a near one-hot softmax, where a wrong max/rescale shows immediately."""
    got, ref = _decode_attn_case(2, 128, quant, 300, seed=77, kstd=4.0)
    assert_close(got, ref, "peaked softmax")


# ------------------------------------------------------------------ Top-K sparse decode attention
def _topk_case(nh, dh, rows, topk, seed, b=3, batch=4, boff=1, dup_rows=False, meta_f16=False):
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 1000, 4096)
    cap = rows + 3
    k16 = _rand16((batch, rows, h1), 1.0, seed)
    if dup_rows:   # every cached key row identical: all scores tie exactly
        k16[:] = k16[:, :1]
    v16 = _rand16((batch, rows, h1), 1.0, seed + 1)
    q16 = _rand16((b, 3 * h1), 1.0, seed + 2)
    okv = O.KVCache.empty(batch, nh, cap, dh, True, meta_f16)
    okv.store(0, 0, k16, v16)
    kv = B.KVCache(cfg, batch, cap, True, meta_f16=meta_f16)
    kv.k_codes.copy_(dev(okv.k_codes)); kv.v_codes.copy_(dev(okv.v_codes))
    kv.k_meta.copy_(dev(okv.k_meta)); kv.v_meta.copy_(dev(okv.v_meta))
    out, kept = B.fg_decode_attention_topk(cfg, dev(q16), 3 * h1, b, rows, topk, kv, boff, want_rows=True)
    torch.cuda.synchronize()
    out, kept = host(out), host(kept)
    ref = np.empty((b, nh, dh))
    exact = 0
    for i in range(b):
        for h in range(nh):
            kh, vh = okv.load(boff + i, h, rows)
            qv = q16[i, h * dh:(h + 1) * dh].astype(np.float64)
            sc = O.attn_decode_scores(qv, kh)
            got = kept[i, h]
            # a valid index set: ascending, distinct, in range
            assert np.all(np.diff(got) > 0) and got[0] >= 0 and got[-1] < rows
            # ... that is a top-k set of the oracle's scores up to the kernel's FP32 score error
            srt = np.sort(sc)[::-1]
            thr = srt[topk - 1]
            eps = 2e-5 * (1.0 + np.abs(sc).max())
            mask = np.zeros(rows, bool)
            mask[got] = True
            assert sc[mask].min() >= thr - eps and (topk == rows or sc[~mask].max() <= thr + eps)
            # where the k-th and (k+1)-th scores are clearly apart the set is THE top-k set
            if topk == rows or srt[topk - 1] - srt[topk] > 2 * eps:
                assert np.array_equal(got, O.topk_indices(sc, topk))
                exact += 1
            ref[i, h] = O.attn_decode_subset(qv, kh, vh, got.astype(np.int64))
    return out, O.round_f16(ref.reshape(b, h1)), kept, exact


@pytest.mark.parametrize("nh,dh", [(2, 128), (3, 64)])
@pytest.mark.parametrize("rows,topk", [(1, 1), (5, 2), (64, 7), (65, 65), (129, 13), (200, 20), (528, 53),
                                       (528, 1), (1100, 110), (2100, 210)])
def test_decode_attention_topk(rows, topk, nh, dh):
    out, ref, _, exact = _topk_case(nh, dh, rows, topk, seed=rows + topk)
    assert exact > 0   # random scores: at least one head must have had an unambiguous boundary
    assert_close(out, ref, "top-k attention rows=%d k=%d dh=%d" % (rows, topk, dh))


@pytest.mark.parametrize("nh,dh", [(2, 128), (3, 64)])
def test_decode_attention_topk_fp16_pair_cache(nh, dh):
    out, ref, _, exact = _topk_case(nh, dh, 300, 30, seed=21, meta_f16=True)
    assert exact > 0
    assert_close(out, ref, "top-k attention, FP16 pairs, dh=%d" % dh)


@pytest.mark.parametrize("nh,dh", [(2, 128), (3, 64)])
def test_decode_attention_topk_ties_keep_lowest_rows(nh, dh):
    out, ref, kept, _ = _topk_case(nh, dh, 300, 37, seed=5, dup_rows=True)
    assert np.array_equal(kept, np.broadcast_to(np.arange(37, dtype=np.int32), kept.shape))
    assert_close(out, ref, "top-k attention, all scores tied")


def test_decode_attention_topk_full_k_equals_dense():
    """Keeping every row must reproduce the dense kernel's result (same cache, same query)."""
    nh, dh, rows = 2, 128, 333
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 1000, 4096)
    kv = B.KVCache(cfg, 2, rows + 1, True)
    k16 = dev(_rand16((2 * rows, h1), 1.0, 1)); v16 = dev(_rand16((2 * rows, h1), 1.0, 2))
    B.fg_kv_append(cfg, k16, v16, h1, 2, rows, kv, 0, 0)
    q = dev(_rand16((2, 3 * h1), 1.0, 3))
    dense = host(B.fg_decode_attention(cfg, q, 3 * h1, 2, rows, kv, 0))
    sparse = host(B.fg_decode_attention_topk(cfg, q, 3 * h1, 2, rows, rows, kv, 0))
    assert_close(sparse, dense.astype(np.float64), "top-k with k = rows vs dense", rel=1e-3, mabs=2e-3)


# ------------------------------------------------------------------ prefill attention
@pytest.mark.parametrize("nh,dh", [(2, 128), (3, 64)])
@pytest.mark.parametrize("b,s", [(1, 1), (2, 7), (1, 64), (2, 65), (1, 100), (1, 200), (3, 32), (1, 127), (2, 128),
                                 (1, 129), (1, 300), (2, 512)])
def test_prefill_attention(b, s, nh, dh):
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 1000, 4096)
    qkv = _rand16((b * s, 3 * h1), 1.0, b * 100 + s)
    x = qkv.astype(np.float64).reshape(b, s, 3, nh, dh)
    ref = np.empty((b, s, nh, dh))
    for i in range(b):
        for h in range(nh):
            ref[i, :, h] = O.attn_prefill(x[i, :, 0, h], x[i, :, 1, h], x[i, :, 2, h])
    ref = O.round_f16(ref.reshape(b * s, h1))
    out = B.fg_prefill_attention(cfg, dev(qkv), b, s)
    torch.cuda.synchronize()
    assert_close(host(out), ref, "prefill attention b=%d s=%d dh=%d" % (b, s, dh))


# ------------------------------------------------------------------ embedding and LM head
def test_embed_bit_exact():
    sh = synth.Shape(h1=256, nh=2, h2=512, vocab=1000, max_pos=64)
    cfg = B.Cfg(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos)
    m = synth.model_tensors(sh, 3, std=0.5)
    ids = synth.prompt_ids(3, 7, sh.vocab, 3)
    ref = O.embed(ids, np.broadcast_to(np.arange(7), (3, 7)), m["embed"], m["pos"]).reshape(21, sh.h1)
    out = B.fg_embed(cfg, dev(m["embed"]), dev(m["pos"]), dev(ids.reshape(-1)), 7, 0)
    assert np.array_equal(host(out), ref)
    ref = O.embed(ids[:, 0], np.full(3, 11), m["embed"], m["pos"])
    out = B.fg_embed(cfg, dev(m["embed"]), dev(m["pos"]), dev(np.ascontiguousarray(ids[:, 0])), 1, 11)
    assert np.array_equal(host(out), ref)


# (400 rows: the LM head on the 256-row prefill tiles, binary32 logits stored two columns per lane, ragged
#  last row block and a last column block of one 32-column tile)
@pytest.mark.parametrize("rows,vocab,h1", [(4, 50272, 768), (37, 1000, 256), (144, 5000, 1024), (400, 4128, 512)])
def test_lm_head_greedy(rows, vocab, h1):
    sh = synth.Shape(h1=h1, nh=h1 // 64, h2=4 * h1, vocab=vocab, max_pos=64)
    ocfg = O.ModelCfg(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos)
    cfg = B.Cfg(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos)
    m = synth.model_tensors(sh, 5, std=0.02)
    x = _rand16((rows, h1), 2.0, 9)
    g = (1 + _rand16(h1, 0.1, 1).astype(np.float32)).astype(np.float16)
    bb = _rand16(h1, 0.1, 2)
    ref = O.lm_head_logits(ocfg, x, g, bb, m["embed"])
    ids, logits = B.fg_lm_head_greedy(cfg, dev(x), dev(g), dev(bb), dev(m["embed"]))
    torch.cuda.synchronize()
    lg = host(logits)
    assert_close(lg, ref, "logits", rel=2e-3, mabs=1e-2)
    # the GPU's ids are the lowest-index argmax of the GPU's own binary32 logits ...
    assert np.array_equal(host(ids), np.argmax(lg, axis=-1).astype(np.int32))
    # ... and equal the oracle's wherever the oracle's top-2 margin exceeds the logit error
    srt = np.sort(ref, axis=-1)
    margin = srt[:, -1] - srt[:, -2]
    err = np.abs(lg - ref).max()
    safe = margin > 2 * err
    assert safe.sum() >= rows * 0.9
    assert np.array_equal(host(ids)[safe], O.greedy(ref)[safe])


def test_argmax_lowest_index_on_exact_ties():
    """All-zero hidden state and beta = 0 give all-zero logits: token 0 must win every row."""
    sh = synth.Shape(h1=128, nh=2, h2=512, vocab=520, max_pos=8)
    cfg = B.Cfg(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos)
    m = synth.model_tensors(sh, 1)
    x = np.zeros((3, 128), np.float16)
    ids, logits = B.fg_lm_head_greedy(cfg, dev(x), dev(np.ones(128, np.float16)), dev(np.zeros(128, np.float16)),
                                      dev(m["embed"]))
    assert np.all(host(logits) == 0) and np.all(host(ids) == 0)


# ------------------------------------------------------------------ determinism
def test_results_are_bit_identical_from_run_to_run():
    """Nothing in the path depends on the order in which workgroups finish: the stream-K partial sums
    are added up by a second pass in a fixed order, the attention kernels merge per-wave results in a
    fixed order.  Same inputs, same bits, every time."""
    w = dev(_rand16((2304, 768), 0.02, 1))
    x = dev(_rand16((144, 768), 1.0, 2))
    wm = B.Mat.from_f16(w, True, tiled=True)
    ref = B.fg_linear(wm, None, x).clone()
    big = B.Mat.from_f16(dev(_rand16((4352, 128), 0.02, 3)), True, tiled=True)
    xb = dev(_rand16((4100, 128), 1.0, 4))
    refb = B.fg_linear(big, None, xb).clone()
    nh, dh, rows = 12, 64, 300
    cfg = B.Cfg(nh * dh, nh, 4 * nh * dh, 1000, 512)
    kv = B.KVCache(cfg, 5, rows, True)
    kvx = dev(_rand16((5 * rows, 3 * nh * dh), 1.0, 5))
    B.fg_kv_append(cfg, kvx[:, nh * dh:], kvx[:, 2 * nh * dh:], 3 * nh * dh, 5, rows, kv, 0, 0)
    q = dev(_rand16((5, 3 * nh * dh), 1.0, 6))
    refa = B.fg_decode_attention(cfg, q, 3 * nh * dh, 5, rows, kv, 0).clone()
    refp = B.fg_prefill_attention(cfg, kvx[:rows * 5], 5, rows).clone()
    torch.cuda.synchronize()
    for _ in range(5):
        assert torch.equal(B.fg_linear(wm, None, x), ref)
        assert torch.equal(B.fg_linear(big, None, xb), refb)
        assert torch.equal(B.fg_decode_attention(cfg, q, 3 * nh * dh, 5, rows, kv, 0), refa)
        assert torch.equal(B.fg_prefill_attention(cfg, kvx[:rows * 5], 5, rows), refp)
