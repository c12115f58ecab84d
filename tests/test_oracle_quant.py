"""Pins for the oracle's quantizer (Section 5) that do not come from the oracle
itself: the four invariants of the format, closed-form groups, brute-force
optimality of every code, rounding-mode and packing examples."""
import os

import numpy as np
import pytest

from oracle import fg_oracle as O
from tests.weight_layout import tile_weights

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()[:2]
        out[k] = float(v)
    return out


def _rand16(shape, std, seed):
    return (np.random.default_rng(seed).standard_normal(shape) * std).astype(np.float16)


def test_format_constants_match_paper():
    g = _gold("paper_quant_format.txt")
    assert O.BITS == g["bits"] and O.GROUP == g["group"] and O.QMAX == g["levels"]
    assert O.bytes_per_element(True) == 0.5 + 8 / 64 == 0.625
    assert O.bytes_per_element(False) == 2.0


@pytest.mark.parametrize("std,seed", [(0.02, 1), (1.0, 2), (30.0, 3)])
def test_invariants(std, seed):
    x = _rand16((37, 64 * 9), std, seed)
    codes, meta = O.quantize_groupwise(x)
    assert codes.dtype == np.uint8 and codes.shape == (37, 64 * 9 // 2)
    assert meta.dtype == np.float32 and meta.shape == (37, 9, 2)
    c = O.unpack_codes(codes)
    assert c.min() >= 0 and c.max() <= 15
    xg = x.astype(np.float64).reshape(37, 9, 64)
    cg = c.reshape(37, 9, 64).astype(np.float64)
    mn = meta[..., 0].astype(np.float64)[..., None]
    sc = meta[..., 1].astype(np.float64)[..., None]
    # every dequantized element within scale/2 of the original (evaluated in double)
    err = np.abs(xg - (mn + cg * sc))
    assert np.all(err <= sc / 2 * (1 + 2.0 ** -20))
    # min and max of each group: codes 0 and 15, values round-trip exactly through FP16
    xh = O.dequantize_groupwise(codes, meta).reshape(37, 9, 64)
    imin = xg.argmin(axis=2)[..., None]
    imax = xg.argmax(axis=2)[..., None]
    assert np.all(np.take_along_axis(cg, imin, 2) == 0)
    assert np.all(np.take_along_axis(cg, imax, 2) == 15)
    assert np.array_equal(np.take_along_axis(xh, imin, 2), np.take_along_axis(xg, imin, 2).astype(np.float32))
    assert np.array_equal(np.take_along_axis(xh, imax, 2).astype(np.float16),
                          np.take_along_axis(xg, imax, 2).astype(np.float16))
    # stored min is the true min, stored scale is (max-min)/15 to binary32 rounding
    assert np.array_equal(meta[..., 0], xg.min(axis=2).astype(np.float32))
    ref_scale = (xg.max(axis=2) - xg.min(axis=2)) / 15.0
    assert np.allclose(meta[..., 1], ref_scale, rtol=2 ** -23, atol=0)


def test_bruteforce_each_code_is_nearest_level():
    """For every element, no other of the 16 levels min + c*scale is closer."""
    x = _rand16((16, 256), 0.5, 7)
    codes, meta = O.quantize_groupwise(x)
    c = O.unpack_codes(codes).reshape(16, 4, 64).astype(np.int64)
    xg = x.astype(np.float64).reshape(16, 4, 64)
    mn = meta[..., 0].astype(np.float64)
    sc = meta[..., 1].astype(np.float64)
    levels = mn[..., None] + np.arange(16)[None, None, :] * sc[..., None]      # [16,4,16]
    d = np.abs(xg[..., None] - levels[:, :, None, :])                           # [16,4,64,16]
    best = d.min(axis=-1)
    chosen = np.take_along_axis(d, c[..., None], -1)[..., 0]
    # the chosen level is optimal up to the binary32 rounding of the quotient
    assert np.all(chosen <= best + sc[..., None] * 2.0 ** -20)


def test_closed_form_integer_group():
    """A group holding 0..15 four times: min 0, scale 1, codes equal the values."""
    v = np.tile(np.arange(16), 4).astype(np.float16)[None, :]
    codes, meta = O.quantize_groupwise(v)
    assert meta[0, 0, 0] == 0.0 and meta[0, 0, 1] == 1.0
    assert np.array_equal(O.unpack_codes(codes)[0], np.tile(np.arange(16), 4))
    assert np.array_equal(O.dequantize_groupwise(codes, meta)[0], v[0].astype(np.float32))


def test_closed_form_affine_group():
    """x = -3 + 0.5*k for k in 0..15 (exact in FP16): scale 0.5, code k."""
    k = np.tile(np.arange(16), 4)
    v = (-3.0 + 0.5 * k).astype(np.float16)[None, :]
    codes, meta = O.quantize_groupwise(v)
    assert meta[0, 0, 0] == -3.0 and meta[0, 0, 1] == 0.5
    assert np.array_equal(O.unpack_codes(codes)[0], k)


def test_ties_round_to_even():
    """With min 0 and max 15 the scale is exactly 1, so 0.5, 1.5, 2.5, 3.5 are
    exact ties: nearest-even gives 0, 2, 2, 4."""
    v = np.zeros(64, np.float16)
    v[1] = 15.0
    v[2:6] = [0.5, 1.5, 2.5, 3.5]
    v[6:9] = [0.49, 1.51, 14.5]
    codes, meta = O.quantize_groupwise(v[None, :])
    c = O.unpack_codes(codes)[0]
    assert list(c[2:6]) == [0, 2, 2, 4]
    assert list(c[6:9]) == [0, 2, 14]
    assert c[0] == 0 and c[1] == 15


def test_dequantize_is_single_rounding_of_the_exact_value():
    """min + code*scale evaluated exactly (Python fractions) and rounded once, to binary32 for the
    cache form and to FP16 for the weight form."""
    from fractions import Fraction
    x = _rand16((3, 128), 0.02, 21)
    codes, meta = O.quantize_groupwise(x)
    c = O.unpack_codes(codes)
    d32 = O.dequantize_groupwise(codes, meta)
    d16 = O.dequantize_groupwise_f16(codes, meta)
    assert d32.dtype == np.float32 and d16.dtype == np.float16
    for r in range(3):
        for k in range(0, 128, 7):
            exact = Fraction(float(meta[r, k // 64, 0])) + int(c[r, k]) * Fraction(float(meta[r, k // 64, 1]))
            f = float(exact)                       # exact -> double is itself correctly rounded
            assert d32[r, k] == np.float32(f) and d16[r, k] == np.float16(f)
            # nearest: no neighbouring representable number is closer
            for arr, dt in ((d32, np.float32), (d16, np.float16)):
                v = arr[r, k]
                for nb in (np.nextafter(v, dt(np.inf)), np.nextafter(v, dt(-np.inf))):
                    assert abs(Fraction(float(v)) - exact) <= abs(Fraction(float(nb)) - exact)


def test_constant_group_is_exact():
    v = np.full((2, 128), 0.37, np.float16)
    v[1, 64:] = -2.5
    codes, meta = O.quantize_groupwise(v)
    assert np.all(codes == 0)
    assert np.all(meta[..., 1] == 0)
    assert np.array_equal(O.dequantize_groupwise(codes, meta), v.astype(np.float32))


def test_packing_hand_example():
    """Even element in the low nibble: codes 1,2,3,4,15,0,9,10 -> 0x21 0x43 0x0F 0xA9."""
    c = np.array([[1, 2, 3, 4, 15, 0, 9, 10]], np.uint8)
    b = O.pack_codes(c)
    assert list(b[0]) == [0x21, 0x43, 0x0F, 0xA9]
    assert np.array_equal(O.unpack_codes(b), c)
    r = np.random.default_rng(0).integers(0, 16, size=(5, 128)).astype(np.uint8)
    assert np.array_equal(O.unpack_codes(O.pack_codes(r)), r)


def test_groups_are_independent_and_along_last_axis():
    """Changing one group's data changes only that group's codes and meta."""
    x = _rand16((3, 192), 1.0, 11)
    c0, m0 = O.quantize_groupwise(x)
    y = x.copy()
    y[1, 64:128] *= np.float16(3.0)
    c1, m1 = O.quantize_groupwise(y)
    same = np.ones((3, 3), bool)
    same[1, 1] = False
    assert np.array_equal(m0[same], m1[same])
    assert not np.array_equal(m0[1, 1], m1[1, 1])
    cc0 = c0.reshape(3, 3, 32)
    cc1 = c1.reshape(3, 3, 32)
    assert np.array_equal(cc0[same], cc1[same])


def test_independent_library_formulation():
    """The same definition spelled with torch CPU tensor ops (library min / max /
    round, which rounds half to even) gives identical bits."""
    import torch
    x = _rand16((64, 512), 0.02, 5)
    codes, meta = O.quantize_groupwise(x)
    t = torch.from_numpy(x).float().reshape(64, 8, 64)
    mn = t.amin(dim=2, keepdim=True)
    mx = t.amax(dim=2, keepdim=True)
    sc = (mx - mn) / 15.0
    q = torch.clamp(torch.round((t - mn) / sc), 0, 15).to(torch.uint8).reshape(64, 512)
    assert np.array_equal(O.unpack_codes(codes), q.numpy())
    assert np.array_equal(meta[..., 0], mn[..., 0].numpy())
    assert np.array_equal(meta[..., 1], sc[..., 0].numpy())


def test_rejects_bad_arguments():
    with pytest.raises(ValueError):
        O.quantize_groupwise(np.zeros((2, 96), np.float16))
    with pytest.raises(ValueError):
        O.quantize_groupwise(np.zeros((2, 64), np.float32))
    with pytest.raises(ValueError):
        O.quantize_groupwise(np.zeros((2, 64), np.float16), group=32)
    bad = np.zeros((1, 64), np.float16)
    bad[0, 3] = np.inf
    with pytest.raises(ValueError):
        O.quantize_groupwise(bad)


def test_tiled_order_is_the_documented_permutation():
    """Element by element in plain Python: piece (row, k-tile, half) of the canonical layout lands at
    byte ((row//32 * ktiles + ktile) * 64 + 32*half + row%32) * 16 of the tiled one."""
    n, k = 64, 192
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8)
    meta = rng.standard_normal((n, k // 64, 2)).astype(np.float32)
    tc, tm = tile_weights(codes, meta)
    assert tc.shape == codes.shape and tm.shape == meta.shape
    flat, mflat = tc.reshape(-1), tm.reshape(-1, 2)
    kt = k // 64
    for row in range(n):
        for t in range(kt):
            tile = (row // 32) * kt + t
            assert np.array_equal(mflat[tile * 32 + row % 32], meta[row, t])
            for h in range(2):
                src = codes[row, t * 32 + h * 16: t * 32 + h * 16 + 16]
                dst = (tile * 64 + 32 * h + row % 32) * 16
                assert np.array_equal(flat[dst:dst + 16], src)
    assert sorted(flat.tolist()) == sorted(codes.reshape(-1).tolist())


# ---------------------------------------------------------------- FP16 (min, scale) variant
@pytest.mark.parametrize("std,seed", [(1.0, 1), (0.02, 2), (30.0, 3), (1e-4, 4)])
def test_h16_variant_invariants(std, seed):
    """4.5-bit variant: min is stored exactly, scale is the smallest FP16 not below (max-min)/15, codes
    need no clamping, and every element stays within half a (stored) step of its reconstruction."""
    x = _rand16((37, 256), std, seed)
    codes, meta = O.quantize_groupwise_h16(x)
    assert meta.dtype == np.float16 and meta.shape == (37, 4, 2)
    xg = x.astype(np.float64).reshape(37, 4, 64)
    mn, sc = meta[..., 0].astype(np.float64), meta[..., 1].astype(np.float64)
    assert np.array_equal(mn, xg.min(axis=2))                       # FP16 inputs: min round-trips exactly
    want = (xg.max(axis=2).astype(np.float32) - xg.min(axis=2).astype(np.float32)) / np.float32(15)
    assert np.all(sc >= want)                                       # ... scale is rounded UP
    below = np.nextafter(meta[..., 1], np.float16(-np.inf)).astype(np.float64)
    assert np.all((below < want) | (sc == 0))                       # ... and is the smallest such FP16
    c = O.unpack_codes(codes).reshape(37, 4, 64).astype(np.float64)
    assert c.min() >= 0 and c.max() <= 15
    # unclamped rounding already lands in [0, 15]: nothing was clipped
    t = (xg - mn[..., None]) / np.where(sc > 0, sc, 1.0)[..., None]
    assert np.all(np.rint(t) <= 15)
    xh = O.dequantize_groupwise(codes, meta).astype(np.float64).reshape(37, 4, 64)
    assert np.all(np.abs(xh - xg) <= sc[..., None] * (0.5 + 1e-6) + 1e-12)
    # the group's minimum element reconstructs exactly, the maximum within half a step
    assert np.all(np.take_along_axis(xh, xg.argmin(axis=2)[..., None], 2)[..., 0] == xg.min(axis=2))


def test_h16_variant_agrees_with_the_binary32_format_when_scale_is_representable():
    """Ranges 15 * 2^k make (max-min)/15 an FP16 number: both formats then store the same codes."""
    rng = np.random.default_rng(9)
    x = rng.integers(0, 16, size=(6, 128)).astype(np.float16) * np.float16(0.25) - np.float16(1.5)
    x[:, 0] = -1.5
    x[:, 1] = 2.25            # range 3.75 = 15 * 0.25 in both groups?  (second group gets its own extremes)
    x[:, 64] = -1.5
    x[:, 65] = 2.25
    c32, m32 = O.quantize_groupwise(x)
    c16, m16 = O.quantize_groupwise_h16(x)
    assert np.array_equal(c32, c16)
    assert np.array_equal(m32, m16.astype(np.float32))
    assert np.array_equal(O.dequantize_groupwise(c16, m16), x.astype(np.float32))


def test_h16_variant_bruteforce_and_constant_group():
    x = _rand16((3, 64), 1.0, 12)
    codes, meta = O.quantize_groupwise_h16(x)
    c = O.unpack_codes(codes)
    for r in range(3):
        mn, sc = float(meta[r, 0, 0]), float(meta[r, 0, 1])
        for j in range(64):
            errs = [abs(mn + k * sc - float(x[r, j])) for k in range(16)]
            assert errs[c[r, j]] <= min(errs) + 1e-7     # the chosen level is a nearest one
    z = np.full((2, 64), 0.75, np.float16)
    cz, mz = O.quantize_groupwise_h16(z)
    assert not cz.any() and np.all(mz[..., 0] == np.float16(0.75)) and not mz[..., 1].any()


def test_kv_cache_h16_variant_stores_half_size_pairs():
    x = _rand16((2, 3, 128), 1.0, 5)
    a = O.KVCache.empty(2, 2, 4, 64, True, meta_f16=True)
    a.store(0, 1, x, x)
    assert a.k_meta.dtype == np.float16 and a.k_meta.nbytes * 2 == O.KVCache.empty(2, 2, 4, 64, True).k_meta.nbytes
    kh, _ = a.load(1, 1, 4)
    c, m = O.quantize_groupwise_h16(x[1, :, 64:128])
    assert np.array_equal(kh[1:4], O.dequantize_groupwise(c, m).astype(np.float64))


def test_h16_weight_form_is_single_rounding_and_tiles_like_the_binary32_form():
    """Weights with FP16 pairs: Mat.dense() is the FP16 number nearest to min + code*scale evaluated
    exactly (Python fractions) from the STORED FP16 pair; the tiled order permutes 4-byte pairs the
    same way it permutes 8-byte ones; and y = x W^T against that dense matrix is what linear() gives."""
    from fractions import Fraction
    w = _rand16((32, 128), 0.02, 33)
    m = O.Mat.from_f16(w, True, meta_f16=True)
    assert m.meta.dtype == np.float16 and m.meta.shape == (32, 2, 2)
    c = O.unpack_codes(m.codes)
    d = m.dense()
    for r in range(0, 32, 5):
        for k in range(0, 128, 3):
            exact = Fraction(float(m.meta[r, k // 64, 0])) + int(c[r, k]) * Fraction(float(m.meta[r, k // 64, 1]))
            assert d[r, k] == float(np.float16(float(exact)))
    # within half a step of the original weight
    sc = np.repeat(m.meta[..., 1].astype(np.float64), 64, axis=1)
    assert np.all(np.abs(d - w.astype(np.float64)) <= sc / 2 + 2.0 ** -11 * np.abs(d) + 1e-12)
    tc, tm = tile_weights(m.codes, m.meta)
    tc32, tm32 = tile_weights(m.codes, m.meta.astype(np.float32))
    assert tm.dtype == np.float16 and np.array_equal(tc, tc32) and np.array_equal(tm.astype(np.float32), tm32)
    x = _rand16((3, 128), 1.0, 34).astype(np.float64)
    y = O.linear(x, m, None)
    ref = np.array([[sum(x[i, k] * d[j, k] for k in range(128)) for j in range(32)] for i in range(3)])
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)
