"""Property tests (hypothesis) of the oracle on adversarial inputs: the quantizer's invariants on
groups with extreme dynamic range, repeated values, FP16 subnormals and the largest finite values;
algebraic properties of the Section 3 building blocks that a dropped term, a wrong axis or a
transposed operand would break.  CPU only, bounded example counts."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st
from hypothesis.extra import numpy as hnp

from oracle import fg_oracle as O

# the same examples on every run and machine: nothing random at test time, no example database
settings.register_profile("fixed", derandomize=True, database=None, deadline=None)
settings.load_profile("fixed")

F16 = st.floats(width=16, allow_nan=False, allow_infinity=False)
GROUPS = hnp.arrays(np.float16, (3, 128), elements=F16)
# a few values repeated many times, and mixtures of huge and tiny magnitudes
SPIKY = st.lists(st.sampled_from([0.0, -0.0, 6.1e-5, -6.1e-5, 5.96e-8, 1.0, -1.0, 1.0009765625, 65504.0, -65504.0,
                                  0.333251953125, 1024.0, -1023.5]), min_size=128, max_size=128).map(
    lambda v: np.array(v, np.float16).reshape(2, 64))


def _check_invariants(x, codes, meta, exact_max):
    rows, cols = x.shape
    c = O.unpack_codes(codes).reshape(rows, cols // 64, 64).astype(np.float64)
    xg = x.astype(np.float64).reshape(rows, cols // 64, 64)
    mn = meta[..., 0].astype(np.float64)[..., None]
    sc = meta[..., 1].astype(np.float64)[..., None]
    assert c.min() >= 0 and c.max() <= 15
    assert np.all(sc >= 0) and np.all(np.isfinite(sc)) and np.all(np.isfinite(mn))
    err = np.abs(xg - (mn + c * sc))
    assert np.all(err <= sc / 2 * (1 + 2.0 ** -20) + 1e-300)
    assert np.array_equal(mn[..., 0], xg.min(axis=2))                     # stored min is the true min
    assert np.all(np.take_along_axis(c, xg.argmin(axis=2)[..., None], 2) == 0)
    const = xg.max(axis=2) == xg.min(axis=2)
    assert np.all(sc[..., 0][const] == 0) and np.all(c[const] == 0)
    cmax = np.take_along_axis(c, xg.argmax(axis=2)[..., None], 2)[..., 0]
    if exact_max:
        assert np.all(cmax[~const] == 15)
    else:
        # FP16 pairs: the scale is rounded UP to an FP16 number, so the maximum maps to
        # round(range / scale) <= 15: 15 for scales with a full FP16 mantissa, less where the scale falls
        # into the FP16 subnormals (a range of one subnormal unit gives scale = range and code 1)
        normal = sc[..., 0] >= 2.0 ** -14
        assert np.all(cmax[~const & normal] == 15) and np.all(cmax[~const] >= 1)
    if exact_max:
        # The group maximum comes back as fp16(min + 15 * scale).  The binary32 scale carries a relative
        # error of 2^-24, so the sum is off by up to range * 2^-24 (plus its own rounding): the maximum
        # round-trips EXACTLY whenever that is below half an FP16 ulp of it, i.e. unless the maximum is
        # tiny against the range (|max| < range * 2^-12, e.g. a group of negative values whose
        # maximum is 0); then it is still within range * 2^-22 of the true value.
        w = O.dequantize_groupwise_f16(codes, meta).reshape(xg.shape).astype(np.float64)
        wmax = np.take_along_axis(w, xg.argmax(axis=2)[..., None], 2)[..., 0]
        mx, rng_ = xg.max(axis=2), xg.max(axis=2) - xg.min(axis=2)
        safe = np.abs(mx) >= rng_ * 2.0 ** -12
        assert np.array_equal(wmax[safe], mx[safe])
        assert np.all(np.abs(wmax - mx) <= rng_ * 2.0 ** -22)


@settings(max_examples=150, deadline=None)
@given(GROUPS)
def test_quantizer_invariants_on_arbitrary_finite_fp16(x):
    codes, meta = O.quantize_groupwise(x)
    _check_invariants(x, codes, meta, exact_max=True)
    assert np.array_equal(O.pack_codes(O.unpack_codes(codes)), codes)


@settings(max_examples=100, deadline=None)
@given(SPIKY)
def test_quantizer_invariants_on_spiky_groups(x):
    codes, meta = O.quantize_groupwise(x)
    _check_invariants(x, codes, meta, exact_max=True)


@settings(max_examples=150, deadline=None)
@given(GROUPS)
def test_fp16_pair_quantizer_invariants_on_arbitrary_finite_fp16(x):
    # a range beyond 15 * 65504 has no FP16 scale: such groups are outside the variant's domain
    r = x.astype(np.float64).reshape(3, 2, 64)
    if np.any((r.max(axis=2) - r.min(axis=2)) / 15.0 > 65504.0):
        return
    codes, meta = O.quantize_groupwise_h16(x)
    assert meta.dtype == np.float16
    _check_invariants(x, codes, meta, exact_max=False)
    # the stored scale is the smallest FP16 number not below (max - min) / 15 (binary32 quotient)
    q = ((r.max(axis=2) - r.min(axis=2)).astype(np.float32) / np.float32(15)).astype(np.float32)
    s = meta[..., 1].astype(np.float32)
    assert np.all(s >= q)
    below = np.nextafter(meta[..., 1], np.float16(-np.inf)).astype(np.float32)
    assert np.all((below < q) | (s == 0))


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 40), st.integers(0, 2 ** 31 - 1))
def test_decode_attention_algebra(rows, seed):
    rng = np.random.default_rng(seed)
    dh = 64
    q = rng.standard_normal(dh)
    k = rng.standard_normal((rows, dh))
    v = rng.standard_normal((rows, dh))
    out = O.attn_decode(q, k, v)
    # a weighted mean of the value rows: inside their range in every dimension
    assert np.all(out <= v.max(axis=0) + 1e-12) and np.all(out >= v.min(axis=0) - 1e-12)
    # the rows are a set: any common permutation of K and V rows gives the same output
    p = rng.permutation(rows)
    assert np.allclose(O.attn_decode(q, k[p], v[p]), out, rtol=0, atol=1e-12)
    # adding a multiple of one vector to every key shifts all scores alike: softmax unchanged
    assert np.allclose(O.attn_decode(q, k + rng.standard_normal(dh)[None, :], v), out, rtol=0, atol=1e-9)
    # V enters linearly
    v2 = rng.standard_normal((rows, dh))
    assert np.allclose(O.attn_decode(q, k, 2.0 * v - 3.0 * v2), 2.0 * out - 3.0 * O.attn_decode(q, k, v2), atol=1e-11)
    # repeating every row leaves the output unchanged (weights halve, rows double)
    assert np.allclose(O.attn_decode(q, np.repeat(k, 2, axis=0), np.repeat(v, 2, axis=0)), out, atol=1e-12)


@settings(max_examples=40, deadline=None)
@given(st.integers(2, 24), st.integers(0, 2 ** 31 - 1))
def test_prefill_attention_rows_are_decode_attention_over_their_prefix(s, seed):
    rng = np.random.default_rng(seed)
    dh = 64
    q, k, v = (rng.standard_normal((s, dh)) for _ in range(3))
    full = O.attn_prefill(q, k, v)
    for i in (0, s // 2, s - 1):
        assert np.allclose(full[i], O.attn_decode(q[i], k[:i + 1], v[:i + 1]), atol=1e-12)
    # the future does not leak: changing later keys and values leaves earlier rows alone
    k2, v2 = k.copy(), v.copy()
    k2[s // 2 + 1:] += 5.0
    v2[s // 2 + 1:] -= 7.0
    assert np.array_equal(O.attn_prefill(q, k2, v2)[:s // 2 + 1], full[:s // 2 + 1])


@settings(max_examples=40, deadline=None)
@given(st.integers(0, 2 ** 31 - 1), st.floats(1.0, 8.0), st.floats(-4.0, 4.0))
def test_layernorm_and_linear_algebra(seed, a, b):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((3, 128))
    g = rng.standard_normal(128).astype(np.float16)
    be = rng.standard_normal(128).astype(np.float16)
    y = O.layernorm(x, g, be, 1e-5)
    # invariant under a positive affine map of the row (up to the epsilon under the root)
    assert np.allclose(O.layernorm(a * x + b, g, be, 1e-5), y, atol=2e-4)
    # beta shifts, gamma scales
    assert np.allclose(O.layernorm(x, g, np.zeros(128, np.float16), 1e-5) + be.astype(np.float64)[None, :], y, atol=1e-12)
    w16 = (rng.standard_normal((32, 128)) * 0.05).astype(np.float16)
    for quant in (False, True):
        m = O.Mat.from_f16(w16, quant)
        x2 = rng.standard_normal((3, 128))
        assert np.allclose(O.linear(2.0 * x - x2, m, None), 2.0 * O.linear(x, m, None) - O.linear(x2, m, None), atol=1e-10)
        bias = rng.standard_normal(32).astype(np.float16)
        assert np.allclose(O.linear(x, m, bias), O.linear(x, m, None) + bias.astype(np.float64)[None, :], atol=1e-12)
        # [out, in] orientation: output j depends on row j of W only
        assert np.allclose(O.linear(x, m, None)[:, 5], x @ m.dense()[5], atol=1e-12)


def test_group_maximum_near_zero_does_not_round_trip_exactly():
    """The one case where the format cannot return the group maximum exactly: min = -1, max = 0 gives
    scale = fl32(1/15), and -1 + 15 * fl32(1/15) = 2^-24 * 0.87..., which is nearer to the smallest FP16
    subnormal than to 0.  Stated here so that nobody mistakes it for a kernel bug: both sides must
    return 2^-24 for that element, bit for bit."""
    x = np.full((1, 64), -1.0, np.float16)
    x[0, 0] = 0.0
    codes, meta = O.quantize_groupwise(x)
    assert O.unpack_codes(codes)[0, 0] == 15 and meta[0, 0, 0] == -1.0
    assert meta[0, 0, 1] == np.float32(1.0) / np.float32(15.0)
    w = O.dequantize_groupwise_f16(codes, meta)
    assert w[0, 0] == np.float16(2.0 ** -24) and np.all(w[0, 1:] == np.float16(-1.0))
    # with the maximum an FP16 ulp or more above the danger zone it is exact again
    x[0, 0] = 2.0 ** -10
    codes, meta = O.quantize_groupwise(x)
    assert O.dequantize_groupwise_f16(codes, meta)[0, 0] == np.float16(2.0 ** -10)
