"""Parity at the benchmark's full sizes, in the launch configurations bench.py times (same kernel
templates, grids and stream-K splits).  The oracle cannot compute a whole 144 x 36864 x 12288 product
in seconds, so these tests check SAMPLED outputs one by one: output columns (weight rows) and
activation rows are drawn at tile and block boundaries and at random, the oracle quantizes exactly
those weight rows itself, its codes must equal the device's bit for bit, and its FP64 dot products
bound the device outputs with the usual tolerance.  Bulk operands are drawn on the device with a
seeded generator (they are inputs, not results); everything the oracle consumes is copied from
those inputs, never from a kernel's output."""
import numpy as np
import pytest
import torch

from oracle import fg_oracle as O
from paper_2303_06865_amd import binding as B
from tests.util import assert_close, host

pytestmark = pytest.mark.gpu


def _gen(shape, std, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.empty(shape, dtype=torch.float16, device="cuda").normal_(0.0, std, generator=g)


def _sample(n, edges, k, seed):
    rng = np.random.default_rng(seed)
    pts = {0, n - 1}
    for e in edges:
        for d in (-1, 0):
            if 0 <= e + d < n:
                pts.add(e + d)
    pts.update(int(v) for v in rng.integers(0, n, size=k))
    return np.array(sorted(pts), dtype=np.int64)


# (rows, out features, in features, quantized): the four projection shapes of the OPT-175B workload in
# the decode phase (144 rows) and in the prefill phase (36 x 512 rows), the FP16 LM head, and (below) the
# uncompressed workload's shapes
FULL_LINEAR = [
    (144, 36864, 12288, True),
    (144, 12288, 49152, True),
    (144, 49152, 12288, True),
    (18432, 36864, 12288, True),
    (18432, 12288, 49152, True),
    (144, 50272, 12288, False),
    (144, 36864, 12288, "h16"),      # 4-bit weights with FP16 {min, scale} pairs
    (18432, 12288, 49152, "h16"),
    # the uncompressed workload (OPT-6.7B, FP16 weights, 4 x 32 sequences): decode projections (128 rows:
    # whole tiles of 48, 16 and 64 columns, and 64-column tiles split along K) and two prefill projections
    (128, 12288, 4096, False),
    (128, 4096, 4096, False),
    (128, 16384, 4096, False),
    (128, 4096, 16384, False),
    (16384, 12288, 4096, False),
    (16384, 4096, 16384, False),
]


@pytest.mark.parametrize("m,n,k,quant", FULL_LINEAR)
def test_linear_full_size_sampled(m, n, k, quant):
    w = _gen((n, k), 0.02, 1000 + n % 97 + k % 89)
    x = _gen((m, k), 1.0, 2000 + m)
    res = _gen((m, n), 1.0, 3000 + m)
    bias = _gen((n,), 0.5, 4000)
    h16 = quant == "h16"
    quant = bool(quant)
    wm = B.Mat.from_f16(w, quant, tiled=quant, meta_f16=h16)
    out = B.fg_linear(wm, bias, x, res, False)
    torch.cuda.synchronize()

    cols = _sample(n, [255, 256, 32 * 1151, n - 256, n // 2], 24, n + k)
    rows = _sample(m, [31, 32, 159, 160, 255, 256, m // 2, m - 33], 24, m + k) if m > 160 else np.arange(m)
    w_rows = host(w[torch.from_numpy(cols).cuda()])
    om = O.Mat.from_f16(w_rows, quant, h16)
    if quant:   # the device quantized the very same rows to the very same bytes (checked on the canonical form)
        canon = B.Mat.from_f16(w[torch.from_numpy(cols).cuda()].contiguous(), True, meta_f16=h16)
        bits = np.uint16 if h16 else np.uint32
        assert np.array_equal(host(canon.data), om.codes)
        assert np.array_equal(host(canon.meta).view(bits), om.meta.view(bits))
    ti = torch.from_numpy(rows).cuda()
    tj = torch.from_numpy(cols).cuda()
    x_s = host(x[ti]).astype(np.float64)
    y = x_s @ om.dense().T + host(bias[tj]).astype(np.float64)[None, :]
    y = y + host(res[ti][:, tj]).astype(np.float64)
    got = host(out[ti][:, tj])
    assert_close(got, O.round_f16(y), "full-size linear m=%d n=%d k=%d q=%s" % (m, n, k, quant))


@pytest.mark.parametrize("b,rows", [(144, 528), (144, 543)])
def test_decode_attention_full_size_sampled(b, rows):
    """OPT-175B decode attention launch (144 x 96 heads, 4-bit cache).  The cache is filled with
    arbitrary bytes on the device; the sampled (sequence, head) streams are then overwritten with rows
    the oracle quantized, and only those heads are compared."""
    nh, dh = 96, 128
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 50272, 4096)
    cap = rows + 5
    kv = B.KVCache(cfg, b, cap, True, zero=False)
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    kv.k_codes.random_(0, 256, generator=g)
    kv.v_codes.random_(0, 256, generator=g)
    kv.k_meta.normal_(0.0, 0.3, generator=g).abs_()
    kv.v_meta.normal_(0.0, 0.3, generator=g).abs_()
    q = _gen((b, 3 * h1), 1.0, 7)
    rng = np.random.default_rng(rows)
    pairs = [(0, 0), (b - 1, nh - 1), (b // 2, 37)] + [(int(rng.integers(0, b)), int(rng.integers(0, nh))) for _ in range(9)]
    refs = []
    for (si, hi) in pairs:
        k16 = (rng.standard_normal((1, rows, dh))).astype(np.float16)
        v16 = (rng.standard_normal((1, rows, dh))).astype(np.float16)
        okv = O.KVCache.empty(1, 1, cap, dh, True)
        okv.store(0, 0, k16, v16)
        kv.k_codes[si, hi].copy_(torch.from_numpy(okv.k_codes[0, 0]).cuda())
        kv.v_codes[si, hi].copy_(torch.from_numpy(okv.v_codes[0, 0]).cuda())
        kv.k_meta[si, hi].copy_(torch.from_numpy(okv.k_meta[0, 0]).cuda())
        kv.v_meta[si, hi].copy_(torch.from_numpy(okv.v_meta[0, 0]).cuda())
        kh, vh = okv.load(0, 0, rows)
        qv = host(q[si, hi * dh:(hi + 1) * dh]).astype(np.float64)
        refs.append(O.attn_decode(qv, kh, vh))
    out = B.fg_decode_attention(cfg, q, 3 * h1, b, rows, kv, 0)
    torch.cuda.synchronize()
    got = np.stack([host(out[si, hi * dh:(hi + 1) * dh]) for (si, hi) in pairs])
    assert_close(got, O.round_f16(np.stack(refs)), "full-size decode attention rows=%d" % rows)
    assert bool(torch.isfinite(out.float()).all())


def test_prefill_attention_full_size_sampled():
    """One GPU batch of the OPT-175B workload (36 sequences x 96 heads x 512 positions): the launch
    bench.py times (persistent workgroups, 128-query items).  Sampled (sequence, head) pairs are
    computed whole by the oracle from the same FP16 q, k, v."""
    b, s, nh, dh = 36, 512, 96, 128
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 50272, 4096)
    qkv = _gen((b * s, 3 * h1), 1.0, 11)
    out = B.fg_prefill_attention(cfg, qkv, b, s)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    pairs = [(0, 0), (b - 1, nh - 1), (17, 40)] + [(int(rng.integers(0, b)), int(rng.integers(0, nh))) for _ in range(5)]
    for (si, hi) in pairs:
        blk = host(qkv[si * s:(si + 1) * s]).astype(np.float64)
        q, k, v = (blk[:, j * h1 + hi * dh: j * h1 + (hi + 1) * dh] for j in range(3))
        ref = O.round_f16(O.attn_prefill(q, k, v))
        got = host(out[si * s:(si + 1) * s, hi * dh:(hi + 1) * dh])
        assert_close(got, ref, "full-size prefill attention seq %d head %d" % (si, hi))
    assert bool(torch.isfinite(out.float()).all())


def test_layernorm_full_size_sampled():
    rows, cols = 18432, 12288
    x = _gen((rows, cols), 3.0, 21) + 0.5
    g = _gen((cols,), 0.1, 22) + 1.0
    be = _gen((cols,), 0.1, 23)
    out = B.fg_layernorm(x, g, be, 1e-5)
    torch.cuda.synchronize()
    idx = _sample(rows, [255, 256, rows // 2], 12, 3)
    ti = torch.from_numpy(idx).cuda()
    ref = O.round_f16(O.layernorm(host(x[ti]), host(g), host(be), 1e-5))
    assert_close(host(out[ti]), ref, "full-size layernorm", rel=5e-4, mabs=4e-3)


@pytest.mark.parametrize("meta_f16", [False, True])
def test_kv_append_full_size_sampled_bit_exact(meta_f16):
    """The prefill append of one GPU batch of the OPT-175B workload (36 x 512 rows x 12288): sampled
    (sequence, head) streams must hold exactly the oracle's codes and pairs."""
    b, s, nh, dh = 36, 512, 96, 128
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 50272, 4096)
    qkv = _gen((b * s, 3 * h1), 1.0, 31)
    kv = B.KVCache(cfg, b, s + 4, True, zero=False, meta_f16=meta_f16)
    B.fg_kv_append(cfg, qkv[:, h1:], qkv[:, 2 * h1:], 3 * h1, b, s, kv, 0, 0)
    torch.cuda.synchronize()
    quant = O.quantize_groupwise_h16 if meta_f16 else O.quantize_groupwise
    bits = np.uint16 if meta_f16 else np.uint32
    rng = np.random.default_rng(6)
    pairs = [(0, 0), (b - 1, nh - 1)] + [(int(rng.integers(0, b)), int(rng.integers(0, nh))) for _ in range(6)]
    for (si, hi) in pairs:
        for j, (codes_dev, meta_dev) in enumerate(((kv.k_codes, kv.k_meta), (kv.v_codes, kv.v_meta))):
            rows16 = host(qkv[si * s:(si + 1) * s, (j + 1) * h1 + hi * dh:(j + 1) * h1 + (hi + 1) * dh]).copy()
            codes, meta = quant(rows16)
            assert np.array_equal(host(codes_dev[si, hi, :s]), codes)
            assert np.array_equal(host(meta_dev[si, hi, :s]).view(bits), meta.reshape(s, dh // 64, 2).view(bits))
