"""Pins for the oracle's layer pieces (Section 3): textbook closed forms, brute
force in pure Python on tiny inputs, library routines, and identities that any
correct implementation satisfies."""
import math

import numpy as np
import pytest
import torch

from oracle import fg_oracle as O
from paper_2303_06865_amd import synth


def _r(shape, std, seed):
    return np.random.default_rng(seed).standard_normal(shape) * std


# ---------------------------------------------------------------- LayerNorm
def test_layernorm_closed_forms():
    g = np.full(8, 2.0)
    b = np.full(8, 0.5)
    # constant row: zero variance -> output is beta
    y = O.layernorm(np.full((1, 8), 3.0), g, b, 1e-5)
    assert np.allclose(y, 0.5, atol=1e-12)
    # two-valued row (+a, -a alternating): mean 0, var a^2 -> +-gamma*a/sqrt(a^2+eps)+beta
    a = 0.25
    x = np.array([[a, -a] * 4])
    y = O.layernorm(x, g, b, 1e-5)
    e = 2.0 * a / math.sqrt(a * a + 1e-5)
    assert np.allclose(y[0, 0::2], e + 0.5, atol=1e-12) and np.allclose(y[0, 1::2], -e + 0.5, atol=1e-12)


def test_layernorm_matches_library():
    x = _r((5, 768), 3.0, 1) + 0.7
    g = 1 + _r(768, 0.1, 2)
    b = _r(768, 0.1, 3)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (768,), torch.from_numpy(g), torch.from_numpy(b), 1e-5)
    assert np.allclose(O.layernorm(x, g, b, 1e-5), ref.numpy(), rtol=0, atol=1e-11)


# ------------------------------------------------------------------- linear
def test_linear_bruteforce_and_special_cases():
    w16 = (_r((6, 128), 0.5, 4)).astype(np.float16)
    x = _r((3, 128), 1.0, 5)
    bias = _r(6, 1.0, 6)
    for quant in (False, True):
        m = O.Mat.from_f16(w16, quant)
        w = m.dense()
        if quant:
            codes, meta = O.quantize_groupwise(w16)
            c = O.unpack_codes(codes)
            for r in range(6):          # dequantized matrix element by element, plain Python
                for k in range(128):
                    mn, sc = float(meta[r, k // 64, 0]), float(meta[r, k // 64, 1])
                    ref = mn + int(c[r, k]) * sc
                    assert w[r, k] == float(np.float16(ref))          # the FP16 number nearest to it
            half_ulp = np.abs(w16.astype(np.float64)) * 2.0 ** -11 + 2.0 ** -25
            assert np.all(np.abs(w - w16.astype(np.float64)) <= meta[..., 1].repeat(64, axis=1) / 2 * (1 + 1e-6) + half_ulp)
        y = O.linear(x, m, bias)
        for i in range(3):
            for r in range(6):
                ref = math.fsum(float(x[i, k]) * float(w[r, k]) for k in range(128)) + bias[r]
                assert abs(y[i, r] - ref) < 1e-10
    # one-hot input picks a column of W (transposition check: W is [out, in])
    m = O.Mat.from_f16(w16, False)
    e = np.zeros((1, 128))
    e[0, 17] = 1.0
    assert np.allclose(O.linear(e, m, None)[0], w16[:, 17].astype(np.float64))
    # identity weight
    eye = O.Mat.from_f16(np.eye(64, dtype=np.float16), False)
    xx = _r((2, 64), 1.0, 7)
    assert np.allclose(O.linear(xx, eye, None), xx)


# ---------------------------------------------------------------- attention
def _attn_python(q, k, v):
    """softmax(q.K^T/sqrt(dh)).V for one query with Python floats only."""
    dh = len(q)
    s = [sum(q[d] * k[j][d] for d in range(dh)) / math.sqrt(dh) for j in range(len(k))]
    m = max(s)
    e = [math.exp(si - m) for si in s]
    z = sum(e)
    return [sum(e[j] / z * v[j][d] for j in range(len(k))) for d in range(dh)]


def test_decode_attention_bruteforce_tiny_head():
    q = _r(8, 1.0, 8)
    k = _r((5, 8), 1.0, 9)
    v = _r((5, 8), 1.0, 10)
    ref = _attn_python(q.tolist(), k.tolist(), v.tolist())
    assert np.allclose(O.attn_decode(q, k, v), ref, atol=1e-13)


def test_decode_attention_special_cases():
    q = _r(64, 1.0, 11)
    v = _r((9, 64), 1.0, 12)
    # all keys equal -> uniform weights -> mean of V
    k = np.tile(_r((1, 64), 1.0, 13), (9, 1))
    assert np.allclose(O.attn_decode(q, k, v), v.mean(axis=0), atol=1e-12)
    # one dominant key -> that V row
    k = _r((9, 64), 0.01, 14)
    k[4] = q * 50.0
    assert np.allclose(O.attn_decode(q, k, v), v[4], atol=1e-9)
    # single cached row -> that V row exactly
    assert np.allclose(O.attn_decode(q, k[:1], v[:1]), v[0], atol=1e-15)


def test_topk_sparse_attention_pins():
    """Top-K sparse attention (Section 5): brute force in pure Python, the dense limit, a dominant
    key, the tie rule, and the monotone kept mass."""
    q = _r(16, 1.0, 40)
    k = _r((23, 16), 1.0, 41)
    v = _r((23, 16), 1.0, 42)
    # brute force: full softmax in pure Python, keep the 5 largest weights, drop the rest
    s = [sum(a * b for a, b in zip(row, q.tolist())) / 4.0 for row in k.tolist()]
    mx = max(s)
    e = [math.exp(x - mx) for x in s]
    den = sum(e)
    order = sorted(range(23), key=lambda i: (-s[i], i))[:5]
    ref = [sum(e[i] / den * v[i, d] for i in order) for d in range(16)]
    out, idx = O.attn_decode_topk(q, k, v, 5)
    assert sorted(order) == idx.tolist()
    assert np.allclose(out, ref, atol=1e-13)
    # keeping every row is dense attention
    out_all, idx_all = O.attn_decode_topk(q, k, v, 23)
    assert idx_all.tolist() == list(range(23))
    assert np.allclose(out_all, O.attn_decode(q, k, v), atol=1e-14)
    # one dominant key: keeping a single row returns (almost exactly) its V row
    k2 = _r((23, 16), 0.01, 43)
    k2[7] = q * 40.0
    out1, idx1 = O.attn_decode_topk(q, k2, v, 1)
    assert idx1.tolist() == [7] and np.allclose(out1, v[7], atol=1e-9)
    # equal scores: the lowest indices are kept
    k3 = np.tile(_r((1, 16), 1.0, 44), (9, 1))
    _, idx3 = O.attn_decode_topk(q, k3, v[:9], 4)
    assert idx3.tolist() == [0, 1, 2, 3]
    # the weights are those of the FULL softmax (no renormalisation): uniform weights 1/9 each
    out3 = O.attn_decode_subset(q, k3, v[:9], np.array([0, 1, 2, 3]))
    assert np.allclose(out3, v[:4].sum(axis=0) / 9.0, atol=1e-13)
    # the kept probability mass grows with k and reaches 1
    p = O.softmax_rows(O.attn_decode_scores(q, k)[None, :])[0]
    masses = [p[O.topk_indices(O.attn_decode_scores(q, k), kk)].sum() for kk in range(1, 24)]
    assert all(b >= a for a, b in zip(masses, masses[1:])) and abs(masses[-1] - 1.0) < 1e-14
    # and the kept set is optimal: no dropped row outweighs a kept one
    kept = set(idx.tolist())
    assert min(p[i] for i in kept) >= max(p[i] for i in range(23) if i not in kept)


def test_decode_attention_split_merge_invariance():
    """Attention over rows [0,n) equals the log-sum-exp merge of attention over
    any two-way split of the rows."""
    q = _r(64, 1.0, 15)
    k = _r((40, 64), 1.0, 16)
    v = _r((40, 64), 1.0, 17)
    full = O.attn_decode(q, k, v)
    for cut in (1, 13, 39):
        parts = []
        for sl in (slice(0, cut), slice(cut, 40)):
            s = (k[sl] @ q) / 8.0
            parts.append((s.max(), np.exp(s - s.max()).sum(), O.attn_decode(q, k[sl], v[sl])))
        m = max(p[0] for p in parts)
        wts = [p[1] * math.exp(p[0] - m) for p in parts]
        merged = sum(w * p[2] for w, p in zip(wts, parts)) / sum(wts)
        assert np.allclose(full, merged, atol=1e-12)


def test_prefill_attention_causal_against_decode_and_library():
    q = _r((7, 16), 1.0, 18)
    k = _r((7, 16), 1.0, 19)
    v = _r((7, 16), 1.0, 20)
    o = O.attn_prefill(q, k, v)
    for i in range(7):                      # row i = one decode query over rows 0..i
        assert np.allclose(o[i], _attn_python(q[i].tolist(), k[:i + 1].tolist(), v[:i + 1].tolist()), atol=1e-13)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None], is_causal=True)[0]
    assert np.allclose(o, ref.numpy(), atol=1e-12)


# ------------------------------------------------------------ KV cache store
def test_kv_cache_layout_and_quantization_axis():
    """Stored rows come back within scale/2; groups run along the hidden
    dimension of a token row and never straddle a head (dh % 64 == 0)."""
    nh, dh = 3, 128
    kv = O.KVCache.empty(2, nh, 10, dh, True)
    k16 = _r((2, 4, nh * dh), 1.0, 21).astype(np.float16)
    v16 = _r((2, 4, nh * dh), 1.0, 22).astype(np.float16)
    kv.store(0, 3, k16, v16)
    for b in range(2):
        for h in range(nh):
            kh, vh = kv.load(b, h, 7)
            assert np.all(kh[:3] == 0) and np.all(vh[:3] == 0)
            ref = k16[b, :, h * dh:(h + 1) * dh].astype(np.float64)
            sc = kv.k_meta[b, h, 3:7, :, 1].astype(np.float64).repeat(64, axis=1)
            assert np.all(np.abs(kh[3:7] - ref) <= sc / 2 * (1 + 1e-6))
            # the same bytes as quantizing that head's slice on its own
            c, m = O.quantize_groupwise(np.ascontiguousarray(k16[b, :, h * dh:(h + 1) * dh]))
            assert np.array_equal(c, kv.k_codes[b, h, 3:7]) and np.array_equal(m, kv.k_meta[b, h, 3:7])
    kvf = O.KVCache.empty(2, nh, 10, dh, False)
    kvf.store(0, 3, k16, v16)
    kh, vh = kvf.load(1, 2, 7)
    assert np.array_equal(vh[3:7], v16[1, :, 2 * dh:3 * dh].astype(np.float64))


# ------------------------------------------------------------------ layers
def _tiny_layer(quant, seed=0, biases=True):
    sh = synth.Shape(h1=128, nh=2, h2=256, vocab=97, max_pos=32, l=1)
    t = synth.layer_tensors(sh, seed, 0, std=0.05, biases=biases, random_ln=True)
    w = O.LayerWeights(
        wqkv=O.Mat.from_f16(t["wqkv"], quant), wo=O.Mat.from_f16(t["wo"], quant),
        w1=O.Mat.from_f16(t["w1"], quant), w2=O.Mat.from_f16(t["w2"], quant),
        ln1_g=t["ln1_g"], ln1_b=t["ln1_b"], ln2_g=t["ln2_g"], ln2_b=t["ln2_b"],
        bqkv=t["bqkv"], bo=t["bo"], b1=t["b1"], b2=t["b2"])
    cfg = O.ModelCfg(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos)
    return sh, cfg, w


def _torch_layer_f64(cfg, w, x, causal_rows):
    """The layer equations with torch float64 library ops and no intermediate
    FP16 rounding; x is [b, s, h1]."""
    F = torch.nn.functional
    T = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    b, s, h1 = x.shape
    xx = T(x)
    y = F.layer_norm(xx, (h1,), T(w.ln1_g), T(w.ln1_b), cfg.ln_eps)
    qkv = F.linear(y, T(w.wqkv.dense()), T(w.bqkv))
    q, k, v = [t.reshape(b, s, cfg.nh, cfg.dh).transpose(1, 2) for t in qkv.split(h1, dim=-1)]
    o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(b, s, h1)
    x1 = F.linear(o, T(w.wo.dense()), T(w.bo)) + xx
    y2 = F.layer_norm(x1, (h1,), T(w.ln2_g), T(w.ln2_b), cfg.ln_eps)
    return (F.linear(F.relu(F.linear(y2, T(w.w1.dense()), T(w.b1))), T(w.w2.dense()), T(w.b2)) + x1).numpy()


@pytest.mark.parametrize("quant", [False, True])
def test_prefill_layer_matches_library_composition(quant):
    sh, cfg, w = _tiny_layer(quant)
    x16 = synth.activations_f16((2, 6, sh.h1), 0.5, 3)
    kv = O.KVCache.empty(2, sh.nh, 8, sh.dh, quant)
    out = O.prefill_layer(cfg, w, x16, kv).astype(np.float64)
    ref = _torch_layer_f64(cfg, w, x16.astype(np.float64), True)
    # differences are only the FP16 roundings of stored activations
    assert np.sqrt(((out - ref) ** 2).sum() / (ref ** 2).sum()) < 1e-3
    assert np.abs(out - ref).max() < 5e-3


def test_prefill_then_decode_equals_longer_prefill_fp16_path():
    """FP16 weights and cache: prefill(s) followed by one decode step gives the
    last row of prefill(s+1), and leaves the same cache."""
    sh, cfg, w = _tiny_layer(False)
    x16 = synth.activations_f16((2, 7, sh.h1), 0.5, 4)
    kv_a = O.KVCache.empty(2, sh.nh, 8, sh.dh, False)
    full = O.prefill_layer(cfg, w, x16, kv_a)
    kv_b = O.KVCache.empty(2, sh.nh, 8, sh.dh, False)
    O.prefill_layer(cfg, w, x16[:, :6], kv_b)
    last = O.decode_layer(cfg, w, x16[:, 6], 6, kv_b)
    assert np.array_equal(kv_a.k_f16[:, :, :7], kv_b.k_f16[:, :, :7])
    assert np.array_equal(kv_a.v_f16[:, :, :7], kv_b.v_f16[:, :, :7])
    d = np.abs(full[:, 6].astype(np.float64) - last.astype(np.float64))
    assert d.max() <= 2e-3          # a couple of FP16 ulps from summation order


def test_quantized_decode_differs_from_fp16_cache_within_bound():
    """With a compressed cache the decode output differs from the FP16-cache one
    only through the stored rows: per-head output error <= sum_j p_j*scale_j/2,
    which is bounded by max scale / 2 of the V rows (plus the effect on p)."""
    sh, cfg, w = _tiny_layer(False)
    x16 = synth.activations_f16((2, 7, sh.h1), 0.5, 5)
    kvq = O.KVCache.empty(2, sh.nh, 8, sh.dh, True)
    kvf = O.KVCache.empty(2, sh.nh, 8, sh.dh, False)
    O.prefill_layer(cfg, w, x16[:, :6], kvq)
    O.prefill_layer(cfg, w, x16[:, :6], kvf)
    oq = O.decode_layer(cfg, w, x16[:, 6], 6, kvq).astype(np.float64)
    of = O.decode_layer(cfg, w, x16[:, 6], 6, kvf).astype(np.float64)
    assert not np.array_equal(oq, of)
    assert np.sqrt(((oq - of) ** 2).sum() / (of ** 2).sum()) < 0.08


def test_decode_attends_to_its_own_quantized_row():
    """t = 0: the only cached row is the new one, so the attention output is the
    dequantized new V row (not the FP16 one)."""
    sh, cfg, w = _tiny_layer(True, biases=False)
    x16 = synth.activations_f16((1, sh.h1), 0.5, 6)
    kv = O.KVCache.empty(1, sh.nh, 4, sh.dh, True)
    O.decode_layer(cfg, w, x16, 0, kv)
    # recompute v by hand and compare what the cache holds
    y = O.round_f16(O.layernorm(x16.astype(np.float64), w.ln1_g, w.ln1_b, cfg.ln_eps))
    v = O.round_f16(O.linear(y, w.wqkv, None))[:, 2 * sh.h1:].astype(np.float16)
    c, m = O.quantize_groupwise(v)
    assert np.array_equal(c.reshape(sh.nh, sh.dh // 2), kv.v_codes[0, :, 0])
    assert np.array_equal(m.reshape(sh.nh, sh.dh // 64, 2), kv.v_meta[0, :, 0])


def test_sequences_in_a_batch_are_independent():
    sh, cfg, w = _tiny_layer(True)
    x16 = synth.activations_f16((3, 5, sh.h1), 0.5, 7)
    kv = O.KVCache.empty(3, sh.nh, 8, sh.dh, True)
    all3 = O.prefill_layer(cfg, w, x16, kv)
    kv1 = O.KVCache.empty(3, sh.nh, 8, sh.dh, True)
    one = O.prefill_layer(cfg, w, x16[1:2], kv1, batch_offset=1)
    assert np.array_equal(all3[1:2], one)
    assert np.array_equal(kv.k_codes[1], kv1.k_codes[1]) and np.array_equal(kv.v_meta[1], kv1.v_meta[1])
