"""Layer-level parity (Section 3): fg_prefill_layer and fg_decode_layer against the oracle, on the
OPT-125m-shaped configuration (batch 4, prompt 32, 8 decode steps, seed 0) and on other shapes that
span head sizes, biases, FP16 storage and ragged sizes."""
import numpy as np
import pytest
import torch

from oracle import fg_oracle as O
from paper_2303_06865_amd import binding as B
from paper_2303_06865_amd import synth
import copy

from tests.util import (assert_cache_holds_rows, assert_close, assert_close_or_within_sensitivity, cache_rows_dense,
                        cfg_pair, dev, host, nudged_kv_rows, oracle_layer, upload_cache)

pytestmark = pytest.mark.gpu


def _device_kv_rows(cfg, w, t, x_rows):
    """The FP16 K and V rows the device computes for layer input x_rows [rows, h1]: LayerNorm and QKV
    projection through the library's own calls, i.e. the kernels and launch shapes the layer call uses."""
    y = B.fg_layernorm(dev(x_rows), dev(t["ln1_g"]), dev(t["ln1_b"]), cfg.ln_eps)
    qkv = B.fg_linear(w.wqkv, dev(t["bqkv"]), y)
    h1 = cfg.h1
    return qkv[:, h1:2 * h1], qkv[:, 2 * h1:]     # device tensors (column slices)


def _oracle_kv_rows(ocfg, ow, x_rows):
    y = O.round_f16(O.layernorm(x_rows.astype(np.float64), ow.ln1_g, ow.ln1_b, ocfg.ln_eps))
    qkv = O.round_f16(O.linear(y, ow.wqkv, ow.bqkv))
    h1 = ocfg.h1
    return qkv[:, h1:2 * h1], qkv[:, 2 * h1:]


def _run_layer_sequence(sh, quant_w, quant_kv, b, s, steps, seed, biases, random_ln, x_std=0.05, batch=None,
                        boff=0, tiled=False, meta_f16=False, w_meta_f16=False):
    """Prefill then `steps` decode steps on both sides, the decode inputs being fresh seeded
    activations (the same on both sides).  Outputs are compared under the activation tolerance.  The
    cache is checked strictly, in two halves: the device's FP16 K/V rows against the oracle's (activation
    tolerance), and the device cache against the library's standalone quantizer applied to the device's
    rows (bit for bit; that quantizer is bit-exact against the oracle in its own tests).
    Before every decode step the device cache is overwritten with the oracle's bytes, so each step
    starts from identical inputs."""
    ocfg, cfg = cfg_pair(sh)
    t = synth.layer_tensors(sh, seed, 0, std=0.02, biases=biases, random_ln=random_ln)
    ow = oracle_layer(t, quant_w, w_meta_f16)
    w = B.LayerWeights.from_numpy(t, quant_w, tiled=tiled, meta_f16=w_meta_f16)
    batch = batch or b
    cap = s + steps
    okv = O.KVCache.empty(batch, sh.nh, cap, sh.dh, quant_kv, meta_f16)
    kv = B.KVCache(cfg, batch, cap, quant_kv, meta_f16=meta_f16)
    x = synth.activations_f16((b, s, sh.h1), x_std, seed)
    ref = O.prefill_layer(ocfg, ow, x, okv, batch_offset=boff)
    got = B.fg_prefill_layer(cfg, w, dev(x), kv, batch_offset=boff)
    torch.cuda.synchronize()
    assert_close(host(got), ref, "prefill output")
    kg, vg = _device_kv_rows(cfg, w, t, x.reshape(b * s, sh.h1))
    kr, vr = _oracle_kv_rows(ocfg, ow, x.reshape(b * s, sh.h1))
    assert_close(host(kg), kr, "prefill K rows")
    assert_close(host(vg), vr, "prefill V rows")
    assert_cache_holds_rows(kv, kg, vg, b, s, boff, 0, "prefill")
    for i in range(steps):
        xt = synth.activations_f16((b, sh.h1), x_std, seed + 100 + i)
        upload_cache(kv, okv)
        okv_before = copy.deepcopy(okv) if quant_kv else None
        ref = O.decode_layer(ocfg, ow, xt, s + i, okv, batch_offset=boff)
        got = B.fg_decode_layer(cfg, w, dev(xt), s + i, kv, batch_offset=boff)
        torch.cuda.synchronize()
        if quant_kv:
            def alt():   # the oracle again, its new K/V row moved by FP16 ulps before it is quantized
                with nudged_kv_rows(seed + i):
                    return O.decode_layer(ocfg, ow, xt, s + i, okv_before, batch_offset=boff)
            assert_close_or_within_sensitivity(host(got), ref, alt, "decode step %d output (%d x %d, %d rows cached)" % (
                i, sh.h1, sh.h2, s + i))
        else:
            assert_close(host(got), ref, "decode step %d output" % i)
        kg, vg = _device_kv_rows(cfg, w, t, xt)
        kr, vr = _oracle_kv_rows(ocfg, ow, xt)
        assert_close(host(kg), kr, "decode step %d K row" % i)
        assert_close(host(vg), vr, "decode step %d V row" % i)
        assert_cache_holds_rows(kv, kg, vg, b, 1, boff, s + i, "decode step %d" % i)
    if boff or batch > b:   # rows of other sequences stay untouched
        kg, vg = cache_rows_dense(kv, cap)
        untouched = [i for i in range(batch) if not (boff <= i < boff + b)]
        assert np.all(kg[untouched] == 0) and np.all(vg[untouched] == 0)


@pytest.mark.parametrize("tiled", [False, True])
def test_opt125m_layer_q4_batch4_prompt32_8steps(tiled):
    """The small parity configuration: hidden 768, 12 heads x 64, FFN 3072, weights ~N(0,0.02),
    LN gamma=1/beta=0, 4-bit weights and cache, batch 4, prompt 32, 8 decode steps, seed 0; with the
    weights in the canonical and in the streaming (tiled) order."""
    _run_layer_sequence(synth.OPT_125M_LAYER, True, True, b=4, s=32, steps=8, seed=0, biases=False,
                        random_ln=False, x_std=0.03, tiled=tiled)


@pytest.mark.parametrize("dh128", [False, True])
def test_layer_with_fp16_pair_cache(dh128):
    """The 4.5-bit cache variant (FP16 {min, scale} pairs) through prefill and decode."""
    if dh128:
        sh = synth.Shape(h1=512, nh=4, h2=1536, vocab=1000, max_pos=256)
        _run_layer_sequence(sh, True, True, b=3, s=70, steps=3, seed=4, biases=True, random_ln=True, x_std=0.5,
                            batch=4, boff=1, tiled=True, meta_f16=True)
    else:
        _run_layer_sequence(synth.OPT_125M_LAYER, True, True, b=4, s=32, steps=4, seed=3, biases=False,
                            random_ln=False, x_std=0.03, tiled=True, meta_f16=True)


@pytest.mark.parametrize("prefill_rows", [False, True])
def test_layer_with_fp16_pair_weights_and_cache(prefill_rows):
    """Weights AND cache in the 4.5-bit form (FP16 pairs), decode-shape and prefill-shape GEMM launches."""
    if prefill_rows:   # 4 x 96 = 384 rows: the 256-row prefill tile
        _run_layer_sequence(synth.OPT_125M_LAYER, True, True, b=4, s=96, steps=2, seed=6, biases=True,
                            random_ln=True, x_std=0.1, tiled=True, meta_f16=True, w_meta_f16=True)
    else:
        _run_layer_sequence(synth.OPT_125M_LAYER, True, True, b=4, s=32, steps=4, seed=5, biases=False,
                            random_ln=False, x_std=0.03, tiled=True, meta_f16=True, w_meta_f16=True)


@pytest.mark.parametrize("quant_w,quant_kv", [(False, False), (True, False), (False, True)])
def test_opt125m_layer_storage_variants(quant_w, quant_kv):
    _run_layer_sequence(synth.OPT_125M_LAYER, quant_w, quant_kv, b=4, s=32, steps=3, seed=1, biases=True,
                        random_ln=True)


@pytest.mark.parametrize("quant", [True, False])
def test_layer_head128_ragged_sizes_and_offset(quant):
    sh = synth.Shape(h1=512, nh=4, h2=1536, vocab=1000, max_pos=256)
    _run_layer_sequence(sh, quant, quant, b=3, s=70, steps=3, seed=2, biases=True, random_ln=True, x_std=0.5,
                        batch=5, boff=2)


def test_layer_large_m_prefill_path():
    """b*s = 660 rows takes the large-M GEMM kernel in prefill; decode then uses the small-M one."""
    sh = synth.Shape(h1=256, nh=2, h2=1024, vocab=1000, max_pos=512)
    _run_layer_sequence(sh, True, True, b=5, s=132, steps=2, seed=3, biases=True, random_ln=True, x_std=0.5)
    _run_layer_sequence(sh, True, True, b=5, s=132, steps=2, seed=3, biases=True, random_ln=True, x_std=0.5,
                        tiled=True)


def test_layer_6_7b_shape_slice():
    """Real width of OPT-6.7B (hidden 4096, 32 heads x 128, FFN 16384), two sequences."""
    sh = synth.Shape(h1=4096, nh=32, h2=16384, vocab=1000, max_pos=64)
    _run_layer_sequence(sh, True, True, b=2, s=20, steps=2, seed=4, biases=False, random_ln=False, x_std=0.5,
                        tiled=True)


def test_prefill_then_decode_consistency_on_gpu_fp16():
    """FP16 path: prefill(s) + decode(1) reproduces the last row of prefill(s+1) (Section 3)."""
    sh = synth.Shape(h1=256, nh=4, h2=512, vocab=1000, max_pos=64)
    ocfg, cfg = cfg_pair(sh)
    t = synth.layer_tensors(sh, 5, 0, biases=True, random_ln=True)
    w = B.LayerWeights.from_numpy(t, False)
    x = synth.activations_f16((2, 9, sh.h1), 0.5, 5)
    kva = B.KVCache(cfg, 2, 12, False)
    full = host(B.fg_prefill_layer(cfg, w, dev(x), kva))
    kvb = B.KVCache(cfg, 2, 12, False)
    B.fg_prefill_layer(cfg, w, dev(np.ascontiguousarray(x[:, :8])), kvb)
    last = host(B.fg_decode_layer(cfg, w, dev(np.ascontiguousarray(x[:, 8])), 8, kvb))
    assert np.array_equal(host(kva.k_codes[:, :, :9]), host(kvb.k_codes[:, :, :9]))
    assert_close(last, full[:, 8], "prefill vs decode", rel=1e-3, mabs=5e-3)
