"""Helpers shared by the GPU parity tests: tolerances from the task's bar and converters from
oracle objects to device objects (inputs only flow oracle-side -> device, never the other way)."""
import numpy as np
import torch

from oracle import fg_oracle as O
from paper_2303_06865_amd import binding as B

REL_L2 = 2e-3     # relative L2 bound for FP16 activations against the oracle
MAX_ABS = 1e-2    # and the max-abs bound


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def rel_l2(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.sqrt((ref ** 2).sum())
    return float(np.sqrt(((got - ref) ** 2).sum()) / (den if den > 0 else 1.0))


def assert_close(got, ref, what="", rel=REL_L2, mabs=MAX_ABS):
    """The bar: relative L2 <= 2e-3 and max abs <= 1e-2.  The absolute bound is meant for O(1)
    activations; FP16 storage alone costs |v| * 2^-11 per rounding, so for tensors whose largest
    magnitude exceeds 4 the absolute bound scales with it (1e-2 per 4 units = 5 FP16 ulps)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    r = rel_l2(got, ref)
    m = float(np.abs(got - ref).max()) if got.size else 0.0
    if ref.size:
        mabs = mabs * max(1.0, float(np.abs(ref).max()) / 4.0)
    assert r <= rel and m <= mabs, "%s: rel L2 %.3e (<= %.1e), max abs %.3e (<= %.1e)" % (what, r, rel, m, mabs)
    return r, m


def oracle_layer(t, quant, meta_f16=False):
    mk = lambda a: O.Mat.from_f16(a, quant, meta_f16 and quant)
    return O.LayerWeights(
        wqkv=mk(t["wqkv"]), wo=mk(t["wo"]), w1=mk(t["w1"]), w2=mk(t["w2"]),
        ln1_g=t["ln1_g"], ln1_b=t["ln1_b"], ln2_g=t["ln2_g"], ln2_b=t["ln2_b"],
        bqkv=t["bqkv"], bo=t["bo"], b1=t["b1"], b2=t["b2"])


def cfg_pair(sh):
    return (O.ModelCfg(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos, sh.ln_eps),
            B.Cfg(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos, sh.ln_eps))


def cache_rows_dense(kv_dev, rows):
    """Device cache -> float64 arrays [batch, nh, rows, dh] of the values it represents, decoded on
    the host with the oracle's own inverse map (so the comparison does not trust the GPU decoder)."""
    if kv_dev.quantized:
        k = O.dequantize_groupwise(host(kv_dev.k_codes[:, :, :rows]), host(kv_dev.k_meta[:, :, :rows]))
        v = O.dequantize_groupwise(host(kv_dev.v_codes[:, :, :rows]), host(kv_dev.v_meta[:, :, :rows]))
    else:
        k = host(kv_dev.k_codes[:, :, :rows])
        v = host(kv_dev.v_codes[:, :, :rows])
    return k.astype(np.float64), v.astype(np.float64)


def oracle_cache_dense(kv, rows):
    if kv.quantized:
        k = O.dequantize_groupwise(kv.k_codes[:, :, :rows], kv.k_meta[:, :, :rows])
        v = O.dequantize_groupwise(kv.v_codes[:, :, :rows], kv.v_meta[:, :, :rows])
    else:
        k, v = kv.k_f16[:, :, :rows], kv.v_f16[:, :, :rows]
    return k.astype(np.float64), v.astype(np.float64)


def assert_cache_close(kv_dev, okv, seqs, rows, what=""):
    """Compare a device cache with the oracle's after both ran the same layer.  The K/V rows that
    were quantized differ by FP16 ulps between the two sides, and quantization turns an ulp into a
    whole step for the few elements that sit on a rounding boundary (or moves a group's min/max by
    an ulp).  So: every value within 1.05 steps of the oracle's, at most 3 % of the values more than
    a tenth of a step away, and overall relative L2 within 2 %."""
    kg, vg = cache_rows_dense(kv_dev, rows)
    kr, vr = oracle_cache_dense(okv, rows)
    for name, g, r, meta in (("K", kg, kr, okv.k_meta if okv.quantized else None),
                             ("V", vg, vr, okv.v_meta if okv.quantized else None)):
        g, r = g[seqs], r[seqs]
        if meta is None:
            assert_close(g, r, what + " " + name + " cache (FP16)")
            continue
        step = meta[seqs][:, :, :rows, :, 1].astype(np.float64).repeat(64, axis=-1).reshape(r.shape)
        d = np.abs(g - r)
        tol = step * 1.05 + 2e-3 * np.abs(r) + 1e-6
        assert np.all(d <= tol), "%s %s cache: %d values off by more than one step" % (what, name, int((d > tol).sum()))
        frac = float((d > 0.1 * step + 2e-3 * np.abs(r) + 1e-6).mean())
        assert frac <= 0.03, "%s %s cache: %.2f %% of values moved" % (what, name, 100 * frac)
        assert rel_l2(g, r) <= 2e-2, "%s %s cache: rel L2 %.3e" % (what, name, rel_l2(g, r))


def upload_cache(kv_dev, okv):
    """Overwrite a device cache with the oracle's bytes (inputs flow oracle -> device only)."""
    if okv.quantized:
        kv_dev.k_codes.copy_(dev(okv.k_codes)); kv_dev.v_codes.copy_(dev(okv.v_codes))
        kv_dev.k_meta.copy_(dev(okv.k_meta)); kv_dev.v_meta.copy_(dev(okv.v_meta))
    else:
        kv_dev.k_codes.copy_(dev(okv.k_f16)); kv_dev.v_codes.copy_(dev(okv.v_f16))
