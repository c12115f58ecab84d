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
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    r = rel_l2(got, ref)
    m = float(np.abs(got - ref).max()) if got.size else 0.0
    assert r <= rel and m <= mabs, "%s: rel L2 %.3e (<= %.1e), max abs %.3e (<= %.1e)" % (what, r, rel, m, mabs)
    return r, m


def oracle_layer(t, quant):
    return O.LayerWeights(
        wqkv=O.Mat.from_f16(t["wqkv"], quant), wo=O.Mat.from_f16(t["wo"], quant),
        w1=O.Mat.from_f16(t["w1"], quant), w2=O.Mat.from_f16(t["w2"], quant),
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
