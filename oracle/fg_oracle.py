"""CPU oracle for the 4-bit group-wise OPT generation path (FlexGen, arXiv 2303.06865).

TEST INFRASTRUCTURE ONLY.  This module is the plain, slow, obviously-correct
definition the HIP path is compared against.  It shares no code with the HIP
path and must never be imported by the product package; only tests, the smoke
check and the benchmark's cpu_baseline leg may call it.

Precision policy
  * The quantizer (Section 5, "Group-wise Quantization") runs in IEEE binary32
    with one rounding per operation (numpy float32 ops never fuse), because its
    result is an integer code and a stored (min, scale) pair that the HIP path
    must reproduce bit for bit.
  * Dequantization is the real number min + code * scale rounded once: to FP16 for
    weights (the paper dequantizes to FP16 before computation), to binary32 for
    KV-cache rows (their consumer, the attention, works in binary32).
  * Everything else (Section 3 layer equations) runs in float64 on the
    dequantized operands.  Activations are rounded to FP16 at the points where
    the layer stores an activation tensor: after each LayerNorm, after each
    projection epilogue, the attention output and the layer output.
  * Logits are rounded to binary32 before the greedy argmax (lowest index wins).

Parity pins: every function here is pinned by tests/test_oracle_*.py against
invariants, closed forms, brute force or a library routine, except
`generate` (and `generate_diagonal`, pinned to it: same ids in another order), whose
output values for random weights are fixed by nothing the paper prints:
full-model token ids are "parity unpinned" and are pinned only transitively
(layer pins + schedule invariants).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

GROUP = 64
BITS = 4
QMAX = (1 << BITS) - 1  # 15


# --------------------------------------------------------------------------
# Section 5: group-wise asymmetric quantization, b = 4 bits, g = 64 elements
# --------------------------------------------------------------------------
def quantize_groupwise(x16: np.ndarray, group: int = GROUP, bits: int = BITS):
    """Quantize a [rows, cols] FP16 array in groups of `group` contiguous
    elements along the last axis (Section 5: per group take min and max, map
    each element to round((x-min)/(max-min)*(2^b-1))).

    Reading taken where the paper is silent: the stored pair is
    (min, scale=(max-min)/15) in binary32, the element is divided by that same
    stored scale, rounding is to nearest with ties to even, a constant group
    has scale 0 and all codes 0, and two codes share a byte with the even
    element in the low nibble.

    Returns (codes uint8 [rows, cols/2], meta float32 [rows, cols/group, 2]).
    """
    if group != GROUP or bits != BITS:
        raise ValueError("only group=64, bits=4 is defined")
    x16 = np.asarray(x16)
    if x16.dtype != np.float16 or x16.ndim != 2:
        raise ValueError("expects a 2-D float16 array")
    rows, cols = x16.shape
    if cols % group != 0:
        raise ValueError("cols must be a multiple of the group size")
    if not np.all(np.isfinite(x16)):
        raise ValueError("non-finite input")
    ng = cols // group
    x = x16.astype(np.float32).reshape(rows, ng, group)
    mn = x.min(axis=2)
    mx = x.max(axis=2)
    rng = (mx - mn).astype(np.float32)
    scale = (rng / np.float32(QMAX)).astype(np.float32)
    codes = np.zeros((rows, ng, group), dtype=np.uint8)
    nz = scale > 0
    if np.any(nz):
        num = (x[nz] - mn[nz][:, None]).astype(np.float32)
        t = (num / scale[nz][:, None]).astype(np.float32)
        codes[nz] = np.clip(np.rint(t), 0, QMAX).astype(np.uint8)
    meta = np.stack([mn, scale], axis=-1).astype(np.float32)
    return pack_codes(codes.reshape(rows, cols)), meta


def quantize_groupwise_h16(x16: np.ndarray, group: int = GROUP, bits: int = BITS):
    """The 4.5-bit variant of Section 5's format: the pair (min, scale) is stored as two FP16 numbers
    (4 bytes per group of 64 instead of 8).

    Reading taken (the paper does not describe a storage precision for the pair): the inputs are
    FP16, so min is stored exactly; scale is the SMALLEST FP16 number >= (max-min)/15 (binary32
    quotient rounded up), so that every code round((x-min)/scale) still lies in [0, 15] without
    clamping and every element is within scale/2 of its reconstruction; the maximum no longer
    round-trips exactly.  Codes are computed in binary32 with that stored scale.

    Returns (codes uint8 [rows, cols/2], meta float16 [rows, cols/group, 2])."""
    if group != GROUP or bits != BITS:
        raise ValueError("only group=64, bits=4 is defined")
    x16 = np.asarray(x16)
    if x16.dtype != np.float16 or x16.ndim != 2:
        raise ValueError("expects a 2-D float16 array")
    rows, cols = x16.shape
    if cols % group != 0:
        raise ValueError("cols must be a multiple of the group size")
    if not np.all(np.isfinite(x16)):
        raise ValueError("non-finite input")
    ng = cols // group
    x = x16.astype(np.float32).reshape(rows, ng, group)
    mn = x.min(axis=2)
    mx = x.max(axis=2)
    q = ((mx - mn).astype(np.float32) / np.float32(QMAX)).astype(np.float32)
    s16 = q.astype(np.float16)                                  # nearest FP16 ...
    low = s16.astype(np.float32) < q                            # ... stepped up where it fell below
    s16 = np.where(low, np.nextafter(s16, np.float16(np.inf)), s16).astype(np.float16)
    scale = s16.astype(np.float32)
    codes = np.zeros((rows, ng, group), dtype=np.uint8)
    nz = scale > 0
    if np.any(nz):
        num = (x[nz] - mn[nz][:, None]).astype(np.float32)
        t = (num / scale[nz][:, None]).astype(np.float32)
        codes[nz] = np.clip(np.rint(t), 0, QMAX).astype(np.uint8)
    meta = np.stack([mn.astype(np.float16), s16], axis=-1)
    return pack_codes(codes.reshape(rows, cols)), meta


def pack_codes(c: np.ndarray) -> np.ndarray:
    """Two 4-bit codes per byte, even element in the low nibble."""
    c = np.asarray(c, dtype=np.uint8)
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_codes(b: np.ndarray) -> np.ndarray:
    """Inverse of pack_codes: [..., n] bytes -> [..., 2n] codes."""
    b = np.asarray(b, dtype=np.uint8)
    out = np.empty(b.shape[:-1] + (b.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = b & 0x0F
    out[..., 1::2] = b >> 4
    return out


def _dequantize_exact(codes: np.ndarray, meta: np.ndarray, group: int = GROUP) -> np.ndarray:
    """The real number min + code * scale of every element, held in float64 (the product of a
    4-bit code and a binary32 scale is exact there, and so is the sum unless the two terms are
    more than 2^25 apart in magnitude)."""
    c = unpack_codes(codes).astype(np.float64)
    shp = c.shape
    c = c.reshape(shp[:-1] + (shp[-1] // group, group))
    mn = meta[..., 0].astype(np.float64)[..., None]
    sc = meta[..., 1].astype(np.float64)[..., None]
    return (mn + c * sc).reshape(shp)


def dequantize_groupwise(codes: np.ndarray, meta: np.ndarray, group: int = GROUP) -> np.ndarray:
    """x_hat = min + code * scale rounded once to binary32 (Section 5: stored quantized, converted
    back before computation).  Used for the KV cache, whose consumer works in binary32."""
    return _dequantize_exact(codes, meta, group).astype(np.float32)


def dequantize_groupwise_f16(codes: np.ndarray, meta: np.ndarray, group: int = GROUP) -> np.ndarray:
    """The FP16 number nearest to min + code * scale (Section 5: "converted back to FP16 before
    computation").  This is the weight value the projections multiply with."""
    return _dequantize_exact(codes, meta, group).astype(np.float16)


# --------------------------------------------------------------------------
# Section 3 building blocks (float64)
# --------------------------------------------------------------------------
def round_f16(x: np.ndarray) -> np.ndarray:
    """Round to FP16 storage precision and come back to float64."""
    return np.asarray(x, dtype=np.float64).astype(np.float16).astype(np.float64)


def layernorm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float) -> np.ndarray:
    """Row-wise LayerNorm (biased variance), as OPT's pre-LN decoder uses."""
    x = np.asarray(x, dtype=np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(gamma, np.float64) + np.asarray(beta, np.float64)


@dataclass
class Mat:
    """A weight matrix [out, in], row-major: FP16 values, or 4-bit codes with
    one (min, scale) pair per 64 consecutive input-dimension elements."""
    rows: int
    cols: int
    f16: Optional[np.ndarray] = None      # [rows, cols] float16
    codes: Optional[np.ndarray] = None    # [rows, cols/2] uint8
    meta: Optional[np.ndarray] = None     # [rows, cols/64, 2] float32 (float16: the FP16-pair variant)

    @staticmethod
    def from_f16(w16: np.ndarray, quantized: bool, meta_f16: bool = False) -> "Mat":
        w16 = np.ascontiguousarray(w16, dtype=np.float16)
        r, c = w16.shape
        if quantized:
            codes, meta = quantize_groupwise_h16(w16) if meta_f16 else quantize_groupwise(w16)
            return Mat(r, c, codes=codes, meta=meta)
        return Mat(r, c, f16=w16)

    def dense(self) -> np.ndarray:
        """The matrix the layer computes with, as float64: the FP16 values, or the
        values dequantized back to FP16 (Section 5)."""
        if self.f16 is not None:
            return self.f16.astype(np.float64)
        return dequantize_groupwise_f16(self.codes, self.meta).astype(np.float64)


def linear(x: np.ndarray, w: Mat, bias: Optional[np.ndarray]) -> np.ndarray:
    """y = x . W^T + b with W stored [out, in] (Section 3: x . w)."""
    y = np.asarray(x, np.float64) @ w.dense().T
    if bias is not None:
        y = y + np.asarray(bias, np.float64)
    return y


def softmax_rows(s: np.ndarray) -> np.ndarray:
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def attn_decode(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """One head, one query (Section 3, decode phase):
    softmax(q . K^T / sqrt(dh)) . V with q [dh], K and V [rows, dh]."""
    dh = q.shape[-1]
    s = (k @ q) / math.sqrt(dh)
    p = softmax_rows(s[None, :])[0]
    return p @ v


def attn_decode_scores(q: np.ndarray, k: np.ndarray) -> np.ndarray:
    """Scaled attention scores of one query against the cached keys: q . K^T / sqrt(dh)."""
    return (k @ q) / math.sqrt(q.shape[-1])


def topk_indices(s: np.ndarray, topk: int) -> np.ndarray:
    """Indices of the `topk` largest scores, ascending; among equal scores the lowest index wins
    (the paper does not say: this is the reading both sides use)."""
    order = np.argsort(-s, kind="stable")      # stable: equal scores keep index order
    return np.sort(order[:topk])


def attn_decode_subset(q: np.ndarray, k: np.ndarray, v: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Sparse decode attention for a given set of kept rows (Section 5, sparse attention): the
    attention weights are those of the FULL softmax over all cached rows; the rows outside `idx` are
    dropped, i.e. only the V rows in `idx` are read, and nothing is renormalised."""
    p = softmax_rows(attn_decode_scores(q, k)[None, :])[0]
    return p[idx] @ v[idx]


def attn_decode_topk(q: np.ndarray, k: np.ndarray, v: np.ndarray, topk: int):
    """Top-K sparse decode attention (Section 5, sparse attention): after the attention weights of
    the query are known, keep its `topk` highest-weighted rows and load only those rows of V.
    Returns (output [dh], kept indices ascending)."""
    idx = topk_indices(attn_decode_scores(q, k), topk)
    return attn_decode_subset(q, k, v, idx), idx


def attn_prefill(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """One head, s queries, causal (Section 3, prefill phase): row i attends
    to rows 0..i.  q, k, v are [s, dh]."""
    s_len, dh = q.shape
    sc = (q @ k.T) / math.sqrt(dh)
    mask = np.triu(np.ones((s_len, s_len), dtype=bool), k=1)
    sc = np.where(mask, -np.inf, sc)
    return softmax_rows(sc) @ v


# --------------------------------------------------------------------------
# Model containers
# --------------------------------------------------------------------------
@dataclass
class ModelCfg:
    h1: int
    nh: int
    h2: int
    vocab: int
    max_pos: int
    ln_eps: float = 1e-5

    @property
    def dh(self) -> int:
        return self.h1 // self.nh


@dataclass
class LayerWeights:
    wqkv: Mat                       # [3*h1, h1]: rows 0..h1-1 = Wq, then Wk, then Wv
    wo: Mat                         # [h1, h1]
    w1: Mat                         # [h2, h1]
    w2: Mat                         # [h1, h2]
    ln1_g: np.ndarray
    ln1_b: np.ndarray
    ln2_g: np.ndarray
    ln2_b: np.ndarray
    bqkv: Optional[np.ndarray] = None
    bo: Optional[np.ndarray] = None
    b1: Optional[np.ndarray] = None
    b2: Optional[np.ndarray] = None


@dataclass
class KVCache:
    """Per-layer cache, logical layout [batch, nh, cap, dh].  Quantized form:
    codes [batch, nh, cap, dh/2] and meta [batch, nh, cap, dh/64, 2], groups of
    64 along the hidden dimension of each token row (Section 5)."""
    batch: int
    nh: int
    cap: int
    dh: int
    quantized: bool
    meta_f16: bool = False      # quantized only: (min, scale) stored as FP16 (quantize_groupwise_h16)
    k_codes: np.ndarray = field(default=None)
    k_meta: np.ndarray = field(default=None)
    v_codes: np.ndarray = field(default=None)
    v_meta: np.ndarray = field(default=None)
    k_f16: np.ndarray = field(default=None)
    v_f16: np.ndarray = field(default=None)

    @staticmethod
    def empty(batch: int, nh: int, cap: int, dh: int, quantized: bool, meta_f16: bool = False) -> "KVCache":
        c = KVCache(batch, nh, cap, dh, quantized, meta_f16 and quantized)
        if quantized:
            assert dh % GROUP == 0
            mt = np.float16 if meta_f16 else np.float32
            c.k_codes = np.zeros((batch, nh, cap, dh // 2), np.uint8)
            c.v_codes = np.zeros((batch, nh, cap, dh // 2), np.uint8)
            c.k_meta = np.zeros((batch, nh, cap, dh // GROUP, 2), mt)
            c.v_meta = np.zeros((batch, nh, cap, dh // GROUP, 2), mt)
        else:
            c.k_f16 = np.zeros((batch, nh, cap, dh), np.float16)
            c.v_f16 = np.zeros((batch, nh, cap, dh), np.float16)
        return c

    def store(self, b0: int, pos0: int, k16: np.ndarray, v16: np.ndarray) -> None:
        """Store FP16 K/V rows [nb, npos, h1] for sequences b0.. at cache rows
        pos0..; quantizes each token row along its hidden dimension when the
        cache is compressed."""
        nb, npos, h1 = k16.shape
        assert h1 == self.nh * self.dh
        for name, x16 in (("k", k16), ("v", v16)):
            x16 = np.ascontiguousarray(x16, np.float16)
            if self.quantized:
                quant = quantize_groupwise_h16 if self.meta_f16 else quantize_groupwise
                codes, meta = quant(x16.reshape(nb * npos, h1))
                codes = codes.reshape(nb, npos, self.nh, self.dh // 2).transpose(0, 2, 1, 3)
                meta = meta.reshape(nb, npos, self.nh, self.dh // GROUP, 2).transpose(0, 2, 1, 3, 4)
                getattr(self, name + "_codes")[b0:b0 + nb, :, pos0:pos0 + npos] = codes
                getattr(self, name + "_meta")[b0:b0 + nb, :, pos0:pos0 + npos] = meta
            else:
                x = x16.reshape(nb, npos, self.nh, self.dh).transpose(0, 2, 1, 3)
                getattr(self, name + "_f16")[b0:b0 + nb, :, pos0:pos0 + npos] = x

    def load(self, b: int, head: int, rows: int):
        """K_hat, V_hat [rows, dh] float64 for one (sequence, head), converted
        back from the stored format."""
        if self.quantized:
            k = dequantize_groupwise(self.k_codes[b, head, :rows], self.k_meta[b, head, :rows])
            v = dequantize_groupwise(self.v_codes[b, head, :rows], self.v_meta[b, head, :rows])
        else:
            k = self.k_f16[b, head, :rows]
            v = self.v_f16[b, head, :rows]
        return k.astype(np.float64), v.astype(np.float64)


# --------------------------------------------------------------------------
# Section 3: one transformer layer, prefill and decode
# --------------------------------------------------------------------------
def _ffn_and_residual(cfg: ModelCfg, w: LayerWeights, o: np.ndarray, x: np.ndarray) -> np.ndarray:
    """x_out = o.wO + x ;  x' = relu(LN(x_out).w1).w2 + x_out  (Section 3,
    with OPT's pre-LN placement and biases where present)."""
    x1 = round_f16(linear(o, w.wo, w.bo) + x)
    y2 = round_f16(layernorm(x1, w.ln2_g, w.ln2_b, cfg.ln_eps))
    a = round_f16(np.maximum(linear(y2, w.w1, w.b1), 0.0))
    return round_f16(linear(a, w.w2, w.b2) + x1)


def prefill_layer(cfg: ModelCfg, w: LayerWeights, x16: np.ndarray, kv: KVCache,
                  batch_offset: int = 0) -> np.ndarray:
    """Prefill phase of one layer (Section 3).  x16 [b, s, h1] FP16.  Attention
    is causal over the freshly computed FP16 K/V; afterwards the s K/V rows are
    stored (quantized when the cache is compressed) at cache rows 0..s-1 of
    sequences batch_offset..batch_offset+b-1.  Returns [b, s, h1] FP16."""
    b, s, h1 = x16.shape
    nh, dh = cfg.nh, cfg.dh
    x = x16.astype(np.float64).reshape(b * s, h1)
    y = round_f16(layernorm(x, w.ln1_g, w.ln1_b, cfg.ln_eps))
    qkv = round_f16(linear(y, w.wqkv, w.bqkv))
    q = qkv[:, :h1].reshape(b, s, nh, dh)
    k = qkv[:, h1:2 * h1].reshape(b, s, nh, dh)
    v = qkv[:, 2 * h1:].reshape(b, s, nh, dh)
    o = np.empty((b, s, nh, dh))
    for bi in range(b):
        for h in range(nh):
            o[bi, :, h, :] = attn_prefill(q[bi, :, h], k[bi, :, h], v[bi, :, h])
    o = round_f16(o.reshape(b * s, h1))
    kv.store(batch_offset, 0, k.reshape(b, s, h1).astype(np.float16), v.reshape(b, s, h1).astype(np.float16))
    out = _ffn_and_residual(cfg, w, o, x)
    return out.reshape(b, s, h1).astype(np.float16)


def decode_layer(cfg: ModelCfg, w: LayerWeights, x16: np.ndarray, t: int, kv: KVCache,
                 batch_offset: int = 0, topk: int = 0) -> np.ndarray:
    """Decode phase of one layer (Section 3).  x16 [b, h1] FP16 is the current
    token's activation; t rows are already cached.  The new K/V row is appended
    at row t in the storage format, then the query attends to rows 0..t as read
    back from the cache (so it sees its own row dequantized).

    topk > 0: the attention is the sparse one of Section 5 (attn_decode_topk): of the t + 1 rows only
    the min(topk, t + 1) with the largest attention weights contribute their V rows."""
    b, h1 = x16.shape
    nh, dh = cfg.nh, cfg.dh
    x = x16.astype(np.float64)
    y = round_f16(layernorm(x, w.ln1_g, w.ln1_b, cfg.ln_eps))
    qkv = round_f16(linear(y, w.wqkv, w.bqkv))
    q = qkv[:, :h1].reshape(b, nh, dh)
    k_new = qkv[:, h1:2 * h1].astype(np.float16).reshape(b, 1, h1)
    v_new = qkv[:, 2 * h1:].astype(np.float16).reshape(b, 1, h1)
    kv.store(batch_offset, t, k_new, v_new)
    o = np.empty((b, nh, dh))
    for bi in range(b):
        for h in range(nh):
            kh, vh = kv.load(batch_offset + bi, h, t + 1)
            if topk > 0 and topk < t + 1:
                o[bi, h] = attn_decode_topk(q[bi, h], kh, vh, topk)[0]
            else:
                o[bi, h] = attn_decode(q[bi, h], kh, vh)
    o = round_f16(o.reshape(b, h1))
    return _ffn_and_residual(cfg, w, o, x).astype(np.float16)


# --------------------------------------------------------------------------
# Model level: embedding, final LN, tied LM head, greedy token
# --------------------------------------------------------------------------
def embed(tokens: np.ndarray, positions: np.ndarray, emb16: np.ndarray, pos16: np.ndarray) -> np.ndarray:
    """x0 = E[token] + P[position], rounded to FP16."""
    return round_f16(emb16[tokens].astype(np.float64) + pos16[positions].astype(np.float64)).astype(np.float16)


def lm_head_logits(cfg: ModelCfg, x16: np.ndarray, lnf_g, lnf_b, emb16: np.ndarray) -> np.ndarray:
    """Final LayerNorm (FP16 storage) then logits against the tied, unquantized
    embedding; returned as binary32."""
    y = round_f16(layernorm(x16.astype(np.float64), lnf_g, lnf_b, cfg.ln_eps))
    return (y @ emb16.astype(np.float64).T).astype(np.float32)


def greedy(logits32: np.ndarray) -> np.ndarray:
    """argmax per row, lowest index on ties (numpy's argmax rule)."""
    return np.argmax(logits32, axis=-1).astype(np.int32)


def generate(cfg: ModelCfg, layers: List[LayerWeights], emb16, pos16, lnf_g, lnf_b,
             prompt: np.ndarray, n: int, num_gpu_batches: int, gpu_batch_size: int,
             kv_quantized: bool, return_trace: bool = False, kv_meta_f16: bool = False):
    """Generate n tokens for a block of num_gpu_batches x gpu_batch_size
    sequences with the block schedule (Algorithm 1): token step i outermost,
    then layer j, then GPU batch k.  Step 1 is the prefill of the whole prompt
    and emits token 1; steps 2..n are decode steps.  With every tensor resident
    in one memory the load/store calls of Algorithm 1 have nothing to move, so
    only compute(i, j, k) remains.

    prompt int32 [bls, s].  kv_meta_f16: the compressed cache keeps FP16 (min, scale) pairs.
    Returns ids int32 [bls, n] (and, on request, the per-step logits float32 [n, bls, vocab])."""
    bls, s = prompt.shape
    assert bls == num_gpu_batches * gpu_batch_size
    assert n >= 1 and s + n - 1 <= cfg.max_pos
    l = len(layers)
    cap = s + n
    caches = [KVCache.empty(bls, cfg.nh, cap, cfg.dh, kv_quantized, kv_meta_f16) for _ in range(l)]
    ids = np.zeros((bls, n), np.int32)
    trace = []
    sl = [slice(k * gpu_batch_size, (k + 1) * gpu_batch_size) for k in range(num_gpu_batches)]
    for i in range(n):
        if i == 0:
            pos = np.broadcast_to(np.arange(s), (bls, s))
            act = [embed(prompt[sl[k]], pos[sl[k]], emb16, pos16) for k in range(num_gpu_batches)]
        else:
            p = s + i - 1                      # absolute position of the token fed back in
            act = [embed(ids[sl[k], i - 1], np.full(gpu_batch_size, p), emb16, pos16)
                   for k in range(num_gpu_batches)]
        for j in range(l):
            for k in range(num_gpu_batches):
                if i == 0:
                    act[k] = prefill_layer(cfg, layers[j], act[k], caches[j], batch_offset=k * gpu_batch_size)
                else:
                    act[k] = decode_layer(cfg, layers[j], act[k], s + i - 1, caches[j],
                                          batch_offset=k * gpu_batch_size)
        last = np.concatenate([a[:, -1, :] if i == 0 else a for a in act], axis=0)
        logits = lm_head_logits(cfg, last, lnf_g, lnf_b, emb16)
        ids[:, i] = greedy(logits)
        if return_trace:
            trace.append(logits)
    if return_trace:
        return ids, np.stack(trace), caches
    return ids


# --------------------------------------------------------------------------
# Appendix, "Diagonal block schedule": non-contiguous cache, sequences at different steps
# --------------------------------------------------------------------------
PAGE_ROWS = 64


@dataclass
class PagedKVCache:
    """One layer's compressed K/V cache in non-contiguous memory (the appendix names attention over
    non-contiguous memory as what the diagonal block schedule needs in order to save memory).

    A pool of pages; a page holds PAGE_ROWS = 64 consecutive positions of ONE sequence, for all heads:
    codes [n_pages, nh, 64, dh/2], meta [n_pages, nh, 64, dh/64, 2].  table[seq] lists the pages of
    sequence `seq` in position order (position p lives in page table[seq][p // 64], row p % 64).
    Every row is quantized exactly as in KVCache (Section 5, along the hidden dimension of the token
    row): this class only changes where a row is kept.  It has KVCache's store/load interface, the
    sequence id taking the place of the batch index."""
    nh: int
    dh: int
    n_pages: int
    table: np.ndarray                      # int32 [n_seqs, max_pages_per_seq]; -1 = no page
    meta_f16: bool = False
    quantized: bool = True                 # False: the pages hold plain FP16 rows [n_pages, nh, 64, dh]
    k_codes: np.ndarray = field(default=None)
    k_meta: np.ndarray = field(default=None)
    v_codes: np.ndarray = field(default=None)
    v_meta: np.ndarray = field(default=None)
    k_f16: np.ndarray = field(default=None)
    v_f16: np.ndarray = field(default=None)

    @staticmethod
    def empty(nh: int, dh: int, n_pages: int, table: np.ndarray, meta_f16: bool = False,
              quantized: bool = True) -> "PagedKVCache":
        assert dh % GROUP == 0
        c = PagedKVCache(nh, dh, n_pages, np.asarray(table, np.int32), meta_f16 and quantized, quantized)
        if not quantized:
            c.k_f16 = np.zeros((n_pages, nh, PAGE_ROWS, dh), np.float16)
            c.v_f16 = np.zeros((n_pages, nh, PAGE_ROWS, dh), np.float16)
            return c
        mt = np.float16 if meta_f16 else np.float32
        c.k_codes = np.zeros((n_pages, nh, PAGE_ROWS, dh // 2), np.uint8)
        c.v_codes = np.zeros((n_pages, nh, PAGE_ROWS, dh // 2), np.uint8)
        c.k_meta = np.zeros((n_pages, nh, PAGE_ROWS, dh // GROUP, 2), mt)
        c.v_meta = np.zeros((n_pages, nh, PAGE_ROWS, dh // GROUP, 2), mt)
        return c

    def _where(self, seq: int, pos: int):
        page = int(self.table[seq, pos // PAGE_ROWS])
        assert 0 <= page < self.n_pages, "position %d of sequence %d has no page" % (pos, seq)
        return page, pos % PAGE_ROWS

    def store(self, b0: int, pos0: int, k16: np.ndarray, v16: np.ndarray) -> None:
        """FP16 K/V rows [nb, npos, h1] of sequences b0.. at positions pos0..: each token row is
        quantized along its hidden dimension (or kept as FP16) and written row by row through the
        page table."""
        nb, npos, h1 = k16.shape
        assert h1 == self.nh * self.dh
        if not self.quantized:
            for name, x16 in (("k", k16), ("v", v16)):
                x = np.ascontiguousarray(x16, np.float16).reshape(nb, npos, self.nh, self.dh)
                for i in range(nb):
                    for p in range(npos):
                        page, r = self._where(b0 + i, pos0 + p)
                        getattr(self, name + "_f16")[page, :, r] = x[i, p]
            return
        quant = quantize_groupwise_h16 if self.meta_f16 else quantize_groupwise
        for name, x16 in (("k", k16), ("v", v16)):
            codes, meta = quant(np.ascontiguousarray(x16, np.float16).reshape(nb * npos, h1))
            codes = codes.reshape(nb, npos, self.nh, self.dh // 2)
            meta = meta.reshape(nb, npos, self.nh, self.dh // GROUP, 2)
            for i in range(nb):
                for p in range(npos):
                    page, r = self._where(b0 + i, pos0 + p)
                    getattr(self, name + "_codes")[page, :, r] = codes[i, p]
                    getattr(self, name + "_meta")[page, :, r] = meta[i, p]

    def load(self, b: int, head: int, rows: int):
        """K_hat, V_hat [rows, dh] float64 of one (sequence, head): the rows gathered through the
        page table, converted back from the stored format."""
        out = []
        for name in ("k", "v"):
            if not self.quantized:
                x = np.empty((rows, self.dh), np.float16)
                for p in range(rows):
                    page, r = self._where(b, p)
                    x[p] = getattr(self, name + "_f16")[page, head, r]
                out.append(x.astype(np.float64))
                continue
            codes = np.empty((rows, self.dh // 2), np.uint8)
            meta = np.empty((rows, self.dh // GROUP, 2), self.k_meta.dtype)
            for p in range(rows):
                page, r = self._where(b, p)
                codes[p] = getattr(self, name + "_codes")[page, head, r]
                meta[p] = getattr(self, name + "_meta")[page, head, r]
            out.append(dequantize_groupwise(codes, meta).astype(np.float64))
        return out[0], out[1]


def decode_layer_ragged(cfg: ModelCfg, w: LayerWeights, x16: np.ndarray, seq_ids, pos, kv, topk: int = 0) -> np.ndarray:
    """A decode step in which row i belongs to sequence seq_ids[i] and sits at its own position pos[i]
    (pos[i] rows already cached), as in the diagonal block schedule, where the GPU batches of a block
    are at different token steps.  Section 3 treats every sequence on its own, so this is decode_layer
    applied to each row with its own t (and, with topk > 0, its own min(topk, t + 1) kept rows).
    kv: a KVCache or a PagedKVCache.  x16 [b, h1] FP16."""
    out = np.empty_like(np.asarray(x16, np.float16))
    for i in range(out.shape[0]):
        out[i] = decode_layer(cfg, w, x16[i:i + 1], int(pos[i]), kv, batch_offset=int(seq_ids[i]), topk=topk)[0]
    return out


def generate_diagonal(cfg: ModelCfg, layers: List[LayerWeights], emb16, pos16, lnf_g, lnf_b,
                      prompt: np.ndarray, n: int, gpu_batch_size: int, meta_f16: bool = False,
                      return_page_use: bool = False):
    """Generation in the order of the appendix's diagonal block schedule, for a queue of
    prompt.shape[0] sequences cut into GPU batches of gpu_batch_size: one GPU batch is admitted per
    iteration, so in iteration `it` batch g is at token step it - g; an iteration runs, layer by layer,
    the prefill of the newly admitted batch and one decode step of every batch still generating (the
    squares of one diagonal), then emits one token for each of them.  A batch is retired after its
    n-th token and its cache pages return to the pool; pages are taken one at a time as a sequence
    grows.  The compressed cache is paged (PagedKVCache), one pool per layer.

    The schedule only reorders independent work, so the ids equal generate()'s row for row.
    Returns ids int32 [n_seqs, n] (and, on request, the largest number of pages in use at once)."""
    n_seqs, s = prompt.shape
    assert n_seqs % gpu_batch_size == 0 and n >= 1 and s + n - 1 <= cfg.max_pos
    ng = n_seqs // gpu_batch_size
    l = len(layers)
    max_pages = -(-(s + n) // PAGE_ROWS)
    in_flight = min(ng, n)
    pool_pages = in_flight * gpu_batch_size * max_pages          # an upper bound; page_use reports the need
    table = np.full((n_seqs, max_pages), -1, np.int32)
    caches = [PagedKVCache.empty(cfg.nh, cfg.dh, pool_pages, table, meta_f16) for _ in range(l)]
    for c in caches:
        c.table = table                                          # one table, shared by the layers
    free = list(range(pool_pages - 1, -1, -1))
    ids = np.zeros((n_seqs, n), np.int32)
    peak = 0

    def ensure(seq: int, rows: int):
        for slot in range(-(-rows // PAGE_ROWS)):
            if table[seq, slot] < 0:
                table[seq, slot] = free.pop()

    for it in range(ng + n - 1):
        groups = [g for g in range(ng) if 0 <= it - g < n]
        # this iteration's rows: the admitted batch's prompt, and one token of every older batch
        new = [g for g in groups if it - g == 0]
        old = [g for g in groups if it - g > 0]
        old_seqs = np.array([q for g in old for q in range(g * gpu_batch_size, (g + 1) * gpu_batch_size)], np.int64)
        old_pos = np.array([s + (it - q // gpu_batch_size) - 1 for q in old_seqs], np.int64)
        for q, p in zip(old_seqs, old_pos):
            ensure(int(q), int(p) + 1)
        x_new = None
        if new:
            sl = slice(new[0] * gpu_batch_size, (new[0] + 1) * gpu_batch_size)
            for q in range(sl.start, sl.stop):
                ensure(q, s)
            x_new = embed(prompt[sl], np.broadcast_to(np.arange(s), (gpu_batch_size, s)), emb16, pos16)
        peak = max(peak, pool_pages - len(free))
        x_old = None
        if len(old_seqs):
            step = np.array([it - q // gpu_batch_size for q in old_seqs])
            x_old = embed(ids[old_seqs, step - 1], old_pos, emb16, pos16)
        for j in range(l):
            if x_new is not None:
                x_new = prefill_layer(cfg, layers[j], x_new, caches[j], batch_offset=new[0] * gpu_batch_size)
            if x_old is not None:
                x_old = decode_layer_ragged(cfg, layers[j], x_old, old_seqs, old_pos, caches[j])
        if x_new is not None:
            ids[sl, 0] = greedy(lm_head_logits(cfg, x_new[:, -1, :], lnf_g, lnf_b, emb16))
        if x_old is not None:
            ids[old_seqs, step] = greedy(lm_head_logits(cfg, x_old, lnf_g, lnf_b, emb16))
        for g in groups:
            if it - g == n - 1:                                   # retired: its pages go back
                for q in range(g * gpu_batch_size, (g + 1) * gpu_batch_size):
                    for slot in range(max_pages):
                        if table[q, slot] >= 0:
                            free.append(int(table[q, slot]))
                            table[q, slot] = -1
    if return_page_use:
        return ids, peak
    return ids


# --------------------------------------------------------------------------
# Section 3 "Memory Analysis" and Section 4.3 cost-model byte / flop terms
# --------------------------------------------------------------------------
def weight_bytes_fp16(l: int, h1: int, h2: int) -> int:
    """l (8 h1^2 + 4 h1 h2): FP16 bytes of the six matrices of every layer."""
    return l * (8 * h1 * h1 + 4 * h1 * h2)


def kv_bytes_fp16_peak(b: int, l: int, h1: int, s: int, n: int) -> int:
    """4 b l h1 (s + n): FP16 bytes of K and V at the end of generation."""
    return 4 * b * l * h1 * (s + n)


def layer_weight_elements(h1: int, h2: int) -> int:
    return 4 * h1 * h1 + 2 * h1 * h2


def bytes_per_element(quantized: bool) -> float:
    """FP16: 2 bytes.  4-bit groups of 64 with a binary32 (min, scale) pair:
    1/2 + 8/64 = 0.625 bytes."""
    return 0.5 + 8.0 / GROUP if quantized else 2.0


def decode_step_bytes(l: int, h1: int, h2: int, bls: int, rows_attended: int,
                      w_quantized: bool, kv_quantized: bool) -> float:
    """Algorithmic HBM bytes of one decode step of a block: every layer's
    weights once per block (zig-zag order) plus every cached K and V row that
    the step attends to (cost-model terms of Section 4.3, re-priced for the
    storage format)."""
    w = l * layer_weight_elements(h1, h2) * bytes_per_element(w_quantized)
    kv = 2.0 * bls * l * h1 * rows_attended * bytes_per_element(kv_quantized)
    return w + kv


def decode_linear_flops(l: int, h1: int, h2: int, bls: int) -> int:
    """bls (8 h1^2 + 4 h1 h2) per layer (Appendix cost model, linear_layer^g)."""
    return l * bls * (8 * h1 * h1 + 4 * h1 * h2)


def prefill_flops(l: int, h1: int, h2: int, bls: int, s: int) -> int:
    """bls (8 s h1^2 + 4 s h1 h2) + 4 bls s^2 h1 per layer (Appendix, comp^p)."""
    return l * (bls * (8 * s * h1 * h1 + 4 * s * h1 * h2) + 4 * bls * s * s * h1)
