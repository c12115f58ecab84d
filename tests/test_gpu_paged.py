"""GPU parity for the paged cache path (appendix, "Diagonal block schedule": attention over
non-contiguous cache memory, sequences of a block at different token steps): the paged KV append is
bit-exact against the oracle's pool, the paged decode attention and the paged layer calls meet the
activation tolerance against the oracle's per-sequence definitions."""
import numpy as np
import pytest
import torch

from oracle import fg_oracle as O
from paper_2303_06865_amd import binding as B
from paper_2303_06865_amd import synth
from tests.util import assert_close, cfg_pair, dev, host, oracle_layer

pytestmark = pytest.mark.gpu


def _rand16(shape, std, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(shape) * std).astype(np.float16)


def _make_table(lens, n_pages, stride, seed, extra=0):
    """A shuffled assignment of pages to sequences: ceil(len / 64) + extra pages each, -1 elsewhere."""
    rng = np.random.default_rng(seed)
    perm = rng.permutation(n_pages)
    table = np.full((len(lens), stride), -1, np.int32)
    nxt = 0
    for q, ln in enumerate(lens):
        for slot in range(min(stride, -(-ln // 64) + extra)):
            table[q, slot] = perm[nxt]
            nxt += 1
    assert nxt <= n_pages
    return table


def _upload(pages, opaged):
    pages.k_codes.copy_(dev(opaged.k_codes)); pages.v_codes.copy_(dev(opaged.v_codes))
    pages.k_meta.copy_(dev(opaged.k_meta)); pages.v_meta.copy_(dev(opaged.v_meta))


def _pool_equal(pages, opaged, meta_f16):
    bits = np.uint16 if meta_f16 else np.uint32
    return (np.array_equal(host(pages.k_codes), opaged.k_codes) and np.array_equal(host(pages.v_codes), opaged.v_codes)
            and np.array_equal(host(pages.k_meta).view(bits), opaged.k_meta.view(bits))
            and np.array_equal(host(pages.v_meta).view(bits), opaged.v_meta.view(bits)))


@pytest.mark.parametrize("meta_f16", [False, True])
@pytest.mark.parametrize("nh,dh", [(3, 128), (6, 64)])
def test_kv_append_paged_bit_exact(nh, dh, meta_f16):
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 1000, 512)
    lens = [130, 5, 64, 65, 200]
    table = _make_table(lens, 17, 4, seed=nh)
    opaged = O.PagedKVCache.empty(nh, dh, 17, table, meta_f16)
    pages = B.KVPages(cfg, 17, meta_f16)
    dtab = dev(table)
    # (a) whole prompts of three of the sequences, rows given in another order than the ids
    seq_ids = np.array([3, 0, 2], np.int32)
    s = 60
    qkv = _rand16((3 * s, 3 * h1), 1.0, 11)
    k16 = qkv[:, h1:2 * h1].reshape(3, s, h1)
    v16 = qkv[:, 2 * h1:].reshape(3, s, h1)
    for i, q in enumerate(seq_ids):
        opaged.store(int(q), 0, k16[i:i + 1], v16[i:i + 1])
    dq = dev(qkv)
    B.fg_kv_append_paged(cfg, dq[:, h1:], dq[:, 2 * h1:], 3 * h1, 3, s, pages, B.Ragged(dtab, dev(seq_ids), None))
    torch.cuda.synchronize()
    assert _pool_equal(pages, opaged, meta_f16)
    # (b) a ragged step: one new row per sequence at its own position, two of them first rows of a page
    seq_ids = np.array([0, 1, 2, 3, 4], np.int32)
    pos = np.array([64, 4, 60, 64, 199], np.int32)
    qkv = _rand16((5, 3 * h1), 1.0, 12)
    for i, q in enumerate(seq_ids):
        opaged.store(int(q), int(pos[i]), qkv[i:i + 1, h1:2 * h1].reshape(1, 1, h1), qkv[i:i + 1, 2 * h1:].reshape(1, 1, h1))
    dq = dev(qkv)
    B.fg_kv_append_paged(cfg, dq[:, h1:], dq[:, 2 * h1:], 3 * h1, 5, 1, pages, B.Ragged(dtab, dev(seq_ids), dev(pos)))
    torch.cuda.synchronize()
    assert _pool_equal(pages, opaged, meta_f16)
    # (c) destinations that do not exist are skipped: no page for that position, a position past the
    # table, a sequence id out of range; nothing in the pool changes
    seq_ids = np.array([1, 0, 9], np.int32)
    pos = np.array([64, 256, 0], np.int32)
    B.fg_kv_append_paged(cfg, dq[:, h1:], dq[:, 2 * h1:], 3 * h1, 3, 1, pages, B.Ragged(dtab, dev(seq_ids), dev(pos)))
    torch.cuda.synchronize()
    assert _pool_equal(pages, opaged, meta_f16)


def _attention_case(nh, dh, lens, seed, meta_f16=False, shuffle_rows=True, extra_pages=0):
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 1000, 64)
    b = len(lens)
    stride = max(1, max(-(-ln // 64) for ln in lens) + extra_pages)
    n_pages = sum(max(1, -(-ln // 64)) for ln in lens) + 3
    table = _make_table([max(ln, 1) for ln in lens], n_pages, stride, seed)
    opaged = O.PagedKVCache.empty(nh, dh, n_pages, table, meta_f16)
    for q, ln in enumerate(lens):
        if ln:
            opaged.store(q, 0, _rand16((1, ln, h1), 1.0, seed + 10 * q), _rand16((1, ln, h1), 1.0, seed + 10 * q + 1))
    pages = B.KVPages(cfg, n_pages, meta_f16, zero=False)
    _upload(pages, opaged)
    rng = np.random.default_rng(seed)
    order = rng.permutation(b).astype(np.int32) if shuffle_rows else np.arange(b, dtype=np.int32)
    q16 = _rand16((b, 3 * h1), 1.0, seed + 5)
    rows = np.array([lens[q] for q in order], np.int32)
    ref = np.zeros((b, nh, dh))
    for i, q in enumerate(order):
        for h in range(nh):
            if rows[i]:
                kh, vh = opaged.load(int(q), h, int(rows[i]))
                ref[i, h] = O.attn_decode(q16[i, h * dh:(h + 1) * dh].astype(np.float64), kh, vh)
    out = B.fg_decode_attention_paged(cfg, dev(q16), 3 * h1, b, pages, B.Ragged(dev(table), dev(order), dev(rows)), 0)
    torch.cuda.synchronize()
    return host(out).reshape(b, nh, dh), O.round_f16(ref), rows


@pytest.mark.parametrize("meta_f16", [False, True])
@pytest.mark.parametrize("nh,dh", [(2, 128), (4, 64)])
def test_decode_attention_paged_lengths_around_page_edges(nh, dh, meta_f16):
    lens = [1, 63, 64, 65, 127, 128, 129, 200, 257, 300]
    got, ref, _ = _attention_case(nh, dh, lens, seed=3 + nh, meta_f16=meta_f16, extra_pages=1)
    assert_close(got, ref, "paged decode attention nh=%d dh=%d" % (nh, dh))


def test_decode_attention_paged_empty_sequence_gives_zeros():
    got, ref, rows = _attention_case(2, 128, [70, 0, 5], seed=9, shuffle_rows=False)
    assert_close(got, ref, "paged decode attention with an empty sequence")
    assert not got[1].any()


@pytest.mark.parametrize("dh", [64, 128])
def test_decode_attention_paged_more_than_64_pages(dh):
    """A sequence longer than 64 pages: the wave reloads its window of table entries."""
    got, ref, _ = _attention_case(1, dh, [64 * 64 + 70, 64 * 64, 10], seed=21)
    assert_close(got, ref, "paged decode attention, long sequence")


@pytest.mark.parametrize("b,nh,dh", [(48, 24, 64), (20, 128, 64), (17, 128, 128)])
def test_decode_attention_paged_one_and_two_waves_per_head(b, nh, dh):
    """Enough heads for the launches with two waves and with one wave per head."""
    rng = np.random.default_rng(b)
    lens = [int(v) for v in rng.integers(1, 150, size=b)]
    got, ref, _ = _attention_case(nh, dh, lens, seed=31)
    assert_close(got, ref, "paged decode attention b=%d nh=%d" % (b, nh))


def test_decode_attention_paged_equals_contiguous_kernel_bitwise():
    """Same rows, same order of operations: the paged kernel's output equals the contiguous kernel's
    bit for bit when every sequence has the same length."""
    nh, dh, b, rows = 4, 128, 6, 150
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 1000, 64)
    table = _make_table([rows] * b, 20, 3, seed=5)
    opaged = O.PagedKVCache.empty(nh, dh, 20, table)
    okv = O.KVCache.empty(b, nh, rows, dh, True)
    for q in range(b):
        k, v = _rand16((1, rows, h1), 1.0, 70 + q), _rand16((1, rows, h1), 1.0, 80 + q)
        opaged.store(q, 0, k, v)
        okv.store(q, 0, k, v)
    pages = B.KVPages(cfg, 20, zero=False)
    _upload(pages, opaged)
    kv = B.KVCache(cfg, b, rows, True)
    kv.k_codes.copy_(dev(okv.k_codes)); kv.v_codes.copy_(dev(okv.v_codes))
    kv.k_meta.copy_(dev(okv.k_meta)); kv.v_meta.copy_(dev(okv.v_meta))
    q16 = dev(_rand16((b, 3 * h1), 1.0, 90))
    a = B.fg_decode_attention(cfg, q16, 3 * h1, b, rows, kv, 0)
    p = B.fg_decode_attention_paged(cfg, q16, 3 * h1, b, pages,
                                    B.Ragged(dev(table), None, dev(np.full(b, rows, np.int32))), 0)
    torch.cuda.synchronize()
    assert torch.equal(a, p)


@pytest.mark.parametrize("meta_f16", [False, True])
@pytest.mark.parametrize("dh128", [False, True])
def test_layer_paged_prefill_then_ragged_decode(dh128, meta_f16):
    """Prefill three sequences into pages, then ragged decode steps in which the sequences sit at
    different positions (one of them crossing a page boundary), against the oracle."""
    sh = synth.Shape(h1=512, nh=4, h2=1536, vocab=1000, max_pos=256) if dh128 else synth.OPT_125M_LAYER
    ocfg, cfg = cfg_pair(sh)
    t = synth.layer_tensors(sh, 7, 0, std=0.02, biases=True, random_ln=True)
    ow = oracle_layer(t, True)
    w = B.LayerWeights.from_numpy(t, True, tiled=True)
    n_seqs, s, steps = 4, 62, 4
    table = _make_table([s + steps + 8] * n_seqs, 12, 2, seed=1)
    opaged = O.PagedKVCache.empty(sh.nh, sh.dh, 12, table, meta_f16)
    pages = B.KVPages(cfg, 12, meta_f16)
    dtab = dev(table)
    # prefill sequences 3, 0, 1 (sequence 2 stays empty until later)
    pre = np.array([3, 0, 1], np.int32)
    x = synth.activations_f16((3, s, sh.h1), 0.3, 8)
    ref = np.empty_like(x)
    for i, q in enumerate(pre):
        ref[i] = O.prefill_layer(ocfg, ow, x[i:i + 1], opaged, batch_offset=int(q))[0]
    got = B.fg_prefill_layer_paged(cfg, w, dev(x), pages, B.Ragged(dtab, dev(pre), None))
    torch.cuda.synchronize()
    assert_close(host(got), ref, "paged prefill output")
    # ragged decode: sequence 3 is two steps ahead of 0 and 1 (it gets two extra steps first)
    pos = {3: s, 0: s, 1: s}
    for step in range(steps):
        rows = [3] if step < 2 else [1, 3, 0]
        seq_ids = np.array(rows, np.int32)
        p = np.array([pos[q] for q in rows], np.int32)
        xt = synth.activations_f16((len(rows), sh.h1), 0.3, 100 + step)
        _upload(pages, opaged)      # identical histories on both sides before every step
        ref = O.decode_layer_ragged(ocfg, ow, xt, seq_ids, p, opaged)
        got = B.fg_decode_layer_paged(cfg, w, dev(xt), pages, B.Ragged(dtab, dev(seq_ids), dev(p)))
        torch.cuda.synchronize()
        assert_close(host(got), ref, "paged ragged decode step %d" % step)
        for q in rows:
            pos[q] += 1
    assert pos[3] == s + 4 and pos[3] > 64       # crossed into its second page


def test_embed_ragged_bit_exact():
    sh = synth.OPT_125M_LAYER
    _, cfg = cfg_pair(sh)
    emb = _rand16((sh.vocab, sh.h1), 0.02, 1)
    ptab = _rand16((sh.max_pos, sh.h1), 0.02, 2)
    ids = np.array([0, 5, sh.vocab - 1, 17, 17], np.int32)
    positions = np.array([3, 0, sh.max_pos - 1, 40, 41], np.int32)
    ref = O.embed(ids, positions, emb, ptab)
    got = B.fg_embed_ragged(cfg, dev(emb), dev(ptab), dev(ids), dev(positions))
    torch.cuda.synchronize()
    assert np.array_equal(host(got), ref)


def test_paged_calls_reject_bad_arguments():
    sh = synth.OPT_125M_LAYER
    _, cfg = cfg_pair(sh)
    pages = B.KVPages(cfg, 2)
    table = dev(np.zeros((1, 1), np.int32))
    q = dev(_rand16((1, 3 * sh.h1), 1.0, 1))
    with pytest.raises(RuntimeError):      # the attention needs a length per row
        B.fg_decode_attention_paged(cfg, q, 3 * sh.h1, 1, pages, B.Ragged(table, None, None), 0)
    with pytest.raises(RuntimeError):      # row stride smaller than a row
        B.fg_kv_append_paged(cfg, q, q, 8, 1, 1, pages, B.Ragged(table, None, dev(np.zeros(1, np.int32))))


def test_decode_attention_paged_more_heads_than_wave_slots():
    """3720 heads of different lengths: more than the chip holds waves at once."""
    rng = np.random.default_rng(2)
    lens = [int(v) for v in rng.integers(1, 140, size=31)]
    got, ref, _ = _attention_case(120, 64, lens, seed=41)
    assert_close(got, ref, "paged decode attention, 3720 heads")


# ------------------------------------------------------------------ Top-K sparse attention over pages
@pytest.mark.parametrize("meta_f16", [False, True])
@pytest.mark.parametrize("nh,dh", [(2, 128), (3, 64)])
def test_decode_attention_topk_paged(nh, dh, meta_f16):
    """Section 5's sparse attention over a paged cache with a length per sequence: every row keeps its
    min(topk, rows) highest-weighted rows of V.  As for the contiguous kernel, the kept set must be a
    top-k set of the oracle's scores up to the kernel's FP32 score error, THE oracle's set wherever the
    boundary is clear, and the output must match the oracle's sparse attention on that set."""
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 1000, 64)
    lens = [1, 9, 64, 65, 130, 257, 0, 300]
    topk = 12
    b = len(lens)
    stride = 6
    n_pages = sum(max(1, -(-ln // 64)) for ln in lens) + 2
    table = _make_table([max(ln, 1) for ln in lens], n_pages, stride, seed=13)
    opaged = O.PagedKVCache.empty(nh, dh, n_pages, table, meta_f16)
    for q, ln in enumerate(lens):
        if ln:
            opaged.store(q, 0, _rand16((1, ln, h1), 1.0, 50 + q), _rand16((1, ln, h1), 1.0, 70 + q))
    pages = B.KVPages(cfg, n_pages, meta_f16, zero=False)
    _upload(pages, opaged)
    order = np.random.default_rng(4).permutation(b).astype(np.int32)
    q16 = _rand16((b, 3 * h1), 1.0, 90)
    rows = np.array([lens[q] for q in order], np.int32)
    out, kept = B.fg_decode_attention_topk_paged(cfg, dev(q16), 3 * h1, b, topk, pages,
                                                 B.Ragged(dev(table), dev(order), dev(rows)), 0, want_rows=True)
    torch.cuda.synchronize()
    out, kept = host(out).reshape(b, nh, dh), host(kept)
    ref = np.zeros((b, nh, dh))
    exact = 0
    for i, q in enumerate(order):
        n = int(rows[i])
        keep_n = min(topk, n)
        for h in range(nh):
            got = kept[i, h]
            assert np.all(got[keep_n:] == -1)
            if n == 0:
                continue
            got = got[:keep_n]
            kh, vh = opaged.load(int(q), h, n)
            qv = q16[i, h * dh:(h + 1) * dh].astype(np.float64)
            sc = O.attn_decode_scores(qv, kh)
            assert np.all(np.diff(got) > 0) and got[0] >= 0 and got[-1] < n
            srt = np.sort(sc)[::-1]
            thr = srt[keep_n - 1]
            eps = 2e-5 * (1.0 + np.abs(sc).max())
            mask = np.zeros(n, bool)
            mask[got] = True
            assert sc[mask].min() >= thr - eps and (keep_n == n or sc[~mask].max() <= thr + eps)
            if keep_n == n or srt[keep_n - 1] - srt[keep_n] > 2 * eps:
                assert np.array_equal(got, O.topk_indices(sc, keep_n))
                exact += 1
            ref[i, h] = O.attn_decode_subset(qv, kh, vh, got.astype(np.int64))
    assert exact > 0
    assert_close(out, O.round_f16(ref), "paged top-k attention nh=%d dh=%d" % (nh, dh))
    assert not out[list(order).index(6)].any()          # the empty sequence


def _clear_topk_boundaries(ocfg, ow, x_rows, caches_loader, topk, rows_of, margin=1e-3):
    """True if, for every (row, head), the oracle's k-th and (k+1)-th largest scores are further apart
    than `margin` (relative to the score range): then both sides must keep the same rows and the layer
    outputs are comparable under the activation tolerance.  Oracle-side computation only."""
    y = O.round_f16(O.layernorm(x_rows.astype(np.float64), ow.ln1_g, ow.ln1_b, ocfg.ln_eps))
    qkv = O.round_f16(O.linear(y, ow.wqkv, ow.bqkv))
    for i in range(x_rows.shape[0]):
        n = rows_of(i)
        k = min(topk, n)
        if k >= n:
            continue
        for h in range(ocfg.nh):
            kh, _ = caches_loader(i, h, n)
            sc = np.sort(O.attn_decode_scores(qkv[i, h * ocfg.dh:(h + 1) * ocfg.dh], kh))[::-1]
            if sc[k - 1] - sc[k] <= margin * (1.0 + np.abs(sc).max()):
                return False
    return True


@pytest.mark.parametrize("paged", [False, True])
def test_decode_layer_with_topk_sparse_attention(paged):
    """fg_decode_layer / fg_decode_layer_paged with topk > 0 against the oracle's layer around the
    sparse attention of Section 5.  The cache is the oracle's (uploaded), the inputs are seeded, and
    the seed is one for which every head's selection boundary is clear in the oracle's own scores
    (asserted), so that both sides keep the same rows."""
    sh = synth.Shape(h1=512, nh=4, h2=1536, vocab=1000, max_pos=256)
    ocfg, cfg = cfg_pair(sh)
    t = synth.layer_tensors(sh, 3, 0, std=0.02, biases=True, random_ln=True)
    ow = oracle_layer(t, True)
    w = B.LayerWeights.from_numpy(t, True, tiled=True)
    topk = 9
    if paged:
        lens = [70, 5, 64, 130]                    # rows already cached per sequence (5 < topk: dense for that row)
        b = len(lens)
        table = _make_table([ln + 1 for ln in lens], 9, 3, seed=2)
        okv = O.PagedKVCache.empty(sh.nh, sh.dh, 9, table)
        for q, ln in enumerate(lens):
            okv.store(q, 0, _rand16((1, ln, sh.h1), 1.0, 10 + q), _rand16((1, ln, sh.h1), 1.0, 20 + q))
        pages = B.KVPages(cfg, 9, zero=False)
        _upload(pages, okv)
        seq_ids = np.array([2, 0, 3, 1], np.int32)
        pos = np.array([lens[q] for q in seq_ids], np.int32)
        xt = synth.activations_f16((b, sh.h1), 0.5, 31)
        ref = O.decode_layer_ragged(ocfg, ow, xt, seq_ids, pos, okv, topk=topk)
        assert _clear_topk_boundaries(ocfg, ow, xt, lambda i, h, n: okv.load(int(seq_ids[i]), h, n), topk,
                                      lambda i: int(pos[i]) + 1)
        got = B.fg_decode_layer_paged(cfg, w, dev(xt), pages, B.Ragged(dev(table), dev(seq_ids), dev(pos)), topk=topk)
        dense = B.fg_decode_layer_paged(cfg, w, dev(xt), pages, B.Ragged(dev(table), dev(seq_ids), dev(pos)))
    else:
        b, rows = 3, 75
        okv = O.KVCache.empty(b, sh.nh, rows + 1, sh.dh, True)
        okv.store(0, 0, _rand16((b, rows, sh.h1), 1.0, 40), _rand16((b, rows, sh.h1), 1.0, 41))
        kv = B.KVCache(cfg, b, rows + 1, True)
        kv.k_codes.copy_(dev(okv.k_codes)); kv.v_codes.copy_(dev(okv.v_codes))
        kv.k_meta.copy_(dev(okv.k_meta)); kv.v_meta.copy_(dev(okv.v_meta))
        xt = synth.activations_f16((b, sh.h1), 0.5, 49)
        ref = O.decode_layer(ocfg, ow, xt, rows, okv, topk=topk)
        assert _clear_topk_boundaries(ocfg, ow, xt, lambda i, h, n: okv.load(i, h, n), topk, lambda i: rows + 1)
        got = B.fg_decode_layer(cfg, w, dev(xt), rows, kv, topk=topk)
        kv.k_codes.copy_(dev(okv.k_codes)); kv.v_codes.copy_(dev(okv.v_codes))   # (the call above appended row `rows`)
        dense = B.fg_decode_layer(cfg, w, dev(xt), rows, kv)
    torch.cuda.synchronize()
    assert_close(host(got), ref, "decode layer with top-k attention (paged=%s)" % paged)
    assert not torch.equal(got, dense)             # the sparse attention really took part


# ------------------------------------------------------------------ FP16 rows in pages
@pytest.mark.parametrize("nh,dh", [(3, 128), (6, 64)])
def test_fp16_pages_append_bit_exact_and_attention(nh, dh):
    h1 = nh * dh
    cfg = B.Cfg(h1, nh, 4 * h1, 1000, 512)
    lens = [130, 5, 64, 65, 200, 0]
    b = len(lens)
    table = _make_table([ln + 1 for ln in lens], 14, 4, seed=nh)      # room for one more row each
    opaged = O.PagedKVCache.empty(nh, dh, 14, table, quantized=False)
    pages = B.KVPages(cfg, 14, quantized=False)
    dtab = dev(table)
    # whole histories, sequence by sequence (rows of different lengths: one call each)
    for q, ln in enumerate(lens):
        if not ln:
            continue
        kv16 = _rand16((ln, 2 * h1), 1.0, 30 + q)
        opaged.store(q, 0, kv16[:, :h1].reshape(1, ln, h1), kv16[:, h1:].reshape(1, ln, h1))
        d = dev(kv16)
        B.fg_kv_append_paged(cfg, d[:, :h1], d[:, h1:], 2 * h1, 1, ln, pages,
                             B.Ragged(dtab, dev(np.array([q], np.int32)), None))
    # a ragged step: one more row for three of the sequences, one of them the first row of a new page
    seq_ids = np.array([2, 0, 1], np.int32)
    pos = np.array([64, 130, 5], np.int32)
    row16 = _rand16((3, 2 * h1), 1.0, 77)
    for i, q in enumerate(seq_ids):
        opaged.store(int(q), int(pos[i]), row16[i:i + 1, :h1].reshape(1, 1, h1), row16[i:i + 1, h1:].reshape(1, 1, h1))
    d = dev(row16)
    B.fg_kv_append_paged(cfg, d[:, :h1], d[:, h1:], 2 * h1, 3, 1, pages, B.Ragged(dtab, dev(seq_ids), dev(pos)))
    torch.cuda.synchronize()
    assert np.array_equal(host(pages.k_codes), opaged.k_f16) and np.array_equal(host(pages.v_codes), opaged.v_f16)
    # attention over the pages, a length per sequence
    now = [ln + (1 if q in (0, 1, 2) else 0) for q, ln in enumerate(lens)]
    order = np.array([5, 3, 0, 4, 1, 2], np.int32)
    rows = np.array([now[q] for q in order], np.int32)
    q16 = _rand16((b, 3 * h1), 1.0, 78)
    ref = np.zeros((b, nh, dh))
    for i, q in enumerate(order):
        for h in range(nh):
            if rows[i]:
                kh, vh = opaged.load(int(q), h, int(rows[i]))
                ref[i, h] = O.attn_decode(q16[i, h * dh:(h + 1) * dh].astype(np.float64), kh, vh)
    out = B.fg_decode_attention_paged(cfg, dev(q16), 3 * h1, b, pages, B.Ragged(dtab, dev(order), dev(rows)), 0)
    torch.cuda.synchronize()
    out = host(out).reshape(b, nh, dh)
    assert_close(out, O.round_f16(ref), "decode attention over FP16 pages nh=%d dh=%d" % (nh, dh))
    assert not out[0].any()


def test_fp16_pages_layer_and_diagonal_generate():
    """FP16 weights and FP16 rows in pages through the paged layer calls and the diagonal driver."""
    sh = synth.Shape(h1=256, nh=4, h2=512, vocab=2000, max_pos=96, l=2)
    ocfg, cfg = cfg_pair(sh)
    olayers, layers = [], []
    for j in range(sh.l):
        t = synth.layer_tensors(sh, 17, j, std=0.08, biases=True, random_ln=True)
        olayers.append(oracle_layer(t, False))
        layers.append(B.LayerWeights.from_numpy(t, False))
    m = synth.model_tensors(sh, 17, std=0.08)
    n_seqs, gbs, s, n = 4, 2, 60, 7
    prompt = synth.prompt_ids(n_seqs, s, sh.vocab, 19)
    ref = O.generate(ocfg, olayers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, n, n_seqs // gbs, gbs, False)
    need = B.fg_diagonal_pages_needed(n_seqs, s, n, gbs)
    pages = [B.KVPages(cfg, need, quantized=False, zero=False) for _ in layers]
    ids, st = B.fg_generate_diagonal(cfg, layers, dev(m["embed"]), dev(m["pos"]), dev(m["lnf_g"]), dev(m["lnf_b"]),
                                     dev(prompt), n, gbs, pages)
    torch.cuda.synchronize()
    assert np.array_equal(host(ids), ref)          # FP16 caches: no quantization steps to amplify an ulp
