"""Pins for the oracle's paged cache, ragged decode step and diagonal-schedule generation (appendix,
"Diagonal block schedule").  None of these add arithmetic: they move rows and reorder independent work,
so each is pinned to the contiguous cache / block schedule it must agree with, plus brute-force
index checks of the documented page layout."""
import numpy as np
import pytest

from oracle import fg_oracle as O
from paper_2303_06865_amd import synth


def _rows16(shape, std, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(shape) * std).astype(np.float16)


@pytest.mark.parametrize("meta_f16", [False, True])
def test_paged_cache_is_a_relocation_of_the_contiguous_cache(meta_f16):
    nh, dh, h1 = 3, 64, 192
    lens = [130, 5, 64, 65]                       # 3, 1, 1 and 2 pages
    rng = np.random.default_rng(7)
    n_pages = 11
    perm = rng.permutation(n_pages)
    table = np.full((4, 3), -1, np.int32)
    nxt = 0
    for q, ln in enumerate(lens):
        for slot in range(-(-ln // O.PAGE_ROWS)):
            table[q, slot] = perm[nxt]
            nxt += 1
    used = set(int(p) for p in table.reshape(-1) if p >= 0)
    paged = O.PagedKVCache.empty(nh, dh, n_pages, table, meta_f16)
    flat = O.KVCache.empty(4, nh, 192, dh, True, meta_f16)
    data = {}
    for q, ln in enumerate(lens):
        k, v = _rows16((1, ln, h1), 1.0, 10 + q), _rows16((1, ln, h1), 0.5, 20 + q)
        data[q] = (k, v)
        # in two pieces, the second starting inside a page
        cut = ln // 3
        for lo, hi in ((0, cut), (cut, ln)):
            if hi > lo:
                paged.store(q, lo, k[:, lo:hi], v[:, lo:hi])
                flat.store(q, lo, k[:, lo:hi], v[:, lo:hi])
    for q, ln in enumerate(lens):
        for h in range(nh):
            kp, vp = paged.load(q, h, ln)
            kf, vf = flat.load(q, h, ln)
            assert np.array_equal(kp, kf) and np.array_equal(vp, vf)
    # where a row lives, element by element: position p of sequence q is row p % 64 of page table[q][p // 64]
    for q, p, h in ((0, 0, 0), (0, 63, 2), (0, 64, 1), (0, 129, 0), (3, 64, 2), (1, 4, 1)):
        page = table[q, p // 64]
        assert np.array_equal(paged.k_codes[page, h, p % 64], flat.k_codes[q, h, p])
        assert np.array_equal(paged.v_meta[page, h, p % 64], flat.v_meta[q, h, p])
    # pages nobody owns stay untouched, and rows past a sequence's end inside its last page too
    for page in range(n_pages):
        if page not in used:
            assert not paged.k_codes[page].any() and not paged.v_codes[page].any()
    assert not paged.k_codes[table[1, 0], :, 5:].any()
    with pytest.raises(AssertionError):
        paged.load(1, 0, 65)                      # sequence 1 has no second page


def test_fp16_pages_are_a_relocation_of_the_contiguous_fp16_cache():
    """Unquantized pages: the rows come back bit for bit, and land where the page layout says."""
    nh, dh, h1 = 2, 64, 128
    lens = [70, 3, 64]
    table = np.array([[3, 0], [4, -1], [1, -1]], np.int32)
    paged = O.PagedKVCache.empty(nh, dh, 5, table, quantized=False)
    flat = O.KVCache.empty(3, nh, 80, dh, False)
    for q, ln in enumerate(lens):
        k, v = _rows16((1, ln, h1), 1.0, 60 + q), _rows16((1, ln, h1), 0.5, 70 + q)
        paged.store(q, 0, k, v)
        flat.store(q, 0, k, v)
        for h in range(nh):
            kp, vp = paged.load(q, h, ln)
            assert np.array_equal(kp, k[0, :, h * dh:(h + 1) * dh].astype(np.float64))
            assert np.array_equal(vp, flat.load(q, h, ln)[1])
    assert np.array_equal(paged.k_f16[0, 1, 5], flat.k_f16[0, 1, 69])      # position 69 = row 5 of its second page
    assert not paged.k_f16[2].any() and not paged.v_f16[4, :, 3:].any()   # page 2 is nobody's; rows past the end


def test_decode_layer_with_topk_is_the_layer_around_sparse_attention():
    """decode_layer(topk=k) must be the dense layer with the attention of every (sequence, head)
    replaced by Section 5's sparse form.  Checked without the oracle's own top-k routine: the kept rows
    are found by a plain Python sort of (score descending, row ascending), the layer around it is
    re-assembled from the pinned pieces; and topk >= rows is the dense layer itself."""
    sh, cfg, layers, _ = _tiny_model(l=1)
    w = layers[0]
    b, t, k_keep = 2, 37, 5
    kv = O.KVCache.empty(b, sh.nh, t + 1, sh.dh, True)
    kv.store(0, 0, _rows16((b, t, sh.h1), 1.0, 80), _rows16((b, t, sh.h1), 1.0, 81))
    import copy
    kv_dense, kv_all = copy.deepcopy(kv), copy.deepcopy(kv)
    x = _rows16((b, sh.h1), 0.5, 82)
    got = O.decode_layer(cfg, w, x, t, kv, topk=k_keep)
    dense = O.decode_layer(cfg, w, x, t, kv_dense)
    assert np.array_equal(O.decode_layer(cfg, w, x, t, kv_all, topk=t + 1), dense)
    assert not np.array_equal(got, dense)
    assert np.array_equal(kv.k_codes, kv_dense.k_codes)                    # the cache write does not depend on topk
    # by hand
    y = O.round_f16(O.layernorm(x.astype(np.float64), w.ln1_g, w.ln1_b, cfg.ln_eps))
    qkv = O.round_f16(O.linear(y, w.wqkv, w.bqkv))
    o = np.zeros((b, sh.nh, sh.dh))
    for bi in range(b):
        for h in range(sh.nh):
            kh, vh = kv.load(bi, h, t + 1)
            q = qkv[bi, h * sh.dh:(h + 1) * sh.dh]
            sc = [float(sum(q[d] * kh[j, d] for d in range(sh.dh))) / np.sqrt(sh.dh) for j in range(t + 1)]
            keep = sorted(sorted(range(t + 1), key=lambda j: (-sc[j], j))[:k_keep])
            mx = max(sc)
            den = sum(np.exp(v - mx) for v in sc)                          # the FULL softmax denominator
            for j in keep:
                o[bi, h] += np.exp(sc[j] - mx) / den * vh[j]
    o = O.round_f16(o.reshape(b, sh.h1))
    x1 = O.round_f16(O.linear(o, w.wo, w.bo) + x.astype(np.float64))
    y2 = O.round_f16(O.layernorm(x1, w.ln2_g, w.ln2_b, cfg.ln_eps))
    a = O.round_f16(np.maximum(O.linear(y2, w.w1, w.b1), 0.0))
    ref = O.round_f16(O.linear(a, w.w2, w.b2) + x1).astype(np.float16)
    assert np.array_equal(got, ref)


def _tiny_model(l=2, seed=0, max_pos=96):
    sh = synth.Shape(h1=128, nh=2, h2=256, vocab=211, max_pos=max_pos, l=l)
    cfg = O.ModelCfg(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos)
    layers = []
    for j in range(l):
        t = synth.layer_tensors(sh, seed, j, std=0.08, biases=True, random_ln=True)
        layers.append(O.LayerWeights(
            wqkv=O.Mat.from_f16(t["wqkv"], True), wo=O.Mat.from_f16(t["wo"], True),
            w1=O.Mat.from_f16(t["w1"], True), w2=O.Mat.from_f16(t["w2"], True),
            ln1_g=t["ln1_g"], ln1_b=t["ln1_b"], ln2_g=t["ln2_g"], ln2_b=t["ln2_b"],
            bqkv=t["bqkv"], bo=t["bo"], b1=t["b1"], b2=t["b2"]))
    m = synth.model_tensors(sh, seed, std=0.08)
    return sh, cfg, layers, m


def test_ragged_decode_step_equals_each_sequence_decoded_alone():
    """Three sequences at positions 3, 64 and 70 in one ragged step over a paged cache give, row for
    row, what decode_layer gives for each of them alone over a contiguous cache with the same history."""
    sh, cfg, layers, _ = _tiny_model(l=1)
    w = layers[0]
    pos = [3, 64, 70]
    table = np.array([[4, -1], [0, 3], [2, 1]], np.int32)
    paged = O.PagedKVCache.empty(sh.nh, sh.dh, 5, table)
    flats = []
    for q, t in enumerate(pos):
        k, v = _rows16((1, t, sh.h1), 1.0, 30 + q), _rows16((1, t, sh.h1), 1.0, 40 + q)
        paged.store(q, 0, k, v)
        f = O.KVCache.empty(1, sh.nh, t + 1, sh.dh, True)
        f.store(0, 0, k, v)
        flats.append(f)
    x = _rows16((3, sh.h1), 0.5, 50)
    # rows given in another order than the sequence ids
    order = [2, 0, 1]
    out = O.decode_layer_ragged(cfg, w, x[order], order, [pos[q] for q in order], paged)
    for i, q in enumerate(order):
        ref = O.decode_layer(cfg, w, x[q:q + 1], pos[q], flats[q])[0]
        assert np.array_equal(out[i], ref)
        kp, vp = paged.load(q, 1, pos[q] + 1)
        kf, vf = flats[q].load(0, 1, pos[q] + 1)
        assert np.array_equal(kp, kf) and np.array_equal(vp, vf)   # the appended row landed in the right page


@pytest.mark.parametrize("n_seqs,gbs,s,n", [(6, 2, 5, 4),      # fewer batches than steps: all in flight together
                                            (5, 1, 6, 2),      # more batches than steps: pages are recycled
                                            (2, 1, 62, 5)])    # a sequence grows across a page boundary
def test_diagonal_schedule_emits_the_tokens_of_the_block_schedule(n_seqs, gbs, s, n):
    sh, cfg, layers, m = _tiny_model(l=2, seed=3)
    prompt = synth.prompt_ids(n_seqs, s, sh.vocab, 5)
    ref = O.generate(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, n, n_seqs // gbs, gbs, True)
    got = O.generate_diagonal(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, n, gbs)
    assert got.dtype == np.int32 and np.array_equal(got, ref)


def test_diagonal_schedule_peak_pages_match_the_staggered_lengths():
    """With one batch admitted per iteration the batches in flight hold s+1 .. s+n rows (one each, once
    the pipeline is full), so the pages in use peak at sum_a ceil((s + a) / 64) per sequence slot of the
    batch, which is below the block schedule's n * ceil((s + n) / 64) as soon as lengths straddle a page."""
    sh, cfg, layers, m = _tiny_model(l=1, seed=4, max_pos=96)
    s, n, gbs, ng = 60, 8, 1, 10
    prompt = synth.prompt_ids(ng * gbs, s, sh.vocab, 6)
    ids, peak = O.generate_diagonal(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, n, gbs,
                                    return_page_use=True)
    # rows held while an iteration runs: the admitted batch s, a batch at step a has s + a (a = 1 .. n-1)
    expect = sum(-(-(s + a) // 64) for a in range(n)) * gbs
    assert peak == expect
    assert peak < n * gbs * -(-(s + n) // 64)
    ref = O.generate(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, n, ng, gbs, True)
    assert np.array_equal(ids, ref)
