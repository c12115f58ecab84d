"""The C-ABI library loads, exports every symbol include/fg.h declares, and turns bad arguments
into error codes on the host before anything touches a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2303_06865_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "fg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fg_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared()
    assert "fg_quantize_groupwise" in names and "fg_prefill_layer" in names
    assert "fg_decode_layer" in names and "fg_generate" in names
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
        assert n in B.EXPORTS, "binding lacks " + n
    assert sorted(B.EXPORTS) == names


def test_struct_sizes_match_the_header_layout():
    assert C.sizeof(B.fg_mat) == 40
    assert C.sizeof(B.fg_model_cfg) == 24
    assert C.sizeof(B.fg_layer_weights) == 4 * 40 + 8 * 8
    assert C.sizeof(B.fg_kv_cache) == 48
    assert C.sizeof(B.fg_stats) == 48


def test_error_strings_and_version():
    L = B.lib()
    assert L.fg_version() >= 100
    assert L.fg_error_string(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert len(L.fg_error_string(code)) > 3
    assert [L.fg_kernel_class_name(i).decode() for i in range(len(B.KERNEL_CLASSES))] == B.KERNEL_CLASSES


def test_quantize_argument_errors_need_no_gpu():
    L = B.lib()
    p = C.c_void_p(16)   # never dereferenced: every call below fails validation first
    assert L.fg_quantize_groupwise(p, 4, 128, 32, 4, p, p, None) == B.FG_ERR_UNSUPPORTED
    assert L.fg_quantize_groupwise(p, 4, 128, 64, 3, p, p, None) == B.FG_ERR_UNSUPPORTED
    assert L.fg_quantize_groupwise(p, 4, 96, 64, 4, p, p, None) == B.FG_ERR_SHAPE
    assert L.fg_quantize_groupwise(p, -1, 128, 64, 4, p, p, None) == B.FG_ERR_SHAPE
    assert L.fg_quantize_groupwise(None, 4, 128, 64, 4, p, p, None) == B.FG_ERR_NULL
    assert L.fg_quantize_groupwise(p, 0, 128, 64, 4, p, p, None) == B.FG_OK      # empty input: no-op
    assert L.fg_dequantize_groupwise(p, p, 2, 100, p, None) == B.FG_ERR_SHAPE
    assert L.fg_layernorm(p, p, p, 2, 12, 1e-5, p, None) == B.FG_ERR_SHAPE


def _cfg(**kw):
    d = dict(h1=768, nh=12, h2=3072, vocab=50272, max_pos=2048, ln_eps=1e-5)
    d.update(kw)
    return B.fg_model_cfg(d["h1"], d["nh"], d["h2"], d["vocab"], d["max_pos"], d["ln_eps"])


def test_layer_argument_errors_need_no_gpu():
    L = B.lib()
    cfg = _cfg()
    a = 4096  # a fake, 16-byte aligned, never dereferenced address
    mat = lambda r, c, dt=B.FG_Q4G64: B.fg_mat(a, a, dt, 0, r, c)
    w = B.fg_layer_weights(mat(2304, 768), mat(768, 768), mat(3072, 768), mat(768, 3072), None, None, None, None,
                           a, a, a, a)
    kv = B.fg_kv_cache(a, a, a, a, B.FG_Q4G64, 4, 40, 0)
    ws = C.c_void_p(a)
    call = lambda cfg_, w_, kv_, b=4, t=32, ws_=ws, nws=1 << 40, topk=0: L.fg_decode_layer(
        C.byref(cfg_), C.byref(w_), a, b, t, topk, C.byref(kv_), 0, a, ws_, nws, None)
    assert call(_cfg(nh=5), w, kv) == B.FG_ERR_SHAPE            # h1 % nh != 0
    assert call(_cfg(h1=768, nh=3), w, kv) == B.FG_ERR_UNSUPPORTED   # head size 256
    assert call(cfg, w, kv, t=40) == B.FG_ERR_SHAPE             # t >= cap
    assert call(cfg, w, kv, b=5) == B.FG_ERR_SHAPE              # more sequences than the cache holds
    assert call(cfg, w, kv, nws=8) == B.FG_ERR_WORKSPACE
    assert call(cfg, w, kv, ws_=None) == B.FG_ERR_WORKSPACE
    bad = B.fg_layer_weights(mat(2304, 768), mat(768, 704), mat(3072, 768), mat(768, 3072), None, None, None, None,
                             a, a, a, a)
    assert call(cfg, bad, kv) == B.FG_ERR_SHAPE
    bad = B.fg_layer_weights(mat(2304, 768, 7), mat(768, 768), mat(3072, 768), mat(768, 3072), None, None, None,
                             None, a, a, a, a)
    assert call(cfg, bad, kv) == B.FG_ERR_UNSUPPORTED
    nometa = B.fg_kv_cache(a, None, a, a, B.FG_Q4G64, 4, 40, 0)
    assert call(cfg, w, nometa) == B.FG_ERR_NULL
    assert L.fg_decode_layer(None, C.byref(w), a, 4, 0, 0, C.byref(kv), 0, a, ws, 1 << 40, None) == B.FG_ERR_NULL
    assert call(cfg, w, kv, topk=-1) == B.FG_ERR_SHAPE
    f16kv = B.fg_kv_cache(a, None, a, None, B.FG_F16, 4, 40, 0)
    assert call(cfg, w, f16kv, topk=3) == B.FG_ERR_UNSUPPORTED      # sparse attention reads 4-bit caches only
    assert L.fg_prefill_layer(C.byref(cfg), C.byref(w), a, 4, 41, C.byref(kv), 0, a, ws, 1 << 40, None) == B.FG_ERR_SHAPE
    # generate: block must fit the caches, positions must exist
    larr = (B.fg_layer_weights * 1)(w)
    karr = (B.fg_kv_cache * 1)(kv)
    gen = lambda s, n, ngb, gbs, c=cfg: L.fg_generate(C.byref(c), 1, larr, a, a, a, a, a, s, n, ngb, gbs, karr, a, ws,
                                                      1 << 40, None, None)
    assert gen(32, 10, 1, 4) == B.FG_ERR_SHAPE       # needs cap >= 41
    assert gen(32, 9, 2, 4) == B.FG_ERR_SHAPE        # 8 sequences, cache holds 4
    assert gen(32, 9, 1, 4, _cfg(max_pos=39)) == B.FG_ERR_SHAPE
    assert gen(0, 9, 1, 4) == B.FG_ERR_SHAPE


def test_topk_attention_argument_errors_need_no_gpu():
    L = B.lib()
    cfg = _cfg()
    a = 4096
    kv = B.fg_kv_cache(a, a, a, a, B.FG_Q4G64, 4, 40, 0)
    call = lambda rows, topk, kv_=kv, b=4: L.fg_decode_attention_topk(C.byref(cfg), a, 2304, b, rows, topk,
                                                                      C.byref(kv_), 0, a, None, None)
    assert call(30, 0) == B.FG_ERR_SHAPE           # keep at least one row
    assert call(30, 31) == B.FG_ERR_SHAPE          # ... and at most all of them
    assert call(41, 4) == B.FG_ERR_SHAPE           # more rows than the cache holds
    assert call(30, 3, b=5) == B.FG_ERR_SHAPE
    f16 = B.fg_kv_cache(a, None, a, None, B.FG_F16, 4, 40, 0)
    assert call(30, 3, f16) == B.FG_ERR_UNSUPPORTED
    big = B.fg_kv_cache(a, a, a, a, B.FG_Q4G64, 4, 40000, 0)
    assert call(36800, 100, big) == B.FG_ERR_UNSUPPORTED   # scores of one head no longer fit on chip
    assert call(30, 3, b=0) == B.FG_OK


def test_workspace_queries_are_pure_host_functions():
    L = B.lib()
    cfg = _cfg()
    a = 4096
    mat = lambda r, c: B.fg_mat(a, a, B.FG_Q4G64, 0, r, c)
    w = B.fg_layer_weights(mat(2304, 768), mat(768, 768), mat(3072, 768), mat(768, 3072), None, None, None, None,
                           a, a, a, a)
    d = L.fg_layer_workspace_bytes(C.byref(cfg), C.byref(w), 4)
    p = L.fg_layer_workspace_bytes(C.byref(cfg), C.byref(w), 4 * 32)
    assert 0 < d and d <= p
    g = L.fg_workspace_bytes(C.byref(cfg), C.byref(w), 4, 1, 32)
    assert g >= p + 4 * 32 * 768 * 2 + 4 * 50272 * 4
    assert L.fg_workspace_bytes(C.byref(cfg), C.byref(w), 0, 1, 32) == 0


def test_paged_and_diagonal_argument_errors_need_no_gpu():
    L = B.lib()
    cfg = _cfg()
    a = 4096
    mat = lambda r, c, dt=B.FG_Q4G64: B.fg_mat(a, a, dt, 0, r, c)
    w = B.fg_layer_weights(mat(2304, 768), mat(768, 768), mat(3072, 768), mat(768, 3072), None, None, None, None,
                           a, a, a, a)
    assert C.sizeof(B.fg_kv_pages) == 40 and C.sizeof(B.fg_ragged) == 32
    pages = B.fg_kv_pages(a, a, a, a, B.FG_Q4G64, 8)
    seqs = B.fg_ragged(a, None, a, 2, 4)
    ws = C.c_void_p(a)
    att = lambda pg=pages, sq=seqs, b=4, bias=1, stride=2304: L.fg_decode_attention_paged(
        C.byref(cfg), a, stride, b, C.byref(pg), C.byref(sq), bias, a, None)
    assert att(pg=B.fg_kv_pages(a, a, a, a, 7, 8)) == B.FG_ERR_UNSUPPORTED            # unknown storage format
    assert att(pg=B.fg_kv_pages(a, None, a, None, B.FG_F16, 8), b=0) == B.FG_OK       # FP16 pages carry no pairs
    assert att(pg=B.fg_kv_pages(a, a, a, a, B.FG_Q4G64, 0)) == B.FG_ERR_SHAPE
    assert att(pg=B.fg_kv_pages(a, None, a, a, B.FG_Q4G64, 8)) == B.FG_ERR_NULL
    assert att(sq=B.fg_ragged(None, None, a, 2, 4)) == B.FG_ERR_NULL                  # no page table
    assert att(sq=B.fg_ragged(a, None, None, 2, 4)) == B.FG_ERR_NULL                  # no length per row
    assert att(sq=B.fg_ragged(a, None, a, 0, 4)) == B.FG_ERR_SHAPE
    assert att(bias=-1) == B.FG_ERR_SHAPE
    assert att(stride=700) == B.FG_ERR_SHAPE
    assert att(b=0) == B.FG_OK
    assert L.fg_kv_append_paged(C.byref(cfg), a, a, 2304, 4, -1, C.byref(pages), C.byref(seqs), None) == B.FG_ERR_SHAPE
    assert L.fg_kv_append_paged(C.byref(cfg), None, a, 2304, 4, 1, C.byref(pages), C.byref(seqs), None) == B.FG_ERR_NULL
    lay = lambda sq=seqs, nws=1 << 40, topk=0, pg=pages: L.fg_decode_layer_paged(
        C.byref(cfg), C.byref(w), a, 4, topk, C.byref(pg), C.byref(sq), a, ws, nws, None)
    assert lay(topk=-2) == B.FG_ERR_SHAPE
    assert lay(topk=3, pg=B.fg_kv_pages(a, None, a, None, B.FG_F16, 8)) == B.FG_ERR_UNSUPPORTED
    tk = lambda topk=3, pg=pages, sq=seqs, b=4: L.fg_decode_attention_topk_paged(
        C.byref(cfg), a, 2304, b, topk, C.byref(pg), C.byref(sq), 1, a, None, None)
    assert tk(topk=0) == B.FG_ERR_SHAPE
    assert tk(pg=B.fg_kv_pages(a, None, a, None, B.FG_F16, 8)) == B.FG_ERR_UNSUPPORTED
    assert tk(sq=B.fg_ragged(a, None, None, 2, 4)) == B.FG_ERR_NULL
    assert tk(b=0) == B.FG_OK
    assert lay(nws=8) == B.FG_ERR_WORKSPACE
    assert lay(sq=B.fg_ragged(a, None, None, 2, 4)) == B.FG_ERR_NULL                  # decode needs positions
    # a prompt longer than the page table can address
    assert L.fg_prefill_layer_paged(C.byref(cfg), C.byref(w), a, 4, 129, C.byref(pages), C.byref(seqs), a, ws, 1 << 40,
                                    None) == B.FG_ERR_SHAPE
    assert L.fg_embed_ragged(C.byref(cfg), a, a, a, None, 4, a, None) == B.FG_ERR_NULL
    # the schedule's page arithmetic is host-only: 4 batches of one sequence in flight at 70..73 rows
    assert L.fg_diagonal_pages_needed(4, 70, 4, 1) == 8
    # 4 batches of two, all in flight at the end (rows 64..67 -> the last three batches hold two pages each)
    assert L.fg_diagonal_pages_needed(8, 60, 8, 2) == 14
    assert L.fg_diagonal_pages_needed(4, 70, 4, 3) == -1                              # 4 % 3 != 0
    assert L.fg_diagonal_pages_needed(4, 0, 4, 1) == -1
    larr = (B.fg_layer_weights * 1)(w)
    parr = (B.fg_kv_pages * 1)(pages)
    gen = lambda n_seqs, s, n, gbs, nws=1 << 40: L.fg_generate_diagonal(C.byref(cfg), 1, larr, a, a, a, a, a, n_seqs, s,
                                                                        n, gbs, parr, a, ws, nws, None, None, None)
    assert gen(4, 70, 4, 3) == B.FG_ERR_SHAPE
    assert gen(4, 126, 4, 1) == B.FG_ERR_WORKSPACE     # rows 126..129 in flight: 9 pages, the pool has 8
    assert gen(4, 70, 4, 1, nws=8) == B.FG_ERR_WORKSPACE
    assert gen(4, 2040, 10, 1) == B.FG_ERR_SHAPE       # positions beyond max_pos
    assert L.fg_diagonal_workspace_bytes(C.byref(cfg), C.byref(w), 4, 70, 4, 1) > 0
    assert L.fg_diagonal_workspace_bytes(C.byref(cfg), C.byref(w), 4, 70, 4, 3) == 0


@pytest.mark.parametrize("h1,nh,h2,dtype", [(768, 12, 3072, B.FG_Q4G64_TILED), (12288, 96, 49152, B.FG_Q4G64_TILED),
                                            (768, 12, 3072, B.FG_Q4G64)])
def test_diagonal_workspace_covers_every_decode_row_count(h1, nh, h2, dtype):
    """The per-layer scratch of the diagonal driver must be large enough for EVERY row count an
    iteration can run, not only the largest: the partial-sum area of the projections depends on the
    tile shape picked for the row count (160 rows take more than 161..192).  Host arithmetic only:
    the driver's total must exceed the largest single need plus what it reserves besides."""
    L = B.lib()
    cfg = _cfg(h1=h1, nh=nh, h2=h2)
    a = 4096
    mat = lambda r, c: B.fg_mat(a, a, dtype, 0, r, c)
    w = B.fg_layer_weights(mat(3 * h1, h1), mat(h1, h1), mat(h2, h1), mat(h1, h2), None, None, None, None, a, a, a, a)
    n_seqs, s, n, gbs = 192, 16, 32, 8
    bmax = min(n_seqs // gbs, n - 1) * gbs
    assert bmax == 192
    need = [L.fg_layer_workspace_bytes(C.byref(cfg), C.byref(w), b) for b in range(gbs, bmax + 1, gbs)]
    need.append(L.fg_layer_workspace_bytes(C.byref(cfg), C.byref(w), gbs * s))
    if dtype == B.FG_Q4G64_TILED:
        # the case behind this test: the need is not monotone in the row count
        assert need[160 // gbs - 1] > need[192 // gbs - 1]
    total = L.fg_diagonal_workspace_bytes(C.byref(cfg), C.byref(w), n_seqs, s, n, gbs)
    other = gbs * s * h1 * 2 + bmax * h1 * 2 + bmax * 50272 * 4     # activations and logits it also holds
    assert total >= max(need) + other
