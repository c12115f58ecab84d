"""ctypes binding of libfg.so: same names as the C ABI in include/fg.h.

Argument marshalling only.  Every step of the path runs in the library's HIP kernels; PyTorch is
used to own device memory and to supply the current stream.  There is no fallback: if the shared
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

FG_OK = 0
FG_ERR_NULL, FG_ERR_SHAPE, FG_ERR_UNSUPPORTED, FG_ERR_WORKSPACE, FG_ERR_DEVICE = -1, -2, -3, -4, -5
FG_F16, FG_Q4G64, FG_Q4G64_TILED, FG_Q4G64_H16, FG_Q4G64_H16_TILED = 0, 1, 2, 3, 4
KERNEL_CLASSES = ["quantize", "dequantize", "layernorm", "gemm_small_m", "gemm_small_m_finish", "gemm_large_m",
                  "kv_append", "attn_decode", "attn_prefill", "embed", "argmax"]

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfg.so")


class fg_mat(C.Structure):
    _fields_ = [("data", C.c_void_p), ("meta", C.c_void_p), ("dtype", C.c_int32), ("reserved", C.c_int32),
                ("rows", C.c_int64), ("cols", C.c_int64)]


class fg_model_cfg(C.Structure):
    _fields_ = [("h1", C.c_int32), ("nh", C.c_int32), ("h2", C.c_int32), ("vocab", C.c_int32),
                ("max_pos", C.c_int32), ("ln_eps", C.c_float)]


class fg_layer_weights(C.Structure):
    _fields_ = [("wqkv", fg_mat), ("wo", fg_mat), ("w1", fg_mat), ("w2", fg_mat),
                ("bqkv", C.c_void_p), ("bo", C.c_void_p), ("b1", C.c_void_p), ("b2", C.c_void_p),
                ("ln1_g", C.c_void_p), ("ln1_b", C.c_void_p), ("ln2_g", C.c_void_p), ("ln2_b", C.c_void_p)]


class fg_kv_cache(C.Structure):
    _fields_ = [("k_codes", C.c_void_p), ("k_meta", C.c_void_p), ("v_codes", C.c_void_p), ("v_meta", C.c_void_p),
                ("dtype", C.c_int32), ("batch", C.c_int32), ("cap", C.c_int32), ("reserved", C.c_int32)]


class fg_kv_pages(C.Structure):
    _fields_ = [("k_codes", C.c_void_p), ("k_meta", C.c_void_p), ("v_codes", C.c_void_p), ("v_meta", C.c_void_p),
                ("dtype", C.c_int32), ("n_pages", C.c_int32)]


class fg_ragged(C.Structure):
    _fields_ = [("page_table", C.c_void_p), ("seq_ids", C.c_void_p), ("pos", C.c_void_p),
                ("table_stride", C.c_int32), ("n_seqs", C.c_int32)]


class fg_stats(C.Structure):
    _fields_ = [("prefill_s", C.c_double), ("decode_s", C.c_double), ("tokens", C.c_int64),
                ("weight_bytes_per_step", C.c_int64), ("kv_bytes_last_step", C.c_int64),
                ("decode_step_s", C.POINTER(C.c_double))]


EXPORTS = {
    "fg_error_string": (C.c_char_p, [C.c_int]),
    "fg_last_device_error": (C.c_char_p, []),
    "fg_version": (C.c_int, []),
    "fg_quantize_groupwise": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                        C.c_void_p]),
    "fg_quantize_groupwise_h16": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_void_p,
                                            C.c_void_p, C.c_void_p]),
    "fg_pack_weights": (C.c_int, [C.POINTER(fg_mat), C.c_void_p, C.c_void_p, C.c_void_p]),
    "fg_dequantize_groupwise": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "fg_dequantize_groupwise_h16": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "fg_layernorm": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_float, C.c_void_p,
                               C.c_void_p]),
    "fg_linear": (C.c_int, [C.POINTER(fg_mat), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int, C.c_void_p,
                            C.c_void_p, C.c_size_t, C.c_void_p]),
    "fg_linear_workspace_bytes": (C.c_size_t, [C.POINTER(fg_mat), C.c_int64]),
    "fg_linear_static": (C.c_int, [C.POINTER(fg_mat), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int, C.c_void_p,
                                   C.c_void_p]),
    "fg_linear_static_scratch_bytes": (C.c_size_t, []),
    "fg_kv_append": (C.c_int, [C.POINTER(fg_model_cfg), C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                               C.POINTER(fg_kv_cache), C.c_int32, C.c_int32, C.c_void_p]),
    "fg_decode_attention": (C.c_int, [C.POINTER(fg_model_cfg), C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                      C.POINTER(fg_kv_cache), C.c_int32, C.c_void_p, C.c_void_p]),
    "fg_decode_attention_topk": (C.c_int, [C.POINTER(fg_model_cfg), C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                           C.c_int32, C.POINTER(fg_kv_cache), C.c_int32, C.c_void_p, C.c_void_p,
                                           C.c_void_p]),
    "fg_prefill_attention": (C.c_int, [C.POINTER(fg_model_cfg), C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                       C.c_void_p]),
    "fg_embed": (C.c_int, [C.POINTER(fg_model_cfg), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                           C.c_int32, C.c_void_p, C.c_void_p]),
    "fg_lm_head_greedy": (C.c_int, [C.POINTER(fg_model_cfg), C.c_void_p, C.c_int64, C.c_int64, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                    C.c_size_t, C.c_void_p]),
    "fg_lm_head_workspace_bytes": (C.c_size_t, [C.POINTER(fg_model_cfg), C.c_int64]),
    "fg_prefill_layer": (C.c_int, [C.POINTER(fg_model_cfg), C.POINTER(fg_layer_weights), C.c_void_p, C.c_int32,
                                   C.c_int32, C.POINTER(fg_kv_cache), C.c_int32, C.c_void_p, C.c_void_p,
                                   C.c_size_t, C.c_void_p]),
    "fg_decode_layer": (C.c_int, [C.POINTER(fg_model_cfg), C.POINTER(fg_layer_weights), C.c_void_p, C.c_int32,
                                  C.c_int32, C.c_int32, C.POINTER(fg_kv_cache), C.c_int32, C.c_void_p, C.c_void_p,
                                  C.c_size_t, C.c_void_p]),
    "fg_layer_workspace_bytes": (C.c_size_t, [C.POINTER(fg_model_cfg), C.POINTER(fg_layer_weights), C.c_int64]),
    "fg_generate": (C.c_int, [C.POINTER(fg_model_cfg), C.c_int32, C.POINTER(fg_layer_weights), C.c_void_p,
                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                              C.c_int32, C.POINTER(fg_kv_cache), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p,
                              C.POINTER(fg_stats)]),
    "fg_workspace_bytes": (C.c_size_t, [C.POINTER(fg_model_cfg), C.POINTER(fg_layer_weights), C.c_int32,
                                        C.c_int32, C.c_int32]),
    "fg_kv_append_paged": (C.c_int, [C.POINTER(fg_model_cfg), C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                     C.POINTER(fg_kv_pages), C.POINTER(fg_ragged), C.c_void_p]),
    "fg_decode_attention_paged": (C.c_int, [C.POINTER(fg_model_cfg), C.c_void_p, C.c_int64, C.c_int32,
                                            C.POINTER(fg_kv_pages), C.POINTER(fg_ragged), C.c_int32, C.c_void_p,
                                            C.c_void_p]),
    "fg_decode_layer_paged": (C.c_int, [C.POINTER(fg_model_cfg), C.POINTER(fg_layer_weights), C.c_void_p, C.c_int32,
                                        C.c_int32, C.POINTER(fg_kv_pages), C.POINTER(fg_ragged), C.c_void_p, C.c_void_p,
                                        C.c_size_t, C.c_void_p]),
    "fg_decode_attention_topk_paged": (C.c_int, [C.POINTER(fg_model_cfg), C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                                 C.POINTER(fg_kv_pages), C.POINTER(fg_ragged), C.c_int32, C.c_void_p,
                                                 C.c_void_p, C.c_void_p]),
    "fg_prefill_layer_paged": (C.c_int, [C.POINTER(fg_model_cfg), C.POINTER(fg_layer_weights), C.c_void_p, C.c_int32,
                                         C.c_int32, C.POINTER(fg_kv_pages), C.POINTER(fg_ragged), C.c_void_p,
                                         C.c_void_p, C.c_size_t, C.c_void_p]),
    "fg_embed_ragged": (C.c_int, [C.POINTER(fg_model_cfg), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                  C.c_void_p, C.c_void_p]),
    "fg_generate_diagonal": (C.c_int, [C.POINTER(fg_model_cfg), C.c_int32, C.POINTER(fg_layer_weights), C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                       C.c_int32, C.POINTER(fg_kv_pages), C.c_void_p, C.c_void_p, C.c_size_t,
                                       C.c_void_p, C.POINTER(fg_stats), C.POINTER(C.c_int32)]),
    "fg_diagonal_workspace_bytes": (C.c_size_t, [C.POINTER(fg_model_cfg), C.POINTER(fg_layer_weights), C.c_int32,
                                                 C.c_int32, C.c_int32, C.c_int32]),
    "fg_diagonal_pages_needed": (C.c_int64, [C.c_int32, C.c_int32, C.c_int32, C.c_int32]),
    "fg_profile_begin": (C.c_int, []),
    "fg_profile_begin_classes": (C.c_int, [C.c_uint32]),
    "fg_profile_end": (C.c_int, []),
    "fg_profile_read": (C.c_int, [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "fg_kernel_class_name": (C.c_char_p, [C.c_int]),
}

_lib = None


def lib() -> C.CDLL:
    """Load libfg.so (built by paper_2303_06865_amd.build); fails loudly when it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libfg.so is not built: run `python -m paper_2303_06865_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


class FgError(RuntimeError):
    def __init__(self, status: int, where: str):
        L = lib()
        msg = L.fg_error_string(status).decode()
        if status == FG_ERR_DEVICE:
            msg += ": " + L.fg_last_device_error().decode()
        super().__init__("%s failed: %s (%d)" % (where, msg, status))
        self.status = status


def _check(status: int, where: str) -> None:
    if status != FG_OK:
        raise FgError(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _p(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _f16(t: torch.Tensor) -> torch.Tensor:
    assert t.dtype == torch.float16 and t.is_cuda and t.is_contiguous()
    return t


# ------------------------------------------------------------------ containers (own the tensors)
class Mat:
    """Device weight matrix [rows, cols] in FG_F16 or FG_Q4G64 storage."""

    def __init__(self, rows: int, cols: int, dtype: int, data: torch.Tensor, meta: Optional[torch.Tensor]):
        self.rows, self.cols, self.dtype, self.data, self.meta = rows, cols, dtype, data, meta
        self.c = fg_mat(_p(data), _p(meta), dtype, 0, rows, cols)

    @staticmethod
    def from_f16(w: torch.Tensor, quantize: bool, tiled: bool = False, meta_f16: bool = False) -> "Mat":
        """quantize: store as 4-bit groups of 64 (quantized on the GPU); tiled: additionally reorder
        into the streaming layout with fg_pack_weights (rows must be a multiple of 32); meta_f16: the
        {min, scale} pairs are FP16 (only the tiled form of such a matrix can be multiplied)."""
        w = _f16(w)
        r, c = w.shape
        if quantize:
            codes, meta = fg_quantize_groupwise(w, meta_f16=meta_f16)
            m = Mat(r, c, FG_Q4G64_H16 if meta_f16 else FG_Q4G64, codes, meta)
            return m.tiled() if tiled else m
        return Mat(r, c, FG_F16, w, None)

    def tiled(self) -> "Mat":
        assert self.dtype in (FG_Q4G64, FG_Q4G64_H16)
        data = torch.empty_like(self.data)
        meta = torch.empty_like(self.meta)
        _check(lib().fg_pack_weights(C.byref(self.c), _p(data), _p(meta), _stream()), "fg_pack_weights")
        return Mat(self.rows, self.cols, FG_Q4G64_TILED if self.dtype == FG_Q4G64 else FG_Q4G64_H16_TILED, data, meta)

    def nbytes(self) -> int:
        return self.data.numel() * self.data.element_size() + (0 if self.meta is None else self.meta.numel() * self.meta.element_size())


class Cfg:
    def __init__(self, h1: int, nh: int, h2: int, vocab: int, max_pos: int, ln_eps: float = 1e-5):
        self.h1, self.nh, self.h2, self.vocab, self.max_pos, self.ln_eps = h1, nh, h2, vocab, max_pos, ln_eps
        self.dh = h1 // nh
        self.c = fg_model_cfg(h1, nh, h2, vocab, max_pos, ln_eps)


class LayerWeights:
    def __init__(self, wqkv: Mat, wo: Mat, w1: Mat, w2: Mat, ln1_g, ln1_b, ln2_g, ln2_b, bqkv=None, bo=None, b1=None,
                 b2=None):
        self.keep = [wqkv, wo, w1, w2, ln1_g, ln1_b, ln2_g, ln2_b, bqkv, bo, b1, b2]
        self.wqkv, self.wo, self.w1, self.w2 = wqkv, wo, w1, w2
        self.c = fg_layer_weights(wqkv.c, wo.c, w1.c, w2.c, _p(bqkv), _p(bo), _p(b1), _p(b2), _p(ln1_g), _p(ln1_b),
                                  _p(ln2_g), _p(ln2_b))

    @staticmethod
    def from_numpy(t: Dict, quantize: bool, device="cuda", tiled: bool = False, meta_f16: bool = False) -> "LayerWeights":
        """t: FP16 numpy tensors as made by synth.layer_tensors; weights are quantized on the GPU."""
        d = lambda a: None if a is None else torch.from_numpy(a).to(device)
        mk = lambda a: Mat.from_f16(d(a), quantize, tiled, meta_f16 and quantize)
        return LayerWeights(mk(t["wqkv"]), mk(t["wo"]), mk(t["w1"]), mk(t["w2"]),
                            d(t["ln1_g"]), d(t["ln1_b"]), d(t["ln2_g"]), d(t["ln2_b"]),
                            d(t.get("bqkv")), d(t.get("bo")), d(t.get("b1")), d(t.get("b2")))

    def nbytes(self) -> int:
        return self.wqkv.nbytes() + self.wo.nbytes() + self.w1.nbytes() + self.w2.nbytes()


class KVCache:
    """One layer's cache, logical layout [batch, nh, cap, dh]."""

    def __init__(self, cfg: Cfg, batch: int, cap: int, quantized: bool, device="cuda", zero: bool = True,
                 meta_f16: bool = False):
        """quantized: 4-bit storage; meta_f16 (quantized only): FP16 {min, scale} pairs (FG_Q4G64_H16)."""
        self.batch, self.cap, self.quantized = batch, cap, quantized
        self.meta_f16 = bool(meta_f16 and quantized)
        mk = torch.zeros if zero else torch.empty
        nh, dh = cfg.nh, cfg.dh
        if quantized:
            self.k_codes = mk((batch, nh, cap, dh // 2), dtype=torch.uint8, device=device)
            self.v_codes = mk((batch, nh, cap, dh // 2), dtype=torch.uint8, device=device)
            mt = torch.float16 if self.meta_f16 else torch.float32
            self.k_meta = mk((batch, nh, cap, dh // 64, 2), dtype=mt, device=device)
            self.v_meta = mk((batch, nh, cap, dh // 64, 2), dtype=mt, device=device)
        else:
            self.k_codes = mk((batch, nh, cap, dh), dtype=torch.float16, device=device)
            self.v_codes = mk((batch, nh, cap, dh), dtype=torch.float16, device=device)
            self.k_meta = self.v_meta = None
        self.c = fg_kv_cache(_p(self.k_codes), _p(self.k_meta), _p(self.v_codes), _p(self.v_meta),
                             (FG_Q4G64_H16 if self.meta_f16 else FG_Q4G64) if quantized else FG_F16, batch, cap, 0)

    def nbytes(self) -> int:
        n = 2 * self.k_codes.numel() * self.k_codes.element_size()
        if self.k_meta is not None:
            n += 2 * self.k_meta.numel() * self.k_meta.element_size()
        return n


PAGE_ROWS = 64


class KVPages:
    """One layer's 4-bit cache as a pool of pages of 64 positions: [n_pages, nh, 64, dh/2] codes and
    [n_pages, nh, 64, dh/64, 2] {min, scale} pairs (binary32, or FP16 with meta_f16)."""

    def __init__(self, cfg: Cfg, n_pages: int, meta_f16: bool = False, device="cuda", zero: bool = True,
                 quantized: bool = True):
        """quantized = False: the pages hold plain FP16 rows [n_pages, nh, 64, dh] (FG_F16)."""
        self.n_pages, self.meta_f16, self.quantized = n_pages, bool(meta_f16 and quantized), quantized
        mk = torch.zeros if zero else torch.empty
        nh, dh = cfg.nh, cfg.dh
        if not quantized:
            self.k_codes = mk((n_pages, nh, PAGE_ROWS, dh), dtype=torch.float16, device=device)
            self.v_codes = mk((n_pages, nh, PAGE_ROWS, dh), dtype=torch.float16, device=device)
            self.k_meta = self.v_meta = None
            self.c = fg_kv_pages(_p(self.k_codes), None, _p(self.v_codes), None, FG_F16, n_pages)
            return
        mt = torch.float16 if meta_f16 else torch.float32
        self.k_codes = mk((n_pages, nh, PAGE_ROWS, dh // 2), dtype=torch.uint8, device=device)
        self.v_codes = mk((n_pages, nh, PAGE_ROWS, dh // 2), dtype=torch.uint8, device=device)
        self.k_meta = mk((n_pages, nh, PAGE_ROWS, dh // 64, 2), dtype=mt, device=device)
        self.v_meta = mk((n_pages, nh, PAGE_ROWS, dh // 64, 2), dtype=mt, device=device)
        self.c = fg_kv_pages(_p(self.k_codes), _p(self.k_meta), _p(self.v_codes), _p(self.v_meta),
                             FG_Q4G64_H16 if meta_f16 else FG_Q4G64, n_pages)

    def nbytes(self) -> int:
        n = 2 * self.k_codes.numel() * self.k_codes.element_size()
        return n if self.k_meta is None else n + 2 * self.k_meta.numel() * self.k_meta.element_size()


class Ragged:
    """Rows of a ragged step: page_table int32 [n_seqs, table_stride], seq_ids int32 [b] or None
    (identity), pos int32 [b] or None (zeros); all on the device."""

    def __init__(self, page_table: torch.Tensor, seq_ids: Optional[torch.Tensor] = None,
                 pos: Optional[torch.Tensor] = None):
        for t in (page_table, seq_ids, pos):
            assert t is None or (t.dtype == torch.int32 and t.is_cuda and t.is_contiguous())
        self.page_table, self.seq_ids, self.pos = page_table, seq_ids, pos
        self.c = fg_ragged(_p(page_table), _p(seq_ids), _p(pos), page_table.shape[1], page_table.shape[0])


def _ws(nbytes: int, device="cuda") -> Optional[torch.Tensor]:
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


# ------------------------------------------------------------------ calls
def fg_version() -> int:
    return lib().fg_version()


def fg_quantize_groupwise(x: torch.Tensor, group: int = 64, bits: int = 4, meta_f16: bool = False):
    """meta_f16: the 4.5-bit variant with FP16 {min, scale} pairs (fg_quantize_groupwise_h16)."""
    x = _f16(x)
    rows, cols = x.shape
    codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device)
    meta = torch.empty((rows, cols // 64, 2), dtype=torch.float16 if meta_f16 else torch.float32, device=x.device)
    fn = lib().fg_quantize_groupwise_h16 if meta_f16 else lib().fg_quantize_groupwise
    _check(fn(_p(x), rows, cols, group, bits, _p(codes), _p(meta), _stream()), "fg_quantize_groupwise")
    return codes, meta


def fg_dequantize_groupwise(codes: torch.Tensor, meta: torch.Tensor) -> torch.Tensor:
    rows, half = codes.shape
    out = torch.empty((rows, half * 2), dtype=torch.float32, device=codes.device)
    fn = lib().fg_dequantize_groupwise_h16 if meta.dtype == torch.float16 else lib().fg_dequantize_groupwise
    _check(fn(_p(codes), _p(meta), rows, half * 2, _p(out), _stream()), "fg_dequantize_groupwise")
    return out


def fg_layernorm(x: torch.Tensor, gamma: torch.Tensor, beta: torch.Tensor, eps: float) -> torch.Tensor:
    x = _f16(x)
    rows, cols = x.shape
    out = torch.empty_like(x)
    _check(lib().fg_layernorm(_p(x), _p(gamma), _p(beta), rows, cols, eps, _p(out), _stream()), "fg_layernorm")
    return out


def fg_linear(w: Mat, bias: Optional[torch.Tensor], x: torch.Tensor, residual: Optional[torch.Tensor] = None,
              relu: bool = False) -> torch.Tensor:
    x = _f16(x)
    m = x.shape[0]
    assert x.shape[1] == w.cols
    out = torch.empty((m, w.rows), dtype=torch.float16, device=x.device)
    nws = lib().fg_linear_workspace_bytes(C.byref(w.c), m)
    ws = _ws(nws)
    _check(lib().fg_linear(C.byref(w.c), _p(bias), _p(x), m, _p(residual), int(relu), _p(out), _p(ws), nws,
                           _stream()), "fg_linear")
    return out


def fg_linear_static(w: Mat, bias: Optional[torch.Tensor], x: torch.Tensor, residual: Optional[torch.Tensor],
                     relu: bool, out: torch.Tensor) -> torch.Tensor:
    """fg_linear on the library's own scratch array: the caller passes inputs and the output, nothing
    is allocated here or in the library."""
    _check(lib().fg_linear_static(C.byref(w.c), _p(bias), _p(x), x.shape[0], _p(residual), int(relu), _p(out),
                                  _stream()), "fg_linear_static")
    return out


def fg_kv_append(cfg: Cfg, k: torch.Tensor, v: torch.Tensor, row_stride: int, b: int, s: int, kv: KVCache,
                 batch_offset: int, pos0: int) -> None:
    _check(lib().fg_kv_append(C.byref(cfg.c), _p(k), _p(v), row_stride, b, s, C.byref(kv.c), batch_offset, pos0,
                              _stream()), "fg_kv_append")


def fg_decode_attention(cfg: Cfg, q: torch.Tensor, q_row_stride: int, b: int, rows: int, kv: KVCache,
                        batch_offset: int = 0) -> torch.Tensor:
    out = torch.empty((b, cfg.h1), dtype=torch.float16, device=q.device)
    _check(lib().fg_decode_attention(C.byref(cfg.c), _p(q), q_row_stride, b, rows, C.byref(kv.c), batch_offset,
                                     _p(out), _stream()), "fg_decode_attention")
    return out


def fg_decode_attention_topk(cfg: Cfg, q: torch.Tensor, q_row_stride: int, b: int, rows: int, topk: int, kv: KVCache,
                             batch_offset: int = 0, want_rows: bool = False):
    """Returns out [b, h1] (and the kept row indices int32 [b, nh, topk] if want_rows)."""
    out = torch.empty((b, cfg.h1), dtype=torch.float16, device=q.device)
    kept = torch.empty((b, cfg.nh, topk), dtype=torch.int32, device=q.device) if want_rows else None
    _check(lib().fg_decode_attention_topk(C.byref(cfg.c), _p(q), q_row_stride, b, rows, topk, C.byref(kv.c),
                                          batch_offset, _p(out), _p(kept), _stream()), "fg_decode_attention_topk")
    return (out, kept) if want_rows else out


def fg_prefill_attention(cfg: Cfg, qkv: torch.Tensor, b: int, s: int) -> torch.Tensor:
    qkv = _f16(qkv)
    out = torch.empty((b * s, cfg.h1), dtype=torch.float16, device=qkv.device)
    _check(lib().fg_prefill_attention(C.byref(cfg.c), _p(qkv), b, s, _p(out), _stream()), "fg_prefill_attention")
    return out


def fg_embed(cfg: Cfg, embed: torch.Tensor, pos: torch.Tensor, ids: torch.Tensor, s_len: int, pos0: int):
    rows = ids.numel()
    out = torch.empty((rows, cfg.h1), dtype=torch.float16, device=ids.device)
    _check(lib().fg_embed(C.byref(cfg.c), _p(embed), _p(pos), _p(ids), rows, s_len, pos0, _p(out), _stream()),
           "fg_embed")
    return out


def fg_lm_head_greedy(cfg: Cfg, x: torch.Tensor, lnf_g, lnf_b, embed: torch.Tensor):
    """Returns (ids int32 [rows], logits float32 [rows, vocab])."""
    x = _f16(x)
    rows = x.shape[0]
    ids = torch.empty((rows,), dtype=torch.int32, device=x.device)
    logits = torch.empty((rows, cfg.vocab), dtype=torch.float32, device=x.device)
    nws = lib().fg_lm_head_workspace_bytes(C.byref(cfg.c), rows)
    ws = _ws(nws)
    _check(lib().fg_lm_head_greedy(C.byref(cfg.c), _p(x), cfg.h1, rows, _p(lnf_g), _p(lnf_b), _p(embed), _p(ids), 1,
                                   _p(logits), _p(ws), nws, _stream()), "fg_lm_head_greedy")
    return ids, logits


def fg_prefill_layer(cfg: Cfg, w: LayerWeights, x: torch.Tensor, kv: KVCache, batch_offset: int = 0,
                     ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    x = _f16(x)
    b, s, _ = x.shape
    out = torch.empty_like(x)
    nws = lib().fg_layer_workspace_bytes(C.byref(cfg.c), C.byref(w.c), b * s)
    if ws is None:
        ws = _ws(nws)
    _check(lib().fg_prefill_layer(C.byref(cfg.c), C.byref(w.c), _p(x), b, s, C.byref(kv.c), batch_offset, _p(out),
                                  _p(ws), ws.numel(), _stream()), "fg_prefill_layer")
    return out


def fg_decode_layer(cfg: Cfg, w: LayerWeights, x: torch.Tensor, t: int, kv: KVCache, batch_offset: int = 0,
                    ws: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None, topk: int = 0) -> torch.Tensor:
    x = _f16(x)
    b = x.shape[0]
    if out is None:
        out = torch.empty_like(x)
    if ws is None:
        ws = _ws(lib().fg_layer_workspace_bytes(C.byref(cfg.c), C.byref(w.c), b))
    _check(lib().fg_decode_layer(C.byref(cfg.c), C.byref(w.c), _p(x), b, t, topk, C.byref(kv.c), batch_offset, _p(out),
                                 _p(ws), ws.numel(), _stream()), "fg_decode_layer")
    return out


def fg_kv_append_paged(cfg: Cfg, k: torch.Tensor, v: torch.Tensor, row_stride: int, b: int, s: int, pages: KVPages,
                       seqs: Ragged) -> None:
    _check(lib().fg_kv_append_paged(C.byref(cfg.c), _p(k), _p(v), row_stride, b, s, C.byref(pages.c), C.byref(seqs.c),
                                    _stream()), "fg_kv_append_paged")


def fg_decode_attention_paged(cfg: Cfg, q: torch.Tensor, q_row_stride: int, b: int, pages: KVPages, seqs: Ragged,
                              rows_bias: int = 0) -> torch.Tensor:
    out = torch.empty((b, cfg.h1), dtype=torch.float16, device=q.device)
    _check(lib().fg_decode_attention_paged(C.byref(cfg.c), _p(q), q_row_stride, b, C.byref(pages.c), C.byref(seqs.c),
                                           rows_bias, _p(out), _stream()), "fg_decode_attention_paged")
    return out


def fg_decode_attention_topk_paged(cfg: Cfg, q: torch.Tensor, q_row_stride: int, b: int, topk: int, pages: KVPages,
                                   seqs: Ragged, rows_bias: int = 0, want_rows: bool = False):
    """Returns out [b, h1] (and the kept positions int32 [b, nh, topk], -1 padded, if want_rows)."""
    out = torch.empty((b, cfg.h1), dtype=torch.float16, device=q.device)
    kept = torch.empty((b, cfg.nh, topk), dtype=torch.int32, device=q.device) if want_rows else None
    _check(lib().fg_decode_attention_topk_paged(C.byref(cfg.c), _p(q), q_row_stride, b, topk, C.byref(pages.c),
                                                C.byref(seqs.c), rows_bias, _p(out), _p(kept), _stream()),
           "fg_decode_attention_topk_paged")
    return (out, kept) if want_rows else out


def fg_decode_layer_paged(cfg: Cfg, w: LayerWeights, x: torch.Tensor, pages: KVPages, seqs: Ragged,
                          ws: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                          topk: int = 0) -> torch.Tensor:
    x = _f16(x)
    b = x.shape[0]
    if out is None:
        out = torch.empty_like(x)
    if ws is None:
        ws = _ws(lib().fg_layer_workspace_bytes(C.byref(cfg.c), C.byref(w.c), b))
    _check(lib().fg_decode_layer_paged(C.byref(cfg.c), C.byref(w.c), _p(x), b, topk, C.byref(pages.c), C.byref(seqs.c),
                                       _p(out), _p(ws), ws.numel(), _stream()), "fg_decode_layer_paged")
    return out


def fg_prefill_layer_paged(cfg: Cfg, w: LayerWeights, x: torch.Tensor, pages: KVPages, seqs: Ragged,
                           ws: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    x = _f16(x)
    b, s, _ = x.shape
    if out is None:
        out = torch.empty_like(x)
    if ws is None:
        ws = _ws(lib().fg_layer_workspace_bytes(C.byref(cfg.c), C.byref(w.c), b * s))
    _check(lib().fg_prefill_layer_paged(C.byref(cfg.c), C.byref(w.c), _p(x), b, s, C.byref(pages.c), C.byref(seqs.c),
                                        _p(out), _p(ws), ws.numel(), _stream()), "fg_prefill_layer_paged")
    return out


def fg_embed_ragged(cfg: Cfg, emb: torch.Tensor, pos_table: torch.Tensor, ids: torch.Tensor,
                    positions: torch.Tensor) -> torch.Tensor:
    rows = ids.numel()
    out = torch.empty((rows, cfg.h1), dtype=torch.float16, device=ids.device)
    _check(lib().fg_embed_ragged(C.byref(cfg.c), _p(emb), _p(pos_table), _p(ids), _p(positions), rows, _p(out),
                                 _stream()), "fg_embed_ragged")
    return out


def fg_workspace_bytes(cfg: Cfg, layer0: LayerWeights, gpu_batch_size: int, num_gpu_batches: int, s: int) -> int:
    return lib().fg_workspace_bytes(C.byref(cfg.c), C.byref(layer0.c), gpu_batch_size, num_gpu_batches, s)


def fg_generate(cfg: Cfg, layers: Sequence[LayerWeights], embed: torch.Tensor, pos: torch.Tensor, lnf_g, lnf_b,
                prompt: torch.Tensor, n: int, num_gpu_batches: int, gpu_batch_size: int, kv: Sequence[KVCache],
                ws: Optional[torch.Tensor] = None, out_ids: Optional[torch.Tensor] = None, want_stats: bool = True):
    """Returns (ids int32 [bls, n], stats dict or None)."""
    assert prompt.dtype == torch.int32 and prompt.is_cuda and prompt.is_contiguous()
    bls, s = prompt.shape
    l = len(layers)
    larr = (fg_layer_weights * l)(*[w.c for w in layers])
    karr = (fg_kv_cache * l)(*[k.c for k in kv])
    if out_ids is None:
        out_ids = torch.zeros((bls, n), dtype=torch.int32, device=prompt.device)
    if ws is None:
        ws = _ws(fg_workspace_bytes(cfg, layers[0], gpu_batch_size, num_gpu_batches, s))
    stats = None
    steps = None
    if want_stats:
        steps = (C.c_double * max(n - 1, 1))()
        stats = fg_stats(0.0, 0.0, 0, 0, 0, C.cast(steps, C.POINTER(C.c_double)))
    _check(lib().fg_generate(C.byref(cfg.c), l, larr, _p(embed), _p(pos), _p(lnf_g), _p(lnf_b), _p(prompt), s, n,
                             num_gpu_batches, gpu_batch_size, karr, _p(out_ids), _p(ws), ws.numel(), _stream(),
                             C.byref(stats) if stats is not None else None), "fg_generate")
    sd = None
    if stats is not None:
        sd = {"prefill_s": stats.prefill_s, "decode_s": stats.decode_s, "tokens": stats.tokens,
              "weight_bytes_per_step": stats.weight_bytes_per_step, "kv_bytes_last_step": stats.kv_bytes_last_step,
              "decode_step_s": [steps[i] for i in range(n - 1)]}
    return out_ids, sd


def fg_diagonal_pages_needed(n_seqs: int, s: int, n: int, gpu_batch_size: int) -> int:
    return lib().fg_diagonal_pages_needed(n_seqs, s, n, gpu_batch_size)


def fg_generate_diagonal(cfg: Cfg, layers: Sequence[LayerWeights], embed: torch.Tensor, pos: torch.Tensor, lnf_g, lnf_b,
                         prompt: torch.Tensor, n: int, gpu_batch_size: int, pages: Sequence[KVPages],
                         ws: Optional[torch.Tensor] = None, out_ids: Optional[torch.Tensor] = None):
    """Returns (ids int32 [n_seqs, n], {"total_s", "tokens", "peak_pages"})."""
    assert prompt.dtype == torch.int32 and prompt.is_cuda and prompt.is_contiguous()
    n_seqs, s = prompt.shape
    l = len(layers)
    larr = (fg_layer_weights * l)(*[w.c for w in layers])
    parr = (fg_kv_pages * l)(*[p.c for p in pages])
    if out_ids is None:
        out_ids = torch.zeros((n_seqs, n), dtype=torch.int32, device=prompt.device)
    if ws is None:
        ws = _ws(lib().fg_diagonal_workspace_bytes(C.byref(cfg.c), C.byref(layers[0].c), n_seqs, s, n, gpu_batch_size))
    stats = fg_stats(0.0, 0.0, 0, 0, 0, None)
    peak = C.c_int32(0)
    _check(lib().fg_generate_diagonal(C.byref(cfg.c), l, larr, _p(embed), _p(pos), _p(lnf_g), _p(lnf_b), _p(prompt),
                                      n_seqs, s, n, gpu_batch_size, parr, _p(out_ids), _p(ws), ws.numel(), _stream(),
                                      C.byref(stats), C.byref(peak)), "fg_generate_diagonal")
    return out_ids, {"total_s": stats.decode_s, "tokens": stats.tokens, "peak_pages": peak.value}


def fg_profile_begin(classes: Optional[Sequence[str]] = None) -> None:
    """classes: names from KERNEL_CLASSES to time (None = all of them)."""
    if classes is None:
        _check(lib().fg_profile_begin(), "fg_profile_begin")
        return
    mask = 0
    for name in classes:
        mask |= 1 << KERNEL_CLASSES.index(name)
    _check(lib().fg_profile_begin_classes(mask), "fg_profile_begin_classes")


def fg_profile_end() -> Dict[str, Dict[str, float]]:
    """Stops timing and returns {kernel class: {"ms": total GPU ms, "launches": n}}."""
    _check(lib().fg_profile_end(), "fg_profile_end")
    out = {}
    for k, name in enumerate(KERNEL_CLASSES):
        ms, n = C.c_double(0), C.c_int64(0)
        lib().fg_profile_read(k, C.byref(ms), C.byref(n))
        if n.value:
            out[name] = {"ms": ms.value, "launches": n.value}
    return out
