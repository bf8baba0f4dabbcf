"""ctypes binding over the C ABI in include/unique.h -- argument marshalling only.

Every function has the name of the C entry point without the ``unique_`` prefix and
passes ``tensor.data_ptr()`` / the current torch HIP stream straight through. torch is
used for device memory and streams; every step of the computation runs in the HIP library.
There is no fallback: if the library is missing and cannot be built, ``load()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import build as _build

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, 1, 2, 3, 4
DTYPE_CODE = {torch.float32: 0, torch.bfloat16: 1}

EXPORTS = ("unique_workspace_bytes", "unique_page_stats_record_bytes", "unique_update_page_stats", "unique_score_select_topk",
           "unique_page_scores", "unique_select_topk", "unique_decode_step", "unique_decode_step_static", "unique_sparse_paged_decode", "unique_dense_paged_decode", "unique_status_string",
           "unique_last_error", "unique_version")


class CacheDesc(C.Structure):
    """Mirror of ``unique_cache_desc``."""
    _fields_ = [("dtype", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("page_size", C.c_int32), ("batch", C.c_int32),
                ("max_pages_per_seq", C.c_int32), ("max_seq_len_hint", C.c_int32),
                ("num_phys_pages", C.c_int64), ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
                ("page_stats", C.c_void_p), ("page_table", C.c_void_p), ("seq_lens", C.c_void_p),
                ("stats_dtype", C.c_int32), ("force_recent_pages", C.c_int32),
                ("kv_page_stride", C.c_int64), ("kv_head_stride", C.c_int64),
                ("min_seq_len_hint", C.c_int32), ("reserved0", C.c_int32)]


class UniqueError(RuntimeError):
    def __init__(self, code: int, status: str, detail: str):
        super().__init__(f"unique status {code} ({status}): {detail}")
        self.code = code


def _p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0)


class Library:
    def __init__(self, path: str):
        self.path = path
        self.c = C.CDLL(path)
        for name in EXPORTS:
            getattr(self.c, name)  # raises AttributeError if a declared symbol is not exported
        for name in ("unique_status_string", "unique_last_error", "unique_version"):
            getattr(self.c, name).restype = C.c_char_p
        self.c.unique_status_string.argtypes = [C.c_int]
        self.c.unique_workspace_bytes.argtypes = [C.POINTER(CacheDesc), C.c_int32, C.POINTER(C.c_size_t)]
        self.c.unique_page_stats_record_bytes.argtypes = [C.POINTER(CacheDesc)]
        self.c.unique_page_stats_record_bytes.restype = C.c_int64
        self.c.unique_update_page_stats.argtypes = [C.POINTER(CacheDesc), C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        self.c.unique_score_select_topk.argtypes = [C.POINTER(CacheDesc), C.c_void_p, C.c_int32, C.c_float,
                                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                                    C.c_void_p]
        self.c.unique_page_scores.argtypes = [C.POINTER(CacheDesc), C.c_void_p, C.c_float, C.c_void_p, C.c_int32,
                                              C.c_void_p]
        self.c.unique_select_topk.argtypes = [C.POINTER(CacheDesc), C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                              C.c_void_p, C.c_void_p]
        self.c.unique_sparse_paged_decode.argtypes = [C.POINTER(CacheDesc), C.c_void_p, C.c_void_p, C.c_void_p,
                                                      C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p,
                                                      C.c_size_t, C.c_void_p]
        self.c.unique_decode_step.argtypes = [C.POINTER(CacheDesc), C.c_void_p, C.c_int32, C.c_float, C.c_float,
                                              C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_size_t, C.c_void_p]
        self.c.unique_decode_step_static.argtypes = [C.POINTER(CacheDesc), C.c_void_p, C.c_int32, C.c_float, C.c_float,
                                                     C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                     C.c_void_p]
        self.c.unique_dense_paged_decode.argtypes = [C.POINTER(CacheDesc), C.c_void_p, C.c_float, C.c_void_p,
                                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]

    # -- helpers -----------------------------------------------------------------------------
    def check(self, rc: int) -> None:
        if rc != OK:
            raise UniqueError(rc, self.c.unique_status_string(rc).decode(), self.c.unique_last_error().decode())

    def version(self) -> str:
        return self.c.unique_version().decode()

    def last_error(self) -> str:
        return self.c.unique_last_error().decode()

    def status_string(self, rc: int) -> str:
        return self.c.unique_status_string(rc).decode()

    # -- the ABI, one method per entry point ---------------------------------------------------
    def workspace_bytes(self, desc: CacheDesc, top_k: int) -> int:
        n = C.c_size_t(0)
        self.check(self.c.unique_workspace_bytes(C.byref(desc), top_k, C.byref(n)))
        return int(n.value)

    def page_stats_record_bytes(self, desc: CacheDesc) -> int:
        return int(self.c.unique_page_stats_record_bytes(C.byref(desc)))

    def update_page_stats(self, desc: CacheDesc, tok_begin=None, tok_end=None, max_pages_touched_per_seq: int = 0):
        self.check(self.c.unique_update_page_stats(C.byref(desc), _p(tok_begin), _p(tok_end),
                                                   max_pages_touched_per_seq, _stream()))

    def score_select_topk(self, desc: CacheDesc, q, top_k: int, lam: float, sel_pages, sel_count, scores_out,
                          workspace):
        self.check(self.c.unique_score_select_topk(C.byref(desc), _p(q), top_k, lam, _p(sel_pages), _p(sel_count),
                                                   _p(scores_out), _p(workspace),
                                                   workspace.numel() * workspace.element_size(), _stream()))

    def page_scores(self, desc: CacheDesc, q, lam: float, scores):
        self.check(self.c.unique_page_scores(C.byref(desc), _p(q), lam, _p(scores), int(scores.shape[-1]), _stream()))

    def select_topk(self, desc: CacheDesc, scores, top_k: int, sel_pages, sel_count):
        self.check(self.c.unique_select_topk(C.byref(desc), _p(scores), int(scores.shape[-1]), top_k, _p(sel_pages),
                                             _p(sel_count), _stream()))

    def sparse_paged_decode(self, desc: CacheDesc, q, sel_pages, sel_count, sel_stride: int, sm_scale: float, out,
                            lse_out, workspace):
        self.check(self.c.unique_sparse_paged_decode(C.byref(desc), _p(q), _p(sel_pages), _p(sel_count), sel_stride,
                                                     sm_scale, _p(out), _p(lse_out), _p(workspace),
                                                     workspace.numel() * workspace.element_size(), _stream()))

    def decode_step(self, desc: CacheDesc, q, top_k: int, lam: float, sm_scale: float, refresh_tail: bool, sel_pages,
                    sel_count, out, lse_out, workspace):
        self.check(self.c.unique_decode_step(C.byref(desc), _p(q), top_k, lam, sm_scale, int(refresh_tail),
                                             _p(sel_pages), _p(sel_count), _p(out), _p(lse_out), _p(workspace),
                                             workspace.numel() * workspace.element_size(), _stream()))

    def decode_step_static(self, desc: CacheDesc, q, top_k: int, lam: float, sm_scale: float, refresh_tail: bool,
                           sel_pages, sel_count, out, lse_out):
        self.check(self.c.unique_decode_step_static(C.byref(desc), _p(q), top_k, lam, sm_scale, int(refresh_tail),
                                                    _p(sel_pages), _p(sel_count), _p(out), _p(lse_out), _stream()))

    def dense_paged_decode(self, desc: CacheDesc, q, sm_scale: float, out, lse_out, workspace):
        self.check(self.c.unique_dense_paged_decode(C.byref(desc), _p(q), sm_scale, _p(out), _p(lse_out),
                                                    _p(workspace), workspace.numel() * workspace.element_size(),
                                                    _stream()))


_lib: Library | None = None


def load() -> Library:
    """Open the built library (building it first only if no built library exists)."""
    global _lib
    if _lib is None:
        path = _build.LIB_PATH
        if not os.path.exists(path):
            path = _build.build_library()
        _lib = Library(path)
    return _lib


STATIC_SCRATCH_BYTES = 8 << 20  # UNIQUE_STATIC_SCRATCH_BYTES
STD_BLOCK_BYTES = 128  # bytes after the means in a page_stats record (fp32 stds + pad)


def stats_record_bytes(num_kv_heads: int, head_dim: int, stats_dtype) -> int:
    return num_kv_heads * head_dim * (2 if stats_dtype == torch.bfloat16 else 4) + STD_BLOCK_BYTES


def make_desc(*, q_heads: int, k_cache, v_cache, page_stats, page_table, seq_lens,
              max_seq_len_hint: int = 0, stats_dtype=torch.float32, force_recent_pages: int = 0,
              min_seq_len_hint: int = 0) -> CacheDesc:
    """Fill a ``unique_cache_desc`` from tensors laid out as include/unique.h describes (shape checks only)."""
    P, Hkv, S, D = k_cache.shape
    # the (S, D) tile of one (page, head) must be contiguous; page and head strides are passed through
    assert k_cache.dtype in DTYPE_CODE and k_cache.stride()[2:] == (D, 1)
    assert v_cache is None or (v_cache.shape == k_cache.shape and v_cache.dtype == k_cache.dtype
                               and v_cache.stride() == k_cache.stride())
    assert page_table.dtype == torch.int32 and page_table.is_contiguous() and page_table.dim() == 2
    assert seq_lens.dtype == torch.int32 and seq_lens.shape == (page_table.shape[0],)
    if page_stats is not None:
        assert page_stats.dtype == torch.uint8 and page_stats.is_contiguous()
        assert page_stats.shape == (P, stats_record_bytes(Hkv, D, stats_dtype))
    return CacheDesc(DTYPE_CODE[k_cache.dtype], q_heads, Hkv, D, S, page_table.shape[0], page_table.shape[1],
                     max_seq_len_hint, P, k_cache.data_ptr(), 0 if v_cache is None else v_cache.data_ptr(),
                     0 if page_stats is None else page_stats.data_ptr(),
                     page_table.data_ptr(), seq_lens.data_ptr(), DTYPE_CODE[stats_dtype], int(force_recent_pages),
                     k_cache.stride(0), k_cache.stride(1), int(min_seq_len_hint), 0)
