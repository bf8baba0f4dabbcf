"""float64 CPU oracle for UNIQUE decode-time sparse attention -- TEST INFRASTRUCTURE ONLY.

Thin ctypes binding over ``unique_oracle.c`` (plain C, double arithmetic), which
transcribes Section 3.1 (paging, Eq. 1, Eq. 2, Eq. 3), and Section 3.2 (Eq. 4,
Eq. 5, Eq. 6 and the top-k page set) of the paper. Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may use
this package; the GPU library never does, and this package imports nothing of it.

All functions take numpy arrays: caches and queries as float32, or as uint16
holding bf16 bit patterns; results are float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "unique_oracle.c")
_LIB = os.path.join(_HERE, "libunique_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over rows in the batch drivers)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Cache(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("H", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("S", C.c_int32), ("B", C.c_int32), ("max_pages_per_seq", C.c_int32),
                ("num_phys_pages", C.c_int64), ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
                ("page_table", C.c_void_p), ("seq_lens", C.c_void_p)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        for name in ("oracle_page_stats", "oracle_page_scores", "oracle_topk", "oracle_attention",
                     "oracle_update_stats", "oracle_sparse_decode_step", "oracle_dense_decode",
                     "oracle_attention_rows", "oracle_num_threads"):
            getattr(_lib, name).restype = C.c_int
        _lib.oracle_round_bf16.restype = None
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _ptr(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


@dataclass
class OracleCache:
    """Host view of a paged KV cache, layout [num_phys_pages][Hkv][S][D]."""
    k_cache: np.ndarray
    v_cache: np.ndarray
    page_table: np.ndarray  # int32 [B][max_pages_per_seq]
    seq_lens: np.ndarray    # int32 [B]
    H: int

    def __post_init__(self):
        assert self.k_cache.ndim == 4 and self.k_cache.shape == self.v_cache.shape
        assert self.k_cache.dtype in (np.float32, np.uint16) and self.v_cache.dtype == self.k_cache.dtype
        assert self.k_cache.flags.c_contiguous and self.v_cache.flags.c_contiguous
        self.page_table = np.ascontiguousarray(self.page_table, dtype=np.int32)
        self.seq_lens = np.ascontiguousarray(self.seq_lens, dtype=np.int32)
        self.num_phys_pages, self.Hkv, self.S, self.D = (int(x) for x in self.k_cache.shape)
        self.B, self.max_pages = (int(x) for x in self.page_table.shape)
        assert self.H % self.Hkv == 0 and self.seq_lens.shape == (self.B,)
        self.G = self.H // self.Hkv
        self.is_bf16 = self.k_cache.dtype == np.uint16
        # host-side sanity: every page the oracle can touch exists
        for b in range(self.B):
            P = self.num_pages(b)
            assert 0 <= P <= self.max_pages
            if P:
                row = self.page_table[b, :P]
                assert row.min() >= 0 and row.max() < self.num_phys_pages
        self._c = _Cache(1 if self.is_bf16 else 0, self.H, self.Hkv, self.D, self.S, self.B,
                         self.max_pages, self.num_phys_pages, self.k_cache.ctypes.data,
                         self.v_cache.ctypes.data, self.page_table.ctypes.data, self.seq_lens.ctypes.data)

    def num_pages(self, b: int) -> int:
        return (int(self.seq_lens[b]) + self.S - 1) // self.S

    def _check_q(self, q: np.ndarray):
        assert q.shape == (self.B, self.H, self.D) and q.dtype == self.k_cache.dtype and q.flags.c_contiguous


def page_stats(c: OracleCache, b: int, hkv: int, p0: int = 0, p1: int | None = None):
    """Eq. 1 / Eq. 2 for logical pages [p0, p1) of (b, hkv) -> (mean [n, D], std [n])."""
    p1 = c.num_pages(b) if p1 is None else p1
    n = max(p1 - p0, 0)
    mean = np.zeros((n, c.D), np.float64)
    std = np.zeros((n,), np.float64)
    rc = _load().oracle_page_stats(C.byref(c._c), b, hkv, p0, p1, _ptr(mean), _ptr(std))
    if rc != 0:
        raise ValueError("oracle_page_stats: bad (b, hkv, page range)")
    return mean, std


def page_scores(c: OracleCache, q: np.ndarray, b: int, hkv: int, lam: float,
                mean: np.ndarray, std: np.ndarray) -> np.ndarray:
    """Eq. 6 (Eq. 3 for G = 1) from the given page statistics -> scores [n]."""
    c._check_q(q)
    mean = np.ascontiguousarray(mean, np.float64)
    std = np.ascontiguousarray(std, np.float64)
    assert mean.shape == (std.shape[0], c.D)
    scores = np.zeros((std.shape[0],), np.float64)
    rc = _load().oracle_page_scores(C.byref(c._c), _ptr(q), b, hkv, C.c_double(lam), std.shape[0],
                                    _ptr(mean), _ptr(std), _ptr(scores))
    if rc != 0:
        raise ValueError("oracle_page_scores: bad (b, hkv)")
    return scores


def topk(scores: np.ndarray, k: int):
    """Ranking by (score desc, index asc) -> (order [P], k_b = min(k, P)); the set is order[:k_b]."""
    scores = np.ascontiguousarray(scores, np.float64)
    order = np.zeros((scores.shape[0],), np.int32)
    kb = _load().oracle_topk(_ptr(scores), scores.shape[0], k, _ptr(order))
    return order, int(kb)


def topk_forced(scores: np.ndarray, k: int, force_recent: int):
    """Selection with the always-keep option of the C ABI (a serving option, not part of the paper: Section 4.3
    states that the method needs no local window, so force_recent = 0 is the paper's behaviour). The last
    n = min(force_recent, k, P) logical pages are selected whatever their scores; the other min(k, P) - n places
    go to the best of the remaining pages under the (score desc, index asc) ranking.
    -> ascending int32 array of min(k, P) pages."""
    scores = np.ascontiguousarray(scores, np.float64)
    P = scores.shape[0]
    kb = min(int(k), P)
    n = min(int(force_recent), kb)
    forced = np.arange(P - n, P, dtype=np.int64)
    rest = np.zeros((0,), np.int64)
    if kb - n > 0:
        order, _ = topk(scores[:P - n], kb - n)
        rest = order[:kb - n].astype(np.int64)
    return np.sort(np.concatenate([rest, forced])).astype(np.int32)


def attention(c: OracleCache, q: np.ndarray, b: int, h: int, pages, sm_scale: float = 0.0):
    """Eq. 5 over the given logical pages (Eq. 4 if they are all pages) -> (out [D], lse)."""
    c._check_q(q)
    pages = np.ascontiguousarray(pages, np.int32)
    out = np.zeros((c.D,), np.float64)
    lse = C.c_double(0.0)
    rc = _load().oracle_attention(C.byref(c._c), _ptr(q), b, h, _ptr(pages), pages.shape[0],
                                  C.c_double(sm_scale), _ptr(out), C.byref(lse))
    if rc != 0:
        raise ValueError(f"oracle_attention failed with {rc}")
    return out, float(lse.value)


def dense_attention(c: OracleCache, q: np.ndarray, b: int, h: int, sm_scale: float = 0.0):
    """Eq. 4: attention over every page of sequence b."""
    return attention(c, q, b, h, np.arange(c.num_pages(b), dtype=np.int32), sm_scale)


def new_stat_cache(c: OracleCache):
    """Logical stat cache: mean [B][Hkv][max_pages][D], std [B][Hkv][max_pages] (float64)."""
    return (np.zeros((c.B, c.Hkv, c.max_pages, c.D), np.float64),
            np.zeros((c.B, c.Hkv, c.max_pages), np.float64))


def update_stats(c: OracleCache, mean_all: np.ndarray, std_all: np.ndarray,
                 tok_begin: np.ndarray | None = None, tok_end: np.ndarray | None = None) -> None:
    """Refresh the stats of every page overlapping [tok_begin[b], tok_end[b]) (None = all pages)."""
    assert mean_all.shape == (c.B, c.Hkv, c.max_pages, c.D) and mean_all.dtype == np.float64
    assert std_all.shape == (c.B, c.Hkv, c.max_pages) and std_all.dtype == np.float64
    if tok_begin is not None:
        tok_begin = np.ascontiguousarray(tok_begin, np.int32)
        tok_end = np.ascontiguousarray(tok_end, np.int32)
    rc = _load().oracle_update_stats(C.byref(c._c), _ptr(tok_begin), _ptr(tok_end), _ptr(mean_all), _ptr(std_all))
    if rc != 0:
        raise ValueError("oracle_update_stats failed")


def sparse_decode_step(c: OracleCache, q: np.ndarray, mean_all: np.ndarray, std_all: np.ndarray,
                       lam: float, top_k: int, sm_scale: float = 0.0, want_scores: bool = True):
    """Scores (Eq. 6) -> top-k set -> Eq. 5, for the whole batch, from cached stats.

    Returns dict(sel [B,Hkv,top_k] ascending, -1 padded; sel_count [B,Hkv];
    scores [B,Hkv,max_pages] or None; out [B,H,D]; lse [B,H])."""
    c._check_q(q)
    sel = np.full((c.B, c.Hkv, top_k), -1, np.int32)
    cnt = np.zeros((c.B, c.Hkv), np.int32)
    scores = np.full((c.B, c.Hkv, c.max_pages), -np.inf, np.float64) if want_scores else None
    out = np.zeros((c.B, c.H, c.D), np.float64)
    lse = np.zeros((c.B, c.H), np.float64)
    rc = _load().oracle_sparse_decode_step(C.byref(c._c), _ptr(q), _ptr(mean_all), _ptr(std_all),
                                           C.c_double(lam), top_k, C.c_double(sm_scale), _ptr(sel),
                                           _ptr(cnt), _ptr(scores), _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError(f"oracle_sparse_decode_step failed with {rc}")
    return dict(sel=sel, sel_count=cnt, scores=scores, out=out, lse=lse)


def dense_decode(c: OracleCache, q: np.ndarray, sm_scale: float = 0.0):
    """Eq. 4 for every (b, h) -> (out [B,H,D], lse [B,H])."""
    c._check_q(q)
    out = np.zeros((c.B, c.H, c.D), np.float64)
    lse = np.zeros((c.B, c.H), np.float64)
    rc = _load().oracle_dense_decode(C.byref(c._c), _ptr(q), C.c_double(sm_scale), _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError(f"oracle_dense_decode failed with {rc}")
    return out, lse


def attention_rows(c: OracleCache, q: np.ndarray, sel: np.ndarray, sel_count: np.ndarray, sm_scale: float = 0.0):
    """Eq. 5 for every (b, h) over the given page lists: sel int32 [B, Hkv, stride] (the first sel_count[b, hkv]
    entries of a row are used) -> (out [B, H, D], lse [B, H]); an empty row gives zeros and lse = -inf."""
    c._check_q(q)
    sel = np.ascontiguousarray(sel, np.int32)
    sel_count = np.ascontiguousarray(sel_count, np.int32)
    assert sel.shape[:2] == (c.B, c.Hkv) and sel_count.shape == (c.B, c.Hkv)
    assert int(sel_count.max(initial=0)) <= sel.shape[2]
    out = np.zeros((c.B, c.H, c.D), np.float64)
    lse = np.zeros((c.B, c.H), np.float64)
    rc = _load().oracle_attention_rows(C.byref(c._c), _ptr(q), _ptr(sel), _ptr(sel_count), int(sel.shape[2]),
                                       C.c_double(sm_scale), _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError(f"oracle_attention_rows failed with {rc}")
    return out, lse


def round_bf16(x: np.ndarray) -> np.ndarray:
    """bf16 storage of the page means (the paper's storage format, Appendix A): each float64 rounded once to the
    nearest bfloat16, ties to even -> uint16 bit patterns of the same shape."""
    x = np.ascontiguousarray(x, np.float64)
    bits = np.zeros(x.shape, np.uint16)
    _load().oracle_round_bf16(_ptr(x), C.c_int64(x.size), _ptr(bits))
    return bits


def bf16_to_double(bits: np.ndarray) -> np.ndarray:
    """The float64 value of bf16 bit patterns (exact)."""
    bits = np.ascontiguousarray(bits, np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
