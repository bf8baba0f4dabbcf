"""Buffer owner for one decode workload: allocates the caller-side device tensors (statistics cache,
selection, outputs, workspace) with torch and forwards to the C ABI through ``binding``. No arithmetic
of the method happens here."""
from __future__ import annotations

import torch

from . import binding
from .workloads import Workload


class DecodeSession:
    def __init__(self, wl: Workload, top_k: int | None = None, max_seq_len_hint: int | None = None,
                 want_scores: bool = True, lib: binding.Library | None = None, stats_dtype=torch.float32,
                 force_recent_pages: int = 0, min_seq_len_hint: int | None = None):
        assert wl.k_cache.is_cuda, "the workload must live on the GPU"
        self.lib = lib or binding.load()
        self.wl = wl
        self.top_k = int(top_k if top_k is not None else wl.top_k)
        dev = wl.k_cache.device
        P = wl.num_phys_pages
        self.stats_dtype = stats_dtype
        rec = binding.stats_record_bytes(wl.Hkv, wl.D, stats_dtype)
        mean_bytes = rec - binding.STD_BLOCK_BYTES
        # one record per physical page, every byte 0xFF (NaN in fp32 and in bf16) until a kernel writes it
        self.page_stats = torch.full((P, rec), 0xFF, device=dev, dtype=torch.uint8)
        # views into the records: means [P, Hkv, D] (fp32 or bf16) and stds [P, Hkv] (fp32)
        self.page_mean = self.page_stats[:, :mean_bytes].view(stats_dtype).view(P, wl.Hkv, wl.D)
        self.page_std = self.page_stats[:, mean_bytes:mean_bytes + 4 * wl.Hkv].view(torch.float32)
        self.page_pad = self.page_stats[:, mean_bytes + 4 * wl.Hkv:]
        if max_seq_len_hint is None:
            max_seq_len_hint = int(wl.seq_lens.max().item()) + int(wl.meta.get("spare_tokens", 0))
        if min_seq_len_hint is None:  # sequences only grow while a session lives, so today's shortest is a lower bound
            min_seq_len_hint = min(int(wl.seq_lens.min().item()), max_seq_len_hint)
        self.desc = binding.make_desc(q_heads=wl.H, k_cache=wl.k_cache, v_cache=wl.v_cache,
                                      page_stats=self.page_stats, stats_dtype=stats_dtype,
                                      page_table=wl.page_table, seq_lens=wl.seq_lens,
                                      max_seq_len_hint=max_seq_len_hint, min_seq_len_hint=min_seq_len_hint,
                                      force_recent_pages=force_recent_pages)
        self.force_recent_pages = int(force_recent_pages)
        self.sel_pages = torch.full((wl.B, wl.Hkv, self.top_k), -7, device=dev, dtype=torch.int32)
        self.sel_count = torch.full((wl.B, wl.Hkv), -7, device=dev, dtype=torch.int32)
        self.scores = (torch.full((wl.B, wl.Hkv, wl.max_pages), float("nan"), device=dev, dtype=torch.float32)
                       if want_scores else None)
        self.out = torch.zeros((wl.B, wl.H, wl.D), device=dev, dtype=wl.dtype)
        self.lse = torch.zeros((wl.B, wl.H), device=dev, dtype=torch.float32)
        self.out_dense = torch.zeros_like(self.out)
        self.lse_dense = torch.zeros_like(self.lse)
        assert self.lib.page_stats_record_bytes(self.desc) == self.page_stats.shape[1]
        self.workspace_bytes = self.lib.workspace_bytes(self.desc, self.top_k)
        self.workspace = torch.empty((max(self.workspace_bytes, 256),), device=dev, dtype=torch.uint8)
        assert self.workspace.data_ptr() % 256 == 0

    # one method per entry point, same names
    def update_page_stats(self, tok_begin=None, tok_end=None, max_pages_touched_per_seq: int = 0):
        self.lib.update_page_stats(self.desc, tok_begin, tok_end, max_pages_touched_per_seq)

    def score_select_topk(self, lam: float | None = None):
        self.lib.score_select_topk(self.desc, self.wl.q, self.top_k, self.wl.lam if lam is None else lam,
                                   self.sel_pages, self.sel_count, self.scores, self.workspace)

    def page_scores(self, scores, lam: float | None = None):
        self.lib.page_scores(self.desc, self.wl.q, self.wl.lam if lam is None else lam, scores)

    def select_topk(self, scores):
        self.lib.select_topk(self.desc, scores, self.top_k, self.sel_pages, self.sel_count)

    def sparse_paged_decode(self, sm_scale: float = 0.0, sel_pages=None, sel_count=None):
        sel_pages = self.sel_pages if sel_pages is None else sel_pages
        sel_count = self.sel_count if sel_count is None else sel_count
        self.lib.sparse_paged_decode(self.desc, self.wl.q, sel_pages, sel_count, int(sel_pages.shape[-1]), sm_scale,
                                     self.out, self.lse, self.workspace)

    def decode_step(self, refresh_tail: bool = True, sm_scale: float = 0.0, lam: float | None = None):
        self.lib.decode_step(self.desc, self.wl.q, self.top_k, self.wl.lam if lam is None else lam, sm_scale,
                             refresh_tail, self.sel_pages, self.sel_count, self.out, self.lse, self.workspace)

    def decode_step_static(self, refresh_tail: bool = True, sm_scale: float = 0.0, lam: float | None = None):
        self.lib.decode_step_static(self.desc, self.wl.q, self.top_k, self.wl.lam if lam is None else lam, sm_scale,
                                    refresh_tail, self.sel_pages, self.sel_count, self.out, self.lse)

    def dense_paged_decode(self, sm_scale: float = 0.0):
        self.lib.dense_paged_decode(self.desc, self.wl.q, sm_scale, self.out_dense, self.lse_dense, self.workspace)

    def sparse_step(self):
        """score + select + sparse decode (statistics assumed current)."""
        self.score_select_topk()
        self.sparse_paged_decode()
