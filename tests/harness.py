"""Shared comparison logic of the GPU parity tests: GPU results (through the C ABI) vs the float64 oracle.

Tolerances (fixed here, stated in the tests' assertions):
  statistics  |d mean| <= 1e-5 * max(1, |mean|), |d std| <= 1e-5 * max(1, std)   (fp32 accumulation of <= 32 keys)
  scores      |d s|    <= 1e-5 * max(1, |s|, |q_g| * |mean|...) -> implemented as 2e-5 * (1 + |s|) + 1e-5 * scale
  selection   exact set, except inside the near-tie band: with s_(k), s_(k+1) the oracle's k-th and (k+1)-th
              scores and eps = 1e-4 * max(|s_(k)|, |s_(k+1)|), the GPU set T must satisfy
              {p: s_p > s_(k) + eps} <= T <= {p: s_p >= s_(k) - eps}; |T| = min(k, P), distinct, ascending, -1 padded
  bf16 statistic storage (stats_dtype = bf16): the stored mean must be the bf16 nearest to the oracle's mean
              (|d| <= half a bf16 ulp + 1e-5 * max(1, |mean|) for the fp32 accumulation), the std stays fp32; scores and
              selection are then checked against the oracle's Eq. 6 evaluated on the STORED statistics
  attention   max-abs error 1e-4 (fp32 caches) / 2e-2 (bf16 caches, output rounded to bf16), evaluated by the oracle
              on the GPU's selected set; lse within 1e-4 * max(1, |lse|) (fp32) / 1e-3 (bf16 inputs, fp32 lse)
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from oracle import OracleCache
from paper_2605_27740_amd.session import DecodeSession
from paper_2605_27740_amd.workloads import Workload

OUT_TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}
LSE_TOL = {torch.float32: 1e-4, torch.bfloat16: 1e-3}


def oracle_cache(wl: Workload):
    a = wl.host_arrays()
    return OracleCache(a["k_cache"], a["v_cache"], a["page_table"], a["seq_lens"], wl.H), a["q"]


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def check_stats_row(sess: DecodeSession, oc: OracleCache, b: int, hkv: int, pages=None):
    P = oc.num_pages(b)
    mean_o, std_o = oracle.page_stats(oc, b, hkv)
    phys = oc.page_table[b, :P].astype(np.int64)
    mean_g = sess.page_mean[torch.as_tensor(phys, device=sess.page_mean.device), hkv].double().cpu().numpy()
    std_g = sess.page_std[torch.as_tensor(phys, device=sess.page_std.device), hkv].double().cpu().numpy()
    sl = slice(None) if pages is None else pages
    ds = np.abs(std_g[sl] - std_o[sl]) / np.maximum(1.0, std_o[sl])
    assert np.isfinite(mean_g[sl]).all() and np.isfinite(std_g[sl]).all(), f"non-finite stats in row ({b},{hkv})"
    if sess.stats_dtype == torch.bfloat16:
        a = np.abs(mean_o[sl])
        ulp = np.exp2(np.floor(np.log2(np.maximum(a, 2.0 ** -126))) - 7)   # bf16: 8 significant bits
        excess = np.abs(mean_g[sl] - mean_o[sl]) - (0.5 * ulp + 1e-5 * np.maximum(1.0, a))
        assert excess.max(initial=-1.0) <= 0.0, f"bf16 mean is not the nearest bf16 in row ({b},{hkv}): {excess.max()}"
    else:
        dm = np.abs(mean_g[sl] - mean_o[sl]) / np.maximum(1.0, np.abs(mean_o[sl]))
        assert dm.max(initial=0.0) <= 1e-5, f"mean mismatch row ({b},{hkv}): {dm.max()}"
    assert ds.max(initial=0.0) <= 1e-5, f"std mismatch row ({b},{hkv}): {ds.max()}"
    if sess.stats_dtype == torch.bfloat16:
        return mean_g, std_g   # later stages are exact with respect to what is stored
    return mean_o, std_o


def check_scores_row(sess: DecodeSession, oc: OracleCache, q: np.ndarray, b: int, hkv: int, lam: float,
                     mean_o, std_o):
    P = oc.num_pages(b)
    s_o = oracle.page_scores(oc, q, b, hkv, lam, mean_o, std_o)
    s_g = sess.scores[b, hkv, :P].double().cpu().numpy()
    assert np.isfinite(s_g).all()
    # the score is a sum of D products of magnitude |q_d * mean_d|; bound the fp32 error by their scale
    scale = 1.0 + np.abs(s_o)
    err = np.abs(s_g - s_o) / scale
    assert err.max() <= 2e-5, f"score mismatch row ({b},{hkv}): {err.max()}"
    return s_o


def check_selection_row(sel_row: np.ndarray, count: int, s_o: np.ndarray, top_k: int, where="", force_recent=0):
    """Near-tie-aware comparison of one row's selected set with the oracle ranking. With force_recent = n the last
    min(n, k, P) pages must be selected and the rest of the set is compared with the ranking of the other pages."""
    P = s_o.shape[0]
    kb = min(top_k, P)
    assert count == kb, f"{where}: sel_count {count} != min(k, P) = {kb}"
    T = sel_row[:kb]
    assert (sel_row[kb:] == -1).all(), f"{where}: padding is not -1"
    assert (T >= 0).all() and (T < P).all(), f"{where}: page index out of range"
    assert (np.diff(T) > 0).all(), f"{where}: not strictly ascending (duplicates?)"
    if kb == P:
        assert T.tolist() == list(range(P))
        return True
    if force_recent > 0:
        n = min(force_recent, kb)
        assert T[kb - n:].tolist() == list(range(P - n, P)), f"{where}: the last {n} pages are not all selected"
        if kb == n:
            return True
        rest = np.concatenate([T[:kb - n], np.full((top_k - (kb - n),), -1, T.dtype)])
        return check_selection_row(rest, kb - n, s_o[:P - n], top_k - n, where, 0)   # here kb = top_k < P
    order, _ = oracle.topk(s_o, top_k)
    s_k, s_k1 = s_o[order[kb - 1]], s_o[order[kb]]
    eps = 1e-4 * max(abs(s_k), abs(s_k1))
    Tset = set(T.tolist())
    must = set(np.nonzero(s_o > s_k + eps)[0].tolist())
    allowed = set(np.nonzero(s_o >= s_k - eps)[0].tolist())
    assert must <= Tset, f"{where}: clearly better pages missing: {sorted(must - Tset)[:8]}"
    assert Tset <= allowed, f"{where}: pages below the tie band selected: {sorted(Tset - allowed)[:8]}"
    exact = Tset == set(order[:kb].tolist())
    if s_k - s_k1 > eps:
        assert exact, f"{where}: set differs from the oracle although the boundary gap exceeds the band"
    return exact


def check_attention_head(out_g: torch.Tensor, lse_g: torch.Tensor, oc: OracleCache, q: np.ndarray, b: int, h: int,
                         pages, dtype, sm_scale=0.0, where=""):
    o_o, lse_o = oracle.attention(oc, q, b, h, pages, sm_scale)
    o_g = to_f64(out_g[b, h])
    assert np.isfinite(o_g).all(), f"{where}: non-finite output"
    err = np.abs(o_g - o_o).max()
    assert err <= OUT_TOL[dtype], f"{where}: attention max-abs error {err} > {OUT_TOL[dtype]}"
    if lse_g is not None:
        lerr = abs(float(lse_g[b, h]) - lse_o)
        assert lerr <= LSE_TOL[dtype] * max(1.0, abs(lse_o)), f"{where}: lse error {lerr}"
    return err


def full_check(wl: Workload, sess: DecodeSession | None = None, rows=None, dense_heads=None, lam=None,
               run_stats=True, stats_dtype=torch.float32):
    """Run stats -> score+select -> sparse decode (+ dense) on the GPU and check the given (b, hkv) rows
    (all rows when None) stage by stage. Returns the session and a small report."""
    sess = sess or DecodeSession(wl, stats_dtype=stats_dtype)
    lam = wl.lam if lam is None else lam
    if run_stats:
        sess.update_page_stats()
    sess.score_select_topk(lam)
    sess.sparse_paged_decode()
    sess.dense_paged_decode()
    torch.cuda.synchronize()
    oc, q = oracle_cache(wl)
    sel = sess.sel_pages.cpu().numpy()
    cnt = sess.sel_count.cpu().numpy()
    rows = rows if rows is not None else [(b, h) for b in range(wl.B) for h in range(wl.Hkv)]
    n_exact, worst = 0, 0.0
    for (b, hkv) in rows:
        mean_o, std_o = check_stats_row(sess, oc, b, hkv)
        s_o = check_scores_row(sess, oc, q, b, hkv, lam, mean_o, std_o)
        n_exact += bool(check_selection_row(sel[b, hkv], int(cnt[b, hkv]), s_o, sess.top_k, f"row ({b},{hkv})",
                                            getattr(sess, "force_recent_pages", 0)))
        T = sel[b, hkv, :cnt[b, hkv]]
        for g in range(wl.G):
            h = hkv * wl.G + g
            worst = max(worst, check_attention_head(sess.out, sess.lse, oc, q, b, h, T, wl.dtype,
                                                    where=f"sparse ({b},{h})"))
    dense_heads = dense_heads if dense_heads is not None else [(b, hkv * wl.G + g) for (b, hkv) in rows
                                                               for g in range(wl.G)]
    for (b, h) in dense_heads:
        worst = max(worst, check_attention_head(sess.out_dense, sess.lse_dense, oc, q, b, h,
                                                np.arange(oc.num_pages(b), dtype=np.int32), wl.dtype,
                                                where=f"dense ({b},{h})"))
    return sess, dict(rows=len(rows), exact_sets=n_exact, worst_abs_err=worst)
