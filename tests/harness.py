"""Shared comparison logic of the GPU parity tests: GPU results (through the C ABI) vs the float64 oracle.

Tolerances (fixed here, stated in the tests' assertions):
  statistics  |d mean| <= 1e-5 * max(1, |mean|), |d std| <= 1e-5 * max(1, std)   (fp32 accumulation of <= 32 keys)
  scores      |d s|    <= 2e-5 * (1 + |s|)   (a D <= 128 fp32 dot product of O(1) terms errs by about 1e-6 absolute)
  selection   exact set, except inside the near-tie band: with s_(k), s_(k+1) the oracle's k-th and (k+1)-th
              scores and eps = 1e-4 * max(|s_(k)|, |s_(k+1)|), the GPU set T must satisfy
              {p: s_p > s_(k) + eps} <= T <= {p: s_p >= s_(k) - eps}; |T| = min(k, P), distinct, ascending, -1 padded
  bf16 statistic storage (stats_dtype = bf16): the stored mean must be, BIT FOR BIT, the oracle's float64 mean m rounded
              once to bf16 (oracle.round_bf16, ties to even). The one exception: the kernel rounds an fp32 mean, which
              lies within e = (n + 2) * 2^-24 * mean_j |k_j,d| of m for a page of n keys, so a stored value that differs
              must be the rounding of some number in [m - e, m + e]: RNE(m - e) <= stored <= RNE(m + e). In practice
              that is the neighbour across a rounding boundary m almost sits on, or, where a page's keys cancel
              (|m| << e), one of the tiny values around zero. Such elements are counted and the worst fraction of e
              that was needed is reported.
              The std stays fp32. Scores and selection are then checked against Eq. 6 evaluated by the oracle on its
              own rounded means (with the accepted stored values substituted in those few elements)
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


BF16_TIES = {"elements": 0, "accepted_neighbours": 0, "worst_ratio": 0.0}   # running totals over a test session


def bf16_bits_of(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def check_bf16_means(bits_g: np.ndarray, mean_o: np.ndarray, abs_key_mean, where=""):
    """Stored bf16 means (bit patterns, any shape [..., D]) against the oracle's float64 means rounded once to bf16.
    Where the bits differ, the stored value must still be the rounding of SOME real number within the fp32
    accumulation bound e = (n + 2) * 2^-24 * mean_j |k_j,d| of the float64 mean m. Rounding to nearest is monotone, so
    that is: RNE(m - e) <= stored <= RNE(m + e). (Usually e is far below the bf16 spacing and this admits the one
    neighbour across a rounding boundary that m almost sits on; where the keys of a page cancel, |m| << e, it admits
    the few tiny values around zero that an fp32 sum of the same keys can land on.)
    abs_key_mean(idx) -> mean_j |k_j,d| and the key count n of the page for each mismatching element (idx = tuple of
    index arrays into bits_g). Returns the float64 means the later stages are checked with, and (count of accepted
    differences, worst fraction of the bound that was needed)."""
    bits_o = oracle.round_bf16(mean_o)
    diff = np.nonzero(bits_g != bits_o)
    n_diff, worst = int(diff[0].size), 0.0
    if n_diff:
        g, m = bits_g[diff], mean_o[diff]
        vg = oracle.bf16_to_double(g)
        assert np.isfinite(vg).all(), f"{where}: non-finite stored bf16 mean"
        a, n = abs_key_mean(diff)
        bound = (n + 2.0) * 2.0 ** -24 * a

        def reachable(t):   # is the stored value the rounding of a number within t * bound of m ?
            lo = oracle.bf16_to_double(oracle.round_bf16(m - t * bound))
            hi = oracle.bf16_to_double(oracle.round_bf16(m + t * bound))
            return (lo <= vg) & (vg <= hi)
        ok = reachable(1.0)
        if not ok.all():
            i = int(np.nonzero(~ok)[0][0])
            raise AssertionError(
                f"{where}: {int((~ok).sum())} stored bf16 means are not the rounding of any number within the fp32 "
                f"accumulation bound of the float64 mean; first at {[int(d[i]) for d in diff]}: stored {vg[i]!r}, "
                f"float64 mean {m[i]!r}, its rounding {oracle.bf16_to_double(bits_o[diff][i:i + 1])[0]!r}, bound {bound[i]!r}")
        t_lo, t_hi = np.zeros_like(m), np.ones_like(m)     # smallest fraction of the bound that reaches the stored value
        for _ in range(30):
            mid = 0.5 * (t_lo + t_hi)
            r = reachable(mid)
            t_hi = np.where(r, mid, t_hi)
            t_lo = np.where(r, t_lo, mid)
        worst = float(t_hi.max())
    BF16_TIES["elements"] += int(bits_g.size)
    BF16_TIES["accepted_neighbours"] += n_diff
    BF16_TIES["worst_ratio"] = max(BF16_TIES["worst_ratio"], worst)
    used = bits_o.copy()
    used[diff] = bits_g[diff]
    return oracle.bf16_to_double(used), (n_diff, worst)


def _keys_f64(oc: OracleCache, phys, hkv, slot, d):
    k = oc.k_cache[phys, hkv, slot, d]
    return oracle.bf16_to_double(k) if oc.is_bf16 else k.astype(np.float64)


def check_stats_row(sess: DecodeSession, oc: OracleCache, b: int, hkv: int, pages=None):
    P = oc.num_pages(b)
    mean_o, std_o = oracle.page_stats(oc, b, hkv)
    phys = oc.page_table[b, :P].astype(np.int64)
    phys_t = torch.as_tensor(phys, device=sess.page_mean.device)
    std_g = sess.page_std[phys_t, hkv].double().cpu().numpy()
    sl = slice(None) if pages is None else pages
    ds = np.abs(std_g[sl] - std_o[sl]) / np.maximum(1.0, std_o[sl])
    assert np.isfinite(std_g[sl]).all(), f"non-finite stats in row ({b},{hkv})"
    assert ds.max(initial=0.0) <= 1e-5, f"std mismatch row ({b},{hkv}): {ds.max()}"
    if sess.stats_dtype == torch.bfloat16:
        sel_pages = np.arange(P)[sl]
        bits_g = bf16_bits_of(sess.page_mean[phys_t, hkv])[sl]

        def abs_key_mean(idx):
            pg = sel_pages[idx[0]]
            n = np.minimum(oc.S, int(oc.seq_lens[b]) - pg * oc.S)
            a = np.array([np.abs(_keys_f64(oc, phys[p_], hkv, slice(0, n_), d_)).mean()
                          for p_, n_, d_ in zip(pg, n, idx[1])])
            return a, n.astype(np.float64)
        mean_used, _ = check_bf16_means(bits_g, mean_o[sl], abs_key_mean, f"row ({b},{hkv})")
        full = oracle.bf16_to_double(oracle.round_bf16(mean_o))
        full[sl] = mean_used
        return full, std_o
    mean_g = sess.page_mean[phys_t, hkv].double().cpu().numpy()
    assert np.isfinite(mean_g[sl]).all(), f"non-finite stats in row ({b},{hkv})"
    dm = np.abs(mean_g[sl] - mean_o[sl]) / np.maximum(1.0, np.abs(mean_o[sl]))
    assert dm.max(initial=0.0) <= 1e-5, f"mean mismatch row ({b},{hkv}): {dm.max()}"
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


def full_check_batch(wl: Workload, sess: DecodeSession | None = None, stats_dtype=torch.float32, run_stats=True,
                     dense_heads=(), lam=None, host_cache: dict | None = None):
    """EVERY (sequence, KV head) row of a workload, at any size, against the oracle's whole-batch drivers
    (OpenMP over rows): statistics, Eq. 6 scores, the selected sets (near-tie rule), Eq. 5 outputs and lse on the
    GPU's own sets; Eq. 4 on the given (b, h) heads. The comparisons are the same as in full_check, vectorised.
    host_cache: a dict that keeps the host copy of the caches and the oracle's statistics between calls on an
    UNCHANGED workload (they depend on the workload only)."""
    sess = sess or DecodeSession(wl, stats_dtype=stats_dtype)
    lam = wl.lam if lam is None else lam
    if run_stats:
        sess.update_page_stats()
    sess.score_select_topk(lam)
    sess.sparse_paged_decode()
    if dense_heads:
        sess.dense_paged_decode()
    torch.cuda.synchronize()
    B, Hkv, G, D, S = wl.B, wl.Hkv, wl.G, wl.D, wl.S
    if host_cache is not None and "oc" in host_cache:
        oc, q, mean_o, std_o = (host_cache[k] for k in ("oc", "q", "mean_o", "std_o"))
    else:
        oc, q = oracle_cache(wl)
        mean_o, std_o = oracle.new_stat_cache(oc)
        oracle.update_stats(oc, mean_o, std_o)
        if host_cache is not None:
            host_cache.update(oc=oc, q=q, mean_o=mean_o, std_o=std_o)
    bf16 = sess.stats_dtype == torch.bfloat16
    mean_used = np.zeros_like(mean_o) if bf16 else mean_o     # what the oracle scores from
    n_ties, worst_tie = 0, 0.0
    for b in range(B):                                   # statistics, one sequence at a time (bounded host memory)
        P = oc.num_pages(b)
        if P == 0:
            continue
        phys = oc.page_table[b, :P].astype(np.int64)
        phys_t = torch.as_tensor(phys, device=sess.page_mean.device)
        std_g = sess.page_std[phys_t].double().cpu().numpy().T            # [Hkv, P]
        so = std_o[b, :, :P]
        assert np.isfinite(std_g).all(), f"non-finite std in sequence {b}"
        ds = np.abs(std_g - so) / np.maximum(1.0, so)
        assert ds.max() <= 1e-5, f"std mismatch in sequence {b}: {ds.max()}"
        mo = mean_o[b, :, :P]                                              # [Hkv, P, D]
        if bf16:
            bits_g = np.ascontiguousarray(bf16_bits_of(sess.page_mean[phys_t]).transpose(1, 0, 2))

            def abs_key_mean(idx, b=b, phys=phys):
                n = np.minimum(S, int(oc.seq_lens[b]) - idx[1] * S)
                a = np.array([np.abs(_keys_f64(oc, phys[p_], h_, slice(0, n_), d_)).mean()
                              for h_, p_, d_, n_ in zip(idx[0], idx[1], idx[2], n)])
                return a, n.astype(np.float64)
            used, (nt, wt) = check_bf16_means(bits_g, mo, abs_key_mean, f"sequence {b}")
            mean_used[b, :, :P] = used                                     # the oracle scores from its rounded means
            n_ties += nt
            worst_tie = max(worst_tie, wt)
        else:
            mean_g = sess.page_mean[phys_t].double().cpu().numpy().transpose(1, 0, 2)
            assert np.isfinite(mean_g).all(), f"non-finite mean in sequence {b}"
            dm = np.abs(mean_g - mo) / np.maximum(1.0, np.abs(mo))
            assert dm.max() <= 1e-5, f"mean mismatch in sequence {b}: {dm.max()}"
    ref = oracle.sparse_decode_step(oc, q, mean_used, std_o, lam, sess.top_k)
    del mean_used
    sel = sess.sel_pages.cpu().numpy()
    cnt = sess.sel_count.cpu().numpy()
    sc_g = sess.scores.double().cpu().numpy()
    n_exact, worst_score = 0, 0.0
    force = getattr(sess, "force_recent_pages", 0)
    for b in range(B):
        P = oc.num_pages(b)
        for hkv in range(Hkv):
            s_o = ref["scores"][b, hkv, :P]
            s_g = sc_g[b, hkv, :P]
            assert np.isfinite(s_g).all(), f"non-finite score in row ({b},{hkv})"
            err = float((np.abs(s_g - s_o) / (1.0 + np.abs(s_o))).max(initial=0.0))
            assert err <= 2e-5, f"score mismatch row ({b},{hkv}): {err}"
            worst_score = max(worst_score, err)
            n_exact += bool(check_selection_row(sel[b, hkv], int(cnt[b, hkv]), s_o, sess.top_k, f"row ({b},{hkv})", force))
    # Eq. 5 on the GPU's own sets, every head
    out_o, lse_o = oracle.attention_rows(oc, q, sel, cnt)
    out_g, lse_g = to_f64(sess.out), to_f64(sess.lse)
    assert np.isfinite(out_g).all()
    worst = float(np.abs(out_g - out_o).max())
    where = np.unravel_index(int(np.abs(out_g - out_o).argmax()), out_g.shape)
    assert worst <= OUT_TOL[wl.dtype], f"sparse attention max-abs error {worst} at (b, h, d) = {where}"
    live = np.isfinite(lse_o)
    assert np.array_equal(np.isneginf(lse_g), ~live)
    lerr = np.abs(lse_g[live] - lse_o[live]) / np.maximum(1.0, np.abs(lse_o[live]))
    assert lerr.max(initial=0.0) <= LSE_TOL[wl.dtype], f"lse error {lerr.max()}"
    for (b, h) in dense_heads:
        worst = max(worst, check_attention_head(sess.out_dense, sess.lse_dense, oc, q, b, h,
                                                np.arange(oc.num_pages(b), dtype=np.int32), wl.dtype,
                                                where=f"dense ({b},{h})"))
    rep = dict(rows=B * Hkv, exact_sets=n_exact, worst_abs_err=worst, worst_score_err=worst_score,
               dense_heads=len(dense_heads))
    if bf16:
        rep.update(bf16_elements=int(sum(oc.num_pages(b) for b in range(B)) * Hkv * D),
                   bf16_accepted_neighbours=n_ties, bf16_worst_tie_ratio=worst_tie)
    return sess, rep
