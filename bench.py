#!/usr/bin/env python3
"""Benchmark of the UNIQUE sparse decode step on one MI355X.

One "step" = one pass of the hot path over one batch of synthetic input that is already resident in HBM:
  unique_update_page_stats on the last token of every sequence (tail-page refresh)
  -> unique_score_select_topk (Eq. 6 scores + top-k)  -> unique_sparse_paged_decode (Eq. 5).
unique_dense_paged_decode (Eq. 4) is timed beside it as the in-library comparison point, and the float64
CPU oracle is timed on a bounded sample of the same workload as a reported baseline.

Prints ONE JSON line (see the keys at the bottom). Usage: python bench.py [--gpus 1] [--steps K] [--warmup W]
[--workload c2|c3|c4|c5] [--stats-dtype fp32|bf16] [--top-k K] [--no-cpu-baseline] [--no-dense] [--copy-calibration BYTES]
Analysis modes, each printing one JSON line of its own: --paper-shapes (the shapes of the paper's Appendix A / B tables
and Fig. 2), and, on the profiling build of the library, --phase-stamps (where the sparse decode kernel's time goes),
--gather-probe (the bare K/V gather behind it) and --record-probe (the bare stream of page records behind the score
kernel).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--top-k", type=int, default=None)
    ap.add_argument("--batch", type=int, default=None,
                    help="with --workload c3: another batch size (the workload name in the JSON line says so)")
    ap.add_argument("--context", type=int, default=None, help="with --workload c3: another context length")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--stats-dtype", default="fp32", choices=["fp32", "bf16"],
                    help="storage of the page means: fp32 (selection equals an exact fp32 ranking) or bf16 (the paper's format)")
    ap.add_argument("--separate-calls", action="store_true",
                    help="time the step as update_page_stats + score_select_topk + sparse_paged_decode instead of unique_decode_step")
    ap.add_argument("--paper-shapes", action="store_true",
                    help="microbenchmarks at the shapes of the paper's Appendix A / B tables instead of a decode step")
    ap.add_argument("--phase-stamps", action="store_true",
                    help="profiling build: per-wave wall-clock stamps inside the sparse decode kernel of a cold decode step")
    ap.add_argument("--record-probe", action="store_true",
                    help="profiling build: the bare stream of page records behind the score kernel (its ceiling) at the 128K batch's shape")
    ap.add_argument("--gather-probe", action="store_true",
                    help="profiling build: the bare K/V gather of the sparse decode (no page table, no arithmetic) at the "
                         "128K batch's shape, for several chunk placements, load patterns and prefetch depths")
    ap.add_argument("--copy-calibration", type=int, default=0,
                    help="only run a device-to-device copy of this many bytes (counter calibration for rocprofv3 --pmc)")
    return ap.parse_args()


def algorithmic_bytes(wl, sess, sel_count, seq_lens):
    """Bytes the method itself must move per launch, per kernel (the numerators of achieved GB/s)."""
    es = 2 if "bfloat16" in str(sess.stats_dtype) else 4  # bytes per stored mean element
    e = 2 if str(wl.dtype).endswith("bfloat16") else 4
    S, D, G, Hkv, H, B = wl.S, wl.D, wl.G, wl.Hkv, wl.H, wl.B
    pages = [(int(n) + S - 1) // S for n in seq_lens]
    tot_pages = sum(pages)
    out = {}
    # tail-page stats: the valid keys of the last page of each (b, hkv) read, D+1 floats written
    tail = [int(n) - (p - 1) * S for n, p in zip(seq_lens, pages)]
    out["page_stats_kernel"] = sum(t * D * e * Hkv for t in tail) + B * Hkv * (D * es + 4)
    # score: mean + std read per (b, hkv, page), one page-table entry per (b, page), one float written
    out["page_score_kernel"] = tot_pages * Hkv * (D * es + 4) + tot_pages * 4 + tot_pages * Hkv * 4 + B * H * D * e
    # select: the score row read once, k_b + 1 ints written
    out["topk_select_kernel"] = tot_pages * Hkv * 4 + int(sel_count.sum()) * 4 + B * Hkv * 4
    # sparse decode: K and V of the selected pages (full pages; at most one per row is partial), list + table
    # entries, q, and the split-K partials written once
    k_total = int(sel_count.sum())
    kv = k_total * S * D * 2 * e
    out["paged_decode_partial_kernel"] = kv + k_total * 8 + B * H * D * e
    out["paged_decode_partial_kernel_dense"] = tot_pages * Hkv * S * D * 2 * e + tot_pages * Hkv * 4 + B * H * D * e
    return out


def pct(xs):
    """median / p10 / p90 / mean of a list of durations."""
    import statistics as st
    xs = sorted(xs)
    n = len(xs)
    return {"median": xs[n // 2], "p10": xs[n // 10], "p90": xs[min(n - 1, (9 * n) // 10)], "mean": st.fmean(xs)}


class Flusher:
    """Cold mode: between two timed steps (outside the events) one 1 GiB buffer is rewritten and a second one is
    then read, each four times the 256 MB Infinity Cache and far beyond the 8 x 4 MB L2s, and the step gets another
    of several query sets, so neither the statistics, nor the selected K/V pages of an earlier step, nor the page
    table are cached. The read comes last on purpose: it leaves the caches full of CLEAN lines. (A write alone
    leaves them full of dirty lines, whose write-back then competes with the next kernel's reads: the score kernel
    measured 115 us after a write-only flush, 93 us after this one, 90 us warm.)"""

    def __init__(self, torch, wl, dev, n_queries=4, nbytes=1 << 30):
        self.buf = torch.zeros((nbytes,), dtype=torch.uint8, device=dev)
        self.rbuf = torch.zeros((nbytes // 4,), dtype=torch.int32, device=dev)
        g = torch.Generator(device=dev)
        g.manual_seed(977)
        self.wl = wl
        self.q0 = wl.q
        self.qs = [wl.q] + [torch.randn(wl.q.shape, generator=g, device=dev, dtype=torch.float32).to(wl.dtype)
                            for _ in range(n_queries - 1)]

    def before_step(self, i):
        self.wl.q = self.qs[i % len(self.qs)]
        self.buf.add_(1)
        self.rbuf.sum()

    def restore(self):
        self.wl.q = self.q0


def kernel_trace(torch, fn, n):
    """Durations of the individual kernels inside the library calls (the split-K partial kernel apart from the
    merge), from the device timestamps torch's profiler collects; None if the profiler is not usable here (for
    instance when the whole program already runs under rocprofv3)."""
    if any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ) or "rocprof" in os.environ.get("LD_PRELOAD", ""):
        return None
    try:
        from torch.profiler import ProfilerActivity, profile
        with profile(activities=[ProfilerActivity.CUDA]) as prof:
            for i in range(n):
                fn(i)
            torch.cuda.synchronize()
        out = {}
        for ev in prof.events():
            name = ev.name
            if "unique::" not in name:
                continue
            short = name.split("unique::(anonymous namespace)::")[-1].split("(")[0].split("<")[0]
            dur = getattr(ev, "device_time", None)
            if dur is None:
                dur = getattr(ev, "cuda_time", 0.0)
            out.setdefault(short, []).append(float(dur))
        return {k: dict(pct(v), n=len(v)) for k, v in out.items()} or None
    except Exception as exc:  # the profiler is an extra; the event timings above do not depend on it
        return {"error": repr(exc)[:200]}


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py measures one GPU only (asked for --gpus {args.gpus}); the path has no cross-GPU part.",
              file=sys.stderr)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"

    if args.copy_calibration:
        n = args.copy_calibration
        src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": n, "launches": 5}))
        return

    from paper_2605_27740_amd import workloads as W
    from paper_2605_27740_amd.session import DecodeSession

    if args.paper_shapes:
        paper_shapes(dev)
        return
    if args.phase_stamps or args.gather_probe or args.record_probe:
        (phase_stamps if args.phase_stamps else gather_probe if args.gather_probe else record_probe)(args, dev)
        return
    stats_dtype = torch.bfloat16 if args.stats_dtype == "bf16" else torch.float32

    t0 = time.time()
    kw = {} if args.top_k is None else {"top_k": args.top_k}
    if args.batch is not None or args.context is not None:
        assert args.workload == "c3", "--batch / --context vary the c3 recipe only"
        if args.batch is not None:
            kw["batch"] = args.batch
        if args.context is not None:
            kw["context"] = args.context
    wl = {"c2": W.config2, "c3": W.config3, "c4": W.config4, "c5": W.config5}[args.workload](device=dev, **kw)
    if args.batch is not None or args.context is not None:
        wl.name = f"c3_recipe_b{wl.B}_ctx{max(wl.seq_lens.tolist())}"   # a variation, not the 128K benchmark configuration
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    sess = DecodeSession(wl, want_scores=False, stats_dtype=stats_dtype)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    # bulk statistics build (prefill-time work, reported but not part of the step)
    sess.update_page_stats()
    torch.cuda.synchronize()
    a, b_ = ev(), ev()
    a.record(); sess.update_page_stats(); b_.record(); torch.cuda.synchronize()
    bulk_stats_ms = a.elapsed_time(b_)

    tok_end = wl.seq_lens.clone()
    tok_begin = tok_end - 1

    def separate_step():
        sess.update_page_stats(tok_begin, tok_end, 1)
        sess.score_select_topk()
        sess.sparse_paged_decode()

    def fused_step():  # the same work through the one-call entry point (tail refresh inside the score kernel)
        sess.decode_step(refresh_tail=True)

    step = separate_step if args.separate_calls else fused_step
    K = args.steps

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # --- timed region: exactly K steps back to back, bracketed by synchronisations (`value`)
    start, stop = ev(), ev()
    start.record()
    for _ in range(K):
        step()
    stop.record()
    torch.cuda.synchronize()
    ms_per_step = start.elapsed_time(stop) / K

    # --- the same K steps, each between its own pair of events: warm (same buffers every step), then cold
    def per_step(before):
        pairs = [(ev(), ev()) for _ in range(K)]
        for i, (x, y) in enumerate(pairs):
            before(i)
            x.record(); step(); y.record()
        torch.cuda.synchronize()
        return pct([x.elapsed_time(y) * 1e3 for x, y in pairs])

    warm_step = per_step(lambda i: None)
    flusher = Flusher(torch, wl, dev)
    for i in range(4):
        flusher.before_step(i); step()
    cold_step = per_step(flusher.before_step)

    # --- stage breakdown, cold and warm: the same K steps with an event between stages (score and select are
    # launched through their own entry points here: the same two kernels as the fused call)
    stride = (wl.max_pages + 63) // 64 * 64
    score_buf = torch.empty((wl.B, wl.Hkv, stride), device=dev, dtype=torch.float32)

    def staged(before):
        marks = [[ev() for _ in range(5)] for _ in range(K)]
        for i in range(K):
            before(i)
            marks[i][0].record()
            sess.update_page_stats(tok_begin, tok_end, 1)
            marks[i][1].record()
            sess.page_scores(score_buf)
            marks[i][2].record()
            sess.select_topk(score_buf)
            marks[i][3].record()
            sess.sparse_paged_decode()
            marks[i][4].record()
        torch.cuda.synchronize()
        names = ["update_page_stats_tail", "page_scores", "select_topk", "sparse_paged_decode"]
        return {nm: pct([marks[i][j].elapsed_time(marks[i][j + 1]) * 1e3 for i in range(K)]) for j, nm in enumerate(names)}

    stages_cold = staged(flusher.before_step)
    # kernel-level durations inside the calls (partial kernel apart from the merge), cold
    def traced_step(i):
        flusher.before_step(i)
        step()
    kernels_cold = kernel_trace(torch, traced_step, min(K, 20))
    flusher.restore()
    stages = staged(lambda i: None)
    sess.score_select_topk()          # leave the selection of the original queries in place
    torch.cuda.synchronize()

    other = fused_step if args.separate_calls else separate_step
    other()
    torch.cuda.synchronize()
    start.record()
    for _ in range(K):
        other()
    stop.record()
    torch.cuda.synchronize()
    other_us = start.elapsed_time(stop) / K * 1e3

    # --- the one-call step captured once into a HIP graph and replayed (the calls only launch kernels)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fused_step()
    graph.replay()
    torch.cuda.synchronize()
    start.record()
    for _ in range(K):
        graph.replay()
    stop.record()
    torch.cuda.synchronize()
    graph_us = start.elapsed_time(stop) / K * 1e3

    # --- the same K steps with the other statistics format (bf16 means are the paper's storage format and half the
    # bytes of the score stage; fp32 means give a selection that equals an exact fp32 ranking). Reported, not `value`.
    other_dtype = torch.float32 if stats_dtype == torch.bfloat16 else torch.bfloat16
    alt = DecodeSession(wl, want_scores=False, stats_dtype=other_dtype)
    alt.update_page_stats()
    for _ in range(args.warmup):
        alt.decode_step(refresh_tail=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(K):
        alt.decode_step(refresh_tail=True)
    stop.record()
    torch.cuda.synchronize()
    alt_us = start.elapsed_time(stop) / K * 1e3
    alt_pairs = [(ev(), ev()) for _ in range(K)]
    for i, (x, y) in enumerate(alt_pairs):
        flusher.before_step(i)
        x.record(); alt.decode_step(refresh_tail=True); y.record()
    torch.cuda.synchronize()
    flusher.restore()
    alt_cold = pct([x.elapsed_time(y) * 1e3 for x, y in alt_pairs])
    del alt

    def timed(fn, n):
        x, y = ev(), ev()
        x.record()
        for _ in range(n):
            fn()
        y.record()
        torch.cuda.synchronize()
        return x.elapsed_time(y) * 1e3 / n

    dense_us = None
    if not args.no_dense:
        nd = max(3, min(K, 20))
        sess.dense_paged_decode()
        dense_us = timed(sess.dense_paged_decode, nd)

    seq_lens = wl.seq_lens.cpu().tolist()
    sel_count = sess.sel_count.cpu()
    ab = algorithmic_bytes(wl, sess, sel_count, seq_lens)

    # Per kernel: algorithmic bytes over the COLD event-timed duration of its call (median). The page-score, select
    # and stats calls are one kernel each; the decode call is the split-K partial kernel plus the small merge kernel,
    # so the call's duration bounds the partial kernel's from above; the partial kernel's own duration comes from the
    # device timestamps of the profiler pass when that is available.
    def entry(nbytes, us):
        return {"bytes": nbytes, "us": us, "GBps": nbytes / us / 1e3, "frac": nbytes / us / 1e3 / HBM_PEAK_GBPS}
    by_kernel = {
        "page_stats_kernel(tail)": entry(ab["page_stats_kernel"], stages_cold["update_page_stats_tail"]["median"]),
        "page_score_kernel": entry(ab["page_score_kernel"], stages_cold["page_scores"]["median"]),
        "topk_select_kernel": entry(ab["topk_select_kernel"], stages_cold["select_topk"]["median"]),
        "paged_decode_partial_kernel(+merge)": entry(ab["paged_decode_partial_kernel"],
                                                     stages_cold["sparse_paged_decode"]["median"]),
    }
    dom = max(by_kernel, key=lambda k: by_kernel[k]["us"])
    roofline = {"bound": "hbm", "kernel": dom, "mode": "cold", "achieved": by_kernel[dom]["GBps"], "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": by_kernel[dom]["frac"], "traffic": measured_traffic(wl.name, dom),
                "traffic_source": "committed rocprofv3 --pmc summary profiles/hbm_traffic_<workload>.txt (not this run)",
                "algorithmic_bytes_per_launch": by_kernel[dom]["bytes"], "avg_launch_us": by_kernel[dom]["us"],
                "by_kernel": by_kernel}
    if dense_us is not None:
        roofline["dense_decode"] = entry(ab["paged_decode_partial_kernel_dense"], dense_us)

    # The kernel the bandwidth target is stated on: sparse decode. `call` = event-timed unique_sparse_paged_decode
    # (partial + merge launches); `partial_kernel` = the split-K kernel alone (device timestamps).
    nb = ab["paged_decode_partial_kernel"]
    sdk = {"bytes": nb, "traffic": measured_traffic(wl.name, "paged_decode_partial_kernel"),
           "call_cold": entry(nb, stages_cold["sparse_paged_decode"]["median"]),
           "call_warm": entry(nb, stages["sparse_paged_decode"]["median"]),
           "partial_kernel_cold": None, "merge_kernel_cold_us": None}
    if isinstance(kernels_cold, dict) and "error" not in kernels_cold:
        part = [v for k, v in kernels_cold.items() if k.startswith("paged_decode_partial")]
        merge = [v for k, v in kernels_cold.items() if k.startswith("paged_decode_merge")]
        if part:
            sdk["partial_kernel_cold"] = entry(nb, part[0]["median"])
        if merge:
            sdk["merge_kernel_cold_us"] = merge[0]["median"]

    # config 4's decode loop: every step appends one token per sequence (the harness writes K/V into the cache, which
    # is the serving engine's job and costs a few small torch kernels), then the library step refreshes the page that
    # received the token. 64 steps, so every sequence crosses a page boundary twice at S = 32.
    append_loop_us = None
    if args.workload == "c4":
        n_app = 64
        g = torch.Generator(device=dev)
        g.manual_seed(4242)
        newk = torch.randn((n_app, wl.B, wl.Hkv, wl.D), generator=g, device=dev).to(wl.dtype)
        newv = torch.randn((n_app, wl.B, wl.Hkv, wl.D), generator=g, device=dev).to(wl.dtype)
        ar = torch.arange(wl.B, device=dev)
        pt64 = wl.page_table.to(torch.int64)
        def append_and_step(i):
            n = wl.seq_lens.to(torch.int64)
            phys = pt64[ar, n // wl.S]
            wl.k_cache[phys, :, n % wl.S, :] = newk[i]
            wl.v_cache[phys, :, n % wl.S, :] = newv[i]
            wl.seq_lens += 1
            sess.decode_step(refresh_tail=True)
        append_and_step(0)
        torch.cuda.synchronize()
        x, y = ev(), ev()
        x.record()
        for i in range(1, n_app):
            append_and_step(i)
        y.record()
        torch.cuda.synchronize()
        append_loop_us = x.elapsed_time(y) * 1e3 / (n_app - 1)

    cpu = None
    if not args.no_cpu_baseline:
        del flusher
        torch.cuda.empty_cache()
        cpu = cpu_baseline(wl, sess)

    step_bytes = ab["page_stats_kernel"] + ab["page_score_kernel"] + ab["topk_select_kernel"] + ab["paged_decode_partial_kernel"]
    us = ms_per_step * 1e3
    line = {
        "metric": "sparse decode attention us/step (tail-page stats + page score + top-k + sparse paged decode)",
        "value": us, "unit": "us/step", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "storage_dtype": str(wl.dtype).replace("torch.", ""), "stats_dtype": args.stats_dtype,
        "data": "synthetic", "step_call": "separate calls" if args.separate_calls else "unique_decode_step",
        "timing": "value: K steps back to back between two events (same buffers). warm / cold: every step between its "
                  "own events, us; cold = 1 GiB rewritten, another 1 GiB read and another of 4 query sets before each step, "
                  "outside the events. roofline and sparse_decode_kernel use the cold medians.",
        "warm": warm_step, "cold": cold_step,
        "other_step_call_us": other_us, "step_graph_replay_us": graph_us,
        "other_stats_format": {"stats_dtype": "fp32" if other_dtype == torch.float32 else "bf16", "us_per_step": alt_us,
                               "cold": alt_cold},
        "config": {"workload": wl.name, "batch": wl.B, "q_heads": wl.H, "kv_heads": wl.Hkv, "head_dim": wl.D,
                   "page_size": wl.S, "context": max(seq_lens), "total_tokens": sum(seq_lens), "top_k_pages": sess.top_k,
                   "lambda": wl.lam},
        "roofline": roofline, "sparse_decode_kernel": sdk, "cpu_baseline": cpu,
        "stages_us": stages, "stages_cold_us": stages_cold, "kernels_cold_us": kernels_cold,
        "step_algorithmic_bytes": step_bytes, "step_hbm_GBps": step_bytes / us / 1e3,
        "step_hbm_GBps_cold": step_bytes / cold_step["median"] / 1e3,
        "attention_tokens_per_s": wl.B / (us * 1e-6),
        "dense_paged_decode_us": dense_us,
        "speedup_vs_dense": None if dense_us is None else dense_us / us,
        "bulk_stats_build_ms": bulk_stats_ms, "workload_gen_s": gen_s,
        "step_with_cache_append_us": append_loop_us,
        "paper_context": "paper: 11.4x attention-path speedup over dense FlashInfer at 32K, >=5.3x end to end (1x H100, S=8, batch 80)",
    }
    print(json.dumps(line))


def _profiling_library():
    import ctypes as C
    from paper_2605_27740_amd import binding, build
    path = build.PROF_LIB_PATH if os.path.exists(build.PROF_LIB_PATH) else build.build_profiling_library()
    return binding.Library(path), C.CDLL("libamdhip64.so"), C


def _device_kernel_us(torch, fn, n, name):
    """median device duration (us) of the kernels whose name contains `name` over n calls of fn(i)"""
    from torch.profiler import ProfilerActivity, profile
    with profile(activities=[ProfilerActivity.CUDA]) as prof:
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
    xs = sorted(float(ev.device_time) for ev in prof.events() if name in ev.name)
    return xs[len(xs) // 2] if xs else float("nan")


def phase_stamps(args, dev):
    """Where the time of the sparse decode kernel goes: every wave of the profiling build stamps the 100 MHz wall
    clock at entry, once its page ids are resolved, after its first tile, at the end of its loop, after its stores
    and after every tile. Cold decode steps (Flusher), 10 launches after 2 untimed ones. Prints one JSON line."""
    import numpy as np
    import torch
    from paper_2605_27740_amd import workloads as W
    from paper_2605_27740_amd.session import DecodeSession
    lib, hip, C = _profiling_library()
    kw = {} if args.top_k is None else {"top_k": args.top_k}
    wl = {"c2": W.config2, "c3": W.config3, "c4": W.config4, "c5": W.config5}[args.workload](device=dev, **kw)
    sess = DecodeSession(wl, want_scores=False, lib=lib,
                         stats_dtype=torch.bfloat16 if args.stats_dtype == "bf16" else torch.float32)
    sess.update_page_stats()
    ptr, waves, slots = C.c_void_p(), C.c_int(), C.c_int()
    assert lib.c.unique_debug_dec_stamps(C.byref(ptr), C.byref(waves), C.byref(slots)) == 0
    nbytes = waves.value * slots.value * 8
    flusher = Flusher(torch, wl, dev)
    runs, tiles = [], []
    for it in range(12):
        torch.cuda.synchronize()
        assert hip.hipMemset(ptr, 0, C.c_size_t(nbytes)) == 0
        flusher.before_step(it)
        sess.decode_step(refresh_tail=True)
        torch.cuda.synchronize()
        host = np.zeros((waves.value, slots.value), np.uint64)
        assert hip.hipMemcpy(C.c_void_p(host.ctypes.data), ptr, C.c_size_t(nbytes), 2) == 0
        live = host[host[:, 0] > 0].astype(np.int64)
        if it < 2:
            continue
        t0 = live[:, 0].min()
        runs.append((live[:, :5] - t0) / 100.0)                       # us since the first wave entered
        tl = live[:, 6:]
        tiles.append(np.where(tl > 0, (tl - t0) / 100.0, np.nan))
        hw = live[:, 5]          # slot 5: HW_ID register in the high word (compute unit: bits 8-11, shader engine: 13-15), XCC id in the low
    r, tl = np.stack(runs), np.stack(tiles)
    xcc, se, cu = hw & 0xF, (hw >> 45) & 0x7, (hw >> 40) & 0xF
    done = r[:, :, 3].mean(axis=0)
    by = lambda key: {str(int(v)): round(float(done[key == v].mean()), 2) for v in np.unique(key)}
    idx = np.arange(done.shape[0])
    wave_in_wg, wg = idx % 4, idx // 4
    seq = wg // (4 * wl.Hkv)                                   # grid (splits, Hkv, B): the sequence is the slowest index
    tm = np.nanmean(tl, axis=0)                                  # [waves, tiles]: mean time at which each tile was consumed
    tiles_of = lambda b_: [round(float(x), 1) for x in np.nanmean(tm[seq == b_], axis=0) if np.isfinite(x)]
    first_tile = r[:, :, 2].mean(axis=0)
    same_list = float(np.corrcoef(r[0, :, 3], r[4, :, 3])[0, 1])      # launches 0 and 4 use the same query set
    other_list = float(np.corrcoef(r[0, :, 3], r[1, :, 3])[0, 1])
    q = lambda x: [round(float(v), 2) for v in np.percentile(x, [0, 10, 50, 90, 100])]
    names = ["entry", "page_ids_resolved", "first_tile_done", "loop_done", "partials_stored"]
    edges = np.arange(0, 2 * (int(np.nanmax(r[:, :, 4]) // 2) + 2), 2.0)
    hist = sum(np.histogram(t[np.isfinite(t)], bins=edges)[0] for t in tl) / tl.shape[0]
    tile_bytes = 2 * 16 * wl.D * wl.k_cache.element_size()             # one 16-token tile of K and of V
    print(json.dumps({
        "phase_stamps": {"workload": wl.name, "top_k_pages": sess.top_k, "waves": int(r.shape[1]), "launches": int(r.shape[0]),
                         "percentiles": "min, p10, median, p90, max over waves and launches, us since the first wave entered",
                         "stamps_us": {n: q(r[:, :, i]) for i, n in enumerate(names)},
                         "phase_lengths_us": {f"{names[i]}->{names[i + 1]}": q(r[:, :, i + 1] - r[:, :, i]) for i in range(4)},
                         "kernel_span_us_per_launch": [round(float(x), 2) for x in r[:, :, 4].max(axis=1)],
                         "loop_done_us_mean_by_xcc": by(xcc), "loop_done_us_mean_by_shader_engine": by(se),
                         "loop_done_us_mean_by_cu_in_engine": by(cu), "compute_units_seen": int(len(np.unique(xcc * 4096 + se * 16 + cu))),
                         "loop_done_us_mean_by_sequence": by(seq),
                         "tile_done_us_first_sequence": tiles_of(0), "tile_done_us_last_sequence": tiles_of(int(seq.max())),
                         "correlation_first_tile_done_vs_loop_done": round(float(np.corrcoef(first_tile, done)[0, 1]), 3),
                         "loop_done_correlation_between_launches": {"same_page_lists": round(same_list, 3),
                                                                    "different_page_lists": round(other_list, 3)},
                         "consumed_TBps_per_2us_bin": {str(int(e)): round(float(h) * tile_bytes / 2e-6 / 1e12, 2)
                                                       for e, h in zip(edges[:-1], hist)}}}))


def gather_probe(args, dev):
    """The bare memory access of the sparse decode at the 128K batch's shape (128 rows x 256 tiles of 4 KiB K + 4 KiB V
    out of two 4.3 GB pools), kernel durations from the device timestamps, eight different lists in turn (cold)."""
    import torch
    lib, hip, C = _profiling_library()
    rows, k, heads, pool = 128, 256, 8, 131072
    kpool = torch.empty((pool, heads, 2048), dtype=torch.bfloat16, device=dev).fill_(1.0)
    vpool = torch.empty((pool, heads, 2048), dtype=torch.bfloat16, device=dev).fill_(2.0)
    sink = torch.zeros((4096,), dtype=torch.int32, device=dev)
    g = torch.Generator(device="cpu"); g.manual_seed(7)
    lists = {"random_4KiB_chunks": [], "consecutive_pages": [], "random_32KiB_chunks(all heads of a sequence pick the same pages)": []}
    for l in range(8):
        rnd = torch.sort(torch.randint(0, pool, (rows, k), generator=g), dim=1).values
        lists["random_4KiB_chunks"].append(rnd.to(torch.int32).to(dev))
        start = (torch.arange(rows) // heads) * 8192 + (l * 997) % 7000
        lists["consecutive_pages"].append((start[:, None] + torch.arange(k)[None, :]).to(torch.int32).to(dev))
        lists["random_32KiB_chunks(all heads of a sequence pick the same pages)"].append(
            rnd[(torch.arange(rows) // heads) * heads].to(torch.int32).to(dev))
    out, nbytes = [], rows * k * 8192
    fn = lib.c.unique_debug_gather_probe
    fn.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p] + [C.c_int] * 7 + [C.c_void_p, C.c_void_p]
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    for place, ls in lists.items():
        for pattern in (0, 1, 2):
            for depth in (2, 4):
                for waves, ppw in ((4, 64), (4, 128), (8, 128), (4, 256)):
                    if pattern == 2 and waves * depth * 8192 > 160 * 1024:
                        continue
                    def call(i):
                        rc = fn(kpool.data_ptr(), vpool.data_ptr(), ls[i % 8].data_ptr(), rows, k, heads, ppw, waves, depth,
                                pattern, sink.data_ptr(), stream)
                        assert rc == 0, rc
                    call(0); torch.cuda.synchronize()
                    us = _device_kernel_us(torch, call, 16, "gather_probe")
                    out.append({"placement": place, "k_load_pattern": ["contiguous_1KiB", "mfma_operand_64B_x16", "contiguous_1KiB_into_LDS"][pattern],
                                "tiles_in_flight": depth, "waves_per_wg": waves, "pages_per_wg": ppw,
                                "workgroups": rows * ((k + ppw - 1) // ppw), "us": round(us, 2),
                                "TBps": round(nbytes / us / 1e6, 3)})
    print(json.dumps({"gather_probe": {"bytes": nbytes, "rows": rows, "pages_per_row": k, "results": out}}))


def record_probe(args, dev):
    """The bare memory access of the score kernel at the 128K batch's shape (16 sequences x 8192 pages, page table a
    random permutation of the pool, or the identity): every page record's mean block (4 KiB of a 4224-byte record =
    fp32 means, 2 KiB of 2176 = bf16 means) streamed once, kernel durations from the device timestamps, cold (1 GiB
    rewritten and 1 GiB read before every launch)."""
    import torch
    lib, hip, C = _profiling_library()
    B, P = 16, 8192
    pool = B * P
    fn = lib.c.unique_debug_record_probe
    fn.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p] + [C.c_int] * 5 + [C.c_void_p, C.c_void_p]
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    sink = torch.zeros((4096,), dtype=torch.int32, device=dev)
    g = torch.Generator(device="cpu"); g.manual_seed(7)
    tables = {"permuted": torch.randperm(pool, generator=g).to(torch.int32).view(B, P).to(dev),
              "identity": torch.arange(pool, dtype=torch.int32).view(B, P).to(dev)}
    flush_w = torch.zeros((1 << 30,), dtype=torch.uint8, device=dev)
    flush_r = torch.zeros((1 << 28,), dtype=torch.int32, device=dev)
    out = []
    for rec, loads in ((4224, 4), (2176, 2)):
        stats = torch.ones((pool, rec), dtype=torch.uint8, device=dev)
        for place, table in tables.items():
            for tile in (32, 64, 128, 256):
                for depth in (2, 4, 8):
                    def call(i):
                        flush_w.add_(1); flush_r.sum()
                        rc = fn(stats.data_ptr(), rec, loads, table.data_ptr(), P, P, B, tile, depth, sink.data_ptr(), stream)
                        assert rc == 0, rc
                    call(0); torch.cuda.synchronize()
                    us = _device_kernel_us(torch, call, 10, "record_probe")
                    nbytes = pool * loads * 1024
                    out.append({"record_bytes": rec, "bytes_read_per_record": loads * 1024, "page_table": place, "pages_per_wg": tile,
                                "workgroups": B * ((P + tile - 1) // tile), "records_in_flight_per_wave": depth,
                                "us": round(us, 2), "TBps": round(nbytes / us / 1e6, 3), "frac_of_8TBps": round(nbytes / us / 8e6, 3)})
        del stats
    print(json.dumps({"record_probe": {"batch": B, "pages_per_sequence": P, "results": out}}))


def paper_shapes(dev):
    """Score kernel and top-k at the shapes of the paper's Appendix A (fused criticality kernel) and Appendix B
    (radix top-k): batch 32, 32 q / 8 KV heads, D = 128, S = 8, lambda 0.5, k = 64, P = 1024 ... 16384; median of 100
    timed iterations after 20 warm-ups (score) / 300 after 50 (top-k), as the paper does. The paper's numbers are one
    H100 with bf16 scores; they are context, not a target."""
    import torch
    from paper_2605_27740_amd import workloads as W
    from paper_2605_27740_amd.session import DecodeSession
    paper_score_ms = {1024: 0.0388, 2048: 0.0589, 4096: 0.0990, 8192: 0.1804, 16384: 0.3422}
    paper_topk_ms = {1024: 0.013, 2048: 0.013, 4096: 0.014, 8192: 0.018, 16384: 0.022}

    def median_us(fn, n, warm):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in evs:
            a.record(); fn(); b.record()
        torch.cuda.synchronize()
        xs = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
        return xs[len(xs) // 2]

    rows = []
    for P in (1024, 2048, 4096, 8192, 16384):
        wl = W.build(f"paper_appendix_P{P}", 6, dtype=torch.bfloat16, B=32, H=32, Hkv=8, D=128, S=8,
                     seq_lens=[P * 8] * 32, top_k=64, key_mode="shift", plant_mode="none", permute=True,
                     device=dev, poison=False)
        row = {"pages": P, "kv_len": P * 8, "paper_h100_score_us": paper_score_ms[P] * 1e3,
               "paper_h100_topk_us": paper_topk_ms[P] * 1e3}
        stride = (wl.max_pages + 63) // 64 * 64
        buf = torch.empty((wl.B, wl.Hkv, stride), device=dev, dtype=torch.float32)
        for name, sd in (("fp32_stats", torch.float32), ("bf16_stats", torch.bfloat16)):
            sess = DecodeSession(wl, want_scores=False, stats_dtype=sd)
            sess.update_page_stats()
            row[f"score_us_{name}"] = median_us(lambda: sess.page_scores(buf), 100, 20)
            stat_bytes = wl.B * P * sess.page_stats.shape[1]
            row[f"score_GBps_{name}"] = stat_bytes / row[f"score_us_{name}"] / 1e3
            if sd == torch.bfloat16:
                # Ablation (Appendix A's unfused baseline): the same scores from library launches on a contiguous,
                # already gathered copy of the statistics -- a batched GEMM q . mean^T that writes the [B, H, P]
                # intermediate, the rank-one offset, the max over the group. Not part of the product path.
                ptl = wl.page_table[:, :P].long()
                means_c = sess.page_mean[ptl].permute(0, 2, 1, 3).contiguous()        # [B, Hkv, P, D] bf16
                stds_c = sess.page_std[ptl].permute(0, 2, 1).contiguous()             # [B, Hkv, P] fp32
                qg = wl.q.view(wl.B, wl.Hkv, wl.G, wl.D)
                off = (wl.lam * qg.float().norm(dim=-1)).unsqueeze(-1)                # [B, Hkv, G, 1]
                def naive():
                    dots = torch.matmul(qg, means_c.transpose(-1, -2)).float()        # [B, Hkv, G, P]
                    dots.addcmul_(off, stds_c.unsqueeze(2))
                    return dots.amax(dim=2)
                row["naive_library_launches_us_bf16_stats"] = median_us(naive, 100, 20)
                ref = naive()
                sess.page_scores(buf)
                row["naive_max_abs_diff"] = float((ref - buf[:, :, :P]).abs().max())
                del means_c, stds_c, ref
            if sd == torch.float32:
                row["topk_us"] = median_us(lambda: sess.select_topk(buf), 300, 50)
                # Fig. 2 of the paper: attention over a 512-token budget (k = 64 pages of 8) vs dense
                row["sparse_decode_us_k64"] = median_us(sess.sparse_paged_decode, 50, 10)
                if P <= 4096:
                    row["dense_decode_us"] = median_us(sess.dense_paged_decode, 10, 3)
            del sess
        rows.append(row)
        del wl, buf
        torch.cuda.empty_cache()
    # Fig. 2 of the paper: 32 q / 8 KV heads, D = 128, S = 8, budget 512 tokens (k = 64 pages), batch 80, 32K context:
    # score + top-k + sparse attention against dense attention (the paper: 11.4x over dense FlashInfer on one H100)
    wl = W.build("paper_fig2_b80_32k", 6, dtype=torch.bfloat16, B=80, H=32, Hkv=8, D=128, S=8, seq_lens=[32768] * 80,
                 top_k=64, key_mode="shift", plant_mode="none", permute=True, device=dev, poison=False)
    fig2 = {"batch": 80, "kv_len": 32768, "budget_tokens": 512, "paper_h100_speedup_vs_dense_flashinfer": 11.4}
    for name, sd in (("fp32_stats", torch.float32), ("bf16_stats", torch.bfloat16)):
        sess = DecodeSession(wl, want_scores=False, stats_dtype=sd)
        sess.update_page_stats()
        fig2[f"sparse_path_us_{name}"] = median_us(lambda: sess.decode_step(refresh_tail=False), 100, 20)
        if sd == torch.float32:
            fig2["dense_us"] = median_us(sess.dense_paged_decode, 20, 5)
        fig2[f"speedup_vs_own_dense_{name}"] = fig2["dense_us"] / fig2[f"sparse_path_us_{name}"]
        del sess
    print(json.dumps({"paper_shapes": {"batch": 32, "fig2": fig2, "q_heads": 32, "kv_heads": 8, "head_dim": 128, "page_size": 8,
                                        "top_k_pages": 64, "lambda": 0.5, "rows": rows,
                                        "note": "paper columns: one NVIDIA H100, bf16 scores (Appendix A and B); ours: one MI355X"}}))


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload, if any."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == kernel.split("(")[0]:
            return float(parts[2])
    return None


def cpu_baseline(wl, sess):
    """The float64 oracle (as it stands, OpenMP over rows) on the host cores, on the whole batch of the workload:
    tail-page statistics refresh + scores + top-k + sparse attention per step, timed for about 10 s."""
    import numpy as np
    import torch
    import oracle
    from oracle import OracleCache
    nseq = wl.B
    pages = [wl.num_pages(b) for b in range(nseq)]
    a = wl.host_arrays()
    oc = OracleCache(a["k_cache"], a["v_cache"], a["page_table"], a["seq_lens"], wl.H)
    q = a["q"]
    lens = a["seq_lens"].astype(np.int32)
    mean_all, std_all = oracle.new_stat_cache(oc)
    t0 = time.time()
    oracle.update_stats(oc, mean_all, std_all)       # bulk build, like the GPU's prefill-time build (not in the step)
    bulk_s = time.time() - t0
    reps, t_step = 0, 0.0
    while reps < 3 or (t_step < 10.0 and reps < 2000):  # about 10 s of wall time on the host cores
        t0 = time.time()
        oracle.update_stats(oc, mean_all, std_all, lens - 1, lens)
        oracle.sparse_decode_step(oc, q, mean_all, std_all, wl.lam, sess.top_k, 0.0, want_scores=False)
        t_step += time.time() - t0
        reps += 1
    per_step = t_step / reps
    return {"value": per_step * 1e6, "unit": "us/step", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"the whole batch ({nseq} sequences, {nseq * wl.Hkv} rows, {sum(pages)} pages), {reps} steps "
                      f"timed, not scaled; the oracle's bulk statistics build took {bulk_s:.2f} s (not in the step)",
            "sample_seconds_per_step": per_step}


if __name__ == "__main__":
    main()
