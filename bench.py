#!/usr/bin/env python3
"""Benchmark of the SuffixDecoding draft-generation path on one MI355X.

A step is one decode step over the whole batch: sd_speculate (match, expand, select), the
simulated greedy verifier, sd_accept, and sd_index_append of the accepted + bonus tokens.
The two index builds (global corpus, request contexts) happen once per run and are timed
separately in the same run (index_build_tokens_per_s).  Inputs are synthetic, resident in HBM
before any timed region starts.

Prints ONE JSON line.  `value` = speculation trees per second over K timed steps.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def _traffic_from_profiles(kernel: str, workload: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), if a summary
    for this kernel and workload has been committed under profiles/."""
    path = os.path.join(ROOT, "profiles", "%s_%s_pmc.md" % (kernel, workload))
    try:
        m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def cpu_baseline(w, n_requests: int, build_tokens: int):
    """The oracle as it stands, single thread, on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    from tests import parity
    docs = w.docs()
    # (a) index build: plain trie over the first documents, about build_tokens tokens
    t = oracle.Trie(w.D)
    n = 0
    t0 = time.perf_counter()
    for d in docs:
        t.add_doc(d)
        n += len(d)
        if n >= build_tokens:
            break
    build_s = time.perf_counter() - t0
    del t
    # (b) draft generation for the first n_requests requests against the full corpus; the
    # global trie holds exactly the suffixes those requests can reach
    contexts = [w.contexts[b] for b in range(n_requests)]
    tg = parity.oracle_global_trie(docs, w.D, w.vocab, contexts, w.P)
    tries = []
    for x in contexts:
        tr = oracle.Trie(w.D)
        tr.append(x)
        tries.append(tr)
    reps = []
    for _ in range(5):   # median of five passes over the sample
        t0 = time.perf_counter()
        drafted = 0
        for x, tr in zip(contexts, tries):
            g = oracle.generate(tg, tr, x, w.P, w.alpha, w.min_score)
            drafted += g["n_nodes"]
        reps.append(time.perf_counter() - t0)
    spec_s = sorted(reps)[len(reps) // 2]
    return {
        "value": n_requests / spec_s, "unit": "trees/s", "cores": 1, "kind": "oracle",
        "sample": "first %d requests of the batch against the full %d-token corpus "
                  "(GenerateCandidateTree only, tries prebuilt, median of five passes); build leg: plain trie over the "
                  "first %d corpus tokens" % (n_requests, len(w.corpus), n),
        "us_per_drafted_token": spec_s / max(drafted, 1) * 1e6,
        "first_pass_trees_per_s": n_requests / reps[0],   # caches cold: every later pass is faster
        "index_build_tokens_per_s": n / build_s,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--build-reps", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true",
                    help="enqueue every step from the host instead of replaying a captured HIP graph")
    ap.add_argument("--steps-per-graph", type=int, default=0,
                    help="decode steps captured into one HIP graph for the timed loop; 0 (default): "
                         "all of them, one graph launch for the timed region (the steps depend on "
                         "each other through device memory only); 1: one launch per step")
    ap.add_argument("--separate-calls", action="store_true",
                    help="end the step with sd_accept, the collection glue and sd_index_append "
                         "as three launches instead of one fused launch")
    ap.add_argument("--two-launches", action="store_true",
                    help="sd_speculate and sd_accept_append as two launches per step instead of "
                         "sd_accept_append_speculate (the end of a step and the next draft in one)")
    ap.add_argument("--throughput-batches", default="1024,4096,8192",
                    help="batch sizes beyond the workload's own at which sd_speculate is timed as "
                         "throughput work (several workgroups per compute unit); empty: skip")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (the path has no "
              "multi-GPU leg: requests are independent, so more GPUs would each take a share of "
              "the batch with a replica of the global index)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2411_04975_amd as sd
    from workloads import CONFIGS, make_workload, verifier
    from workloads.synth import extra_contexts

    K, W = args.steps, args.warmup
    cfg = CONFIGS[args.workload]
    mn = int(np.floor(cfg["alpha"] * cfg["P"]))
    total_steps = K + W
    w = make_workload(args.workload, seed=args.seed, future_len=(total_steps + 2) * (mn + 1) + mn + 2)
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    B, ctx_len = w.batch, w.ctx_len
    n_tokens, n_docs = int(w.corpus.shape[0]), len(w.doc_offsets) - 1

    i32 = torch.int32
    d_corpus = torch.from_numpy(w.corpus).to(dev)
    d_doc_off = torch.from_numpy(w.doc_offsets).to(dev)
    d_ctx = torch.from_numpy(w.contexts.reshape(-1)).to(dev)
    d_ctx_off = torch.arange(0, (B + 1) * ctx_len, ctx_len, dtype=torch.int64, device=dev)
    d_future = torch.from_numpy(w.future).to(dev)
    d_slots = torch.arange(B, dtype=i32, device=dev)
    max_ctx = ctx_len + (total_steps + 1) * (mn + 1)

    ctx = sd.sd_create(w.vocab, w.D, w.P, w.alpha, w.min_score, B, max_ctx, n_tokens + n_docs, 0)
    trees = sd.Trees(B, mn, dev)
    d_target = torch.zeros((B, mn + 1), dtype=i32, device=dev)
    d_alen = torch.full((B,), -1, dtype=i32, device=dev)
    d_apath = torch.zeros((B, mn), dtype=i32, device=dev)
    d_bonus = torch.zeros(B, dtype=i32, device=dev)
    d_new = torch.zeros(B * (mn + 1), dtype=i32, device=dev)
    d_newoff = torch.zeros(B + 1, dtype=i32, device=dev)
    d_pos = torch.zeros(B, dtype=i32, device=dev)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---- index builds (timed separately, inputs already in HBM) -------------------------
    def build_global():
        sd.sd_index_build(ctx, sd.SD_SCOPE_GLOBAL, None, d_corpus, d_doc_off, n_tokens)

    def build_requests():
        sd.sd_index_build(ctx, sd.SD_SCOPE_REQUESTS, d_slots, d_ctx, d_ctx_off, B * ctx_len)

    build_global()
    torch.cuda.synchronize()
    # The hand-written streaming copy of known size (the corpus: 4 B read + 4 B written per
    # token) lets rocprofv3 counter runs of this script calibrate FETCH_SIZE / WRITE_SIZE; the
    # same kernel over 2 x 512 MiB gives the achievable HBM rate of this run.
    calib = torch.empty_like(d_corpus)
    if n_tokens % 4 == 0:
        verifier.stream_copy(d_corpus, calib)
    torch.cuda.synchronize()
    del calib
    big_a = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
    big_b = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
    big_a.zero_()
    copy_ms = []
    for _ in range(6):
        e0, e1 = ev(), ev()
        e0.record()
        verifier.stream_copy(big_a, big_b)
        e1.record()
        torch.cuda.synchronize()
        copy_ms.append(e0.elapsed_time(e1))
    achievable_gbs = 2.0 * big_a.numel() / (min(copy_ms[1:]) * 1e-3) / 1e9
    del big_a, big_b
    build_ms = []
    for _ in range(args.build_reps):
        e0, e1 = ev(), ev()
        e0.record()
        build_global()
        e1.record()
        torch.cuda.synchronize()
        build_ms.append(e0.elapsed_time(e1))
    build_ms.sort()
    g_build_ms = build_ms[len(build_ms) // 2]
    sd.sd_debug_profile(ctx, 1)
    build_global()
    prof_build = sd.sd_debug_profile_read(ctx)
    sd.sd_debug_profile(ctx, 0)
    e0, e1 = ev(), ev()
    e0.record()
    build_requests()
    e1.record()
    torch.cuda.synchronize()
    r_build_ms = e0.elapsed_time(e1)

    # ---- decode steps ---------------------------------------------------------------------
    def step_separate():
        sd.sd_speculate(ctx, d_slots, trees)
        verifier.targets(trees.n_nodes, trees.parents, d_future, d_pos, d_target)
        sd.sd_accept(ctx, trees, B, d_target, d_alen, d_apath, d_bonus)
        verifier.collect(trees.tokens, d_alen, d_apath, d_bonus, d_new, d_newoff, d_pos)
        sd.sd_index_append(ctx, d_slots, d_new, d_newoff)

    def step_fused():
        # the verifier stand-in moves its positions on by what the previous step produced;
        # sd_accept_append does sd_accept and sd_index_append of the result in one launch
        sd.sd_speculate(ctx, d_slots, trees)
        verifier.targets(trees.n_nodes, trees.parents, d_future, d_pos, d_target, advance=d_alen)
        sd.sd_accept_append(ctx, trees, d_slots, d_target, d_alen, d_apath, d_bonus)

    def step_next():
        # One library launch per step: the trees hold the current drafts; the verifier stand-in
        # produces their target tokens; sd_accept_append_speculate ends the step (acceptance,
        # append) and drafts the next trees from the extended contexts.  Per step the same
        # work as above: one speculation, one verification, one acceptance, one append.
        verifier.targets(trees.n_nodes, trees.parents, d_future, d_pos, d_target, advance=d_alen)
        sd.sd_accept_append_speculate(ctx, trees, d_slots, d_target, d_alen, d_apath, d_bonus)

    one_launch = not (args.separate_calls or args.two_launches)
    step = step_separate if args.separate_calls else step_fused if args.two_launches else step_next

    def reset():
        build_requests()
        d_pos.zero_()
        d_alen.fill_(-1)
        if one_launch:  # the first drafts: every later step leaves the next ones behind
            sd.sd_speculate(ctx, d_slots, trees)

    # The timed loop replays a HIP graph captured from the steps: the same kernels, enqueued by
    # the same C-ABI calls, without the host between them (a graph launch costs about 4 us, so
    # one graph holds all timed steps; --steps-per-graph 1 replays step by step, --no-graph
    # times host-side enqueueing instead).
    for _ in range(W):
        step()
    torch.cuda.synchronize()
    graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        torch.cuda.synchronize()
        S = K if args.steps_per_graph <= 0 else max(1, min(args.steps_per_graph, K))
        graph_s = graph
        if S > 1:
            graph_s = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph_s):
                for _ in range(S):
                    step()
            torch.cuda.synchronize()
        reset()                       # capture ran no work; start the timed region from a
        for _ in range(W):            # known state: W eager warm-up steps after a rebuild
            step()
        torch.cuda.synchronize()
    run_step = graph.replay if graph is not None else step
    t0 = time.perf_counter()
    if graph is not None:
        for _ in range(K // S):
            graph_s.replay()
        for _ in range(K % S):
            graph.replay()
    else:
        for _ in range(K):
            step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    mean_nodes = float(trees.n_nodes.float().mean().item())
    mean_accept = float(d_alen.float().mean().item())
    stats = sd.sd_get_stats(ctx)
    assert stats["err_bad_token"] == 0 and stats["err_bad_slot"] == 0 and \
        stats["err_ctx_overflow"] == 0, stats

    # ---- per-step latency (each step bracketed by events and synchronised) ----------------
    reset()
    for _ in range(W):
        step()
    torch.cuda.synchronize()
    lat = []
    for _ in range(K):
        e0, e1 = ev(), ev()
        e0.record()
        run_step()
        e1.record()
        torch.cuda.synchronize()
        lat.append(e0.elapsed_time(e1))
    lat.sort()
    step_latency = {"median": lat[len(lat) // 2], "p99": lat[min(len(lat) - 1, int(0.99 * len(lat)))],
                    "max": lat[-1]}

    # ---- sd_speculate alone: median over 50 calls from one fixed state, and against batch ---
    reset()
    for _ in range(W):
        step()
    torch.cuda.synchronize()

    def time_speculate(slots_t, reps):
        for _ in range(5):
            sd.sd_speculate(ctx, slots_t, trees)
        torch.cuda.synchronize()
        run = None
        if not args.no_graph:
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2):
                sd.sd_speculate(ctx, slots_t, trees)
            torch.cuda.synchronize()
            run = g2.replay
        else:
            run = lambda: sd.sd_speculate(ctx, slots_t, trees)
        ts = []
        for _ in range(reps):
            e0, e1 = ev(), ev()
            e0.record()
            run()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        ts.sort()
        return ts[len(ts) // 2]

    spec_ms = time_speculate(d_slots, 50)
    latency_by_batch = {}
    nb = 1
    while nb < B:
        latency_by_batch[str(nb)] = time_speculate(d_slots[:nb].contiguous(), 20) * 1e3
        nb *= 4
    latency_by_batch[str(B)] = spec_ms * 1e3

    # ---- sd_speculate against the amount of work: the same batch with contexts cut down to
    # their last L tokens (0: nothing to do at all; 1: one pattern, one bucket; 64: every
    # pattern length and every expansion, next to no scan).  Kernel time per launch, 20
    # launches back to back in one graph: what is left at L = 0 is launch and fixed cost, and
    # every dependent load on the path from there shows as about a microsecond.
    def kernel_us(reps=20):
        for _ in range(3):
            sd.sd_speculate(ctx, d_slots, trees)
        torch.cuda.synchronize()
        gk = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gk):
            for _ in range(reps):
                sd.sd_speculate(ctx, d_slots, trees)
        torch.cuda.synchronize()
        gk.replay()
        torch.cuda.synchronize()
        ts = []
        for _ in range(5):
            e0, e1 = ev(), ev()
            e0.record()
            gk.replay()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3 / reps)
        return min(ts)

    us_by_context = {}
    ctx2d = d_ctx.view(B, ctx_len)
    for L in sorted({0, 1, 64, 1024, ctx_len}):
        if L > ctx_len:
            continue
        cut = ctx2d[:, ctx_len - L:].contiguous().reshape(-1) if L > 0 else d_ctx[:1]
        off = torch.arange(0, (B + 1) * L, max(L, 1), dtype=torch.int64, device=dev) if L > 0 \
            else torch.zeros(B + 1, dtype=torch.int64, device=dev)
        sd.sd_index_build(ctx, sd.SD_SCOPE_REQUESTS, d_slots, cut, off, B * L)
        us_by_context[str(L)] = kernel_us()
    build_requests()

    # ---- per-kernel durations (HIP events on the launch stream) over the same K steps -----
    reset()
    for _ in range(W):
        step()
    torch.cuda.synchronize()
    sd.sd_debug_profile(ctx, 1)
    sd.sd_debug_profile_read(ctx)
    for _ in range(K):
        step()
    prof = sd.sd_debug_profile_read(ctx)
    # ---- algorithmic bytes of the same launches (counting variants, untimed) --------------
    reset()
    for _ in range(W):
        step()
    torch.cuda.synchronize()
    sd.sd_debug_profile(ctx, 2)
    sd.sd_debug_profile_read(ctx)
    for _ in range(K):
        step()
    cnt = sd.sd_debug_profile_read(ctx)
    sd.sd_debug_profile(ctx, 0)

    # ---- latency profile of sd_speculate: wall-clock marks inside the timing variant --------
    reset()
    for _ in range(W):
        step()
    sd.sd_debug_profile(ctx, 3)
    sd.sd_debug_profile_read(ctx)
    for _ in range(3):
        sd.sd_speculate(ctx, d_slots, trees)
    rt, khz = sd.sd_debug_read_request_ticks(ctx, B)
    ut = sd.sd_debug_read_unit_ticks(ctx, B)   # [B, 2, P, 4] microseconds
    sd.sd_debug_profile_read(ctx)
    sd.sd_debug_profile(ctx, 0)
    us = 1e3 / max(khz, 1)
    nw = int(rt[0, 0, 7]) if rt[0, 0, 7] else 16
    rt = rt[:, :nw, :].astype(np.int64)
    start = (rt[:, 0, 0] - rt[:, 0, 0].min()) * us
    req_end = start + rt[:, :, 4].max(axis=1) * us
    runs_us = (rt[:, :, 3] - rt[:, :, 2]) * us

    def pct(a, q):
        return float(np.percentile(a, q))

    # the requests that finish last decide the kernel's duration: what their longest unit was
    slowest = []
    for b_ in np.argsort(req_end)[::-1][:4]:
        src_, p_ = np.unravel_index(int(np.argmax(ut[b_, :, :, 3])), ut[b_, :, :, 3].shape)
        slowest.append({"request": int(b_), "finished_at": float(req_end[b_]),
                        "occurrences_and_matches_done": float(rt[b_, 0, 1] * us),
                        "runs": int(rt[b_, 0, 5]), "longest_wave_in_runs": float(runs_us[b_].max()),
                        "longest_unit": {"index": "request" if src_ else "global", "p": int(p_) + 1,
                                         "root_children_at": float(ut[b_, src_, p_, 2]),
                                         "done_at": float(ut[b_, src_, p_, 3])}})

    latency_profile = {
        "note": "wall-clock marks (100 MHz) inside the timing variant of k_speculate, batch %d, "
                "one workgroup of %d waves per request; microseconds" % (B, nw),
        "workgroup_start_spread": float(start.max()),
        "occurrences_and_matches_done": {"p50": pct(rt[:, 0, 1] * us, 50), "max": float(rt[:, 0, 1].max() * us)},
        "longest_wave_in_runs": {"p50": pct(runs_us.max(axis=1), 50), "p90": pct(runs_us.max(axis=1), 90),
                                 "max": float(runs_us.max())},
        "request_finished_at": {"p50": pct(req_end, 50), "p90": pct(req_end, 90), "max": float(req_end.max())},
        "slowest_requests": slowest,
        "runs_per_request_mean": float(rt[:, 0, 5].mean()),
        "last_token_occurrences_in_context": {"mean": float(rt[:, 0, 6].mean()), "max": int(rt[:, 0, 6].max())},
    }

    # the dominant kernel: k_speculate, in the one-launch step its form that accepts and appends
    # first (the counting variant exists for the separate kernels, which the library falls
    # back to while counting; the bytes of acceptance and append are added by formula: tree
    # tokens and parents, target tokens, path, two result words, appended tokens)
    kname = "accept_speculate" if one_launch else "speculate"
    exp_ms = prof[kname]["ms"] / max(prof[kname]["launches"], 1)
    exp_bytes = cnt["speculate"]["algo_bytes"] / max(cnt["speculate"]["launches"], 1)
    if one_launch:
        exp_bytes += B * (8.0 * mean_nodes + 4.0 * (mn + 1) + 4.0 * mn + 8.0 + 4.0 * (mean_accept + 1))
    achieved = exp_bytes / (exp_ms * 1e-3) / 1e9 if exp_ms > 0 else 0.0
    roofline = {"bound": "hbm",
                "kernel": "k_speculate<accept and append first>" if one_launch else "k_speculate",
                "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": _traffic_from_profiles("k_speculate", w.name),
                "algo_bytes_per_launch": exp_bytes, "avg_launch_ms": exp_ms,
                "achievable": achievable_gbs, "frac_of_achievable": achieved / achievable_gbs}
    N = n_tokens + n_docs
    sc = prof_build["sort_scatter"]
    sc_ms = sc["ms"] / max(sc["launches"], 1)
    sc_ach = 24.0 * N / (sc_ms * 1e-3) / 1e9 if sc_ms > 0 else 0.0
    roofline_build = {"bound": "hbm", "kernel": "k_radix_scatter", "achieved": sc_ach,
                      "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": sc_ach / HBM_PEAK_GBS,
                      "traffic": _traffic_from_profiles("k_radix_scatter", w.name),
                      "algo_bytes_per_launch": 24.0 * N, "avg_launch_ms": sc_ms,
                      "launches_per_build": sc["launches"], "achievable": achievable_gbs,
                      "frac_of_achievable": sc_ach / achievable_gbs}
    kernels_ms = {k: v["ms"] / max(v["launches"], 1) for k, v in prof.items() if v["launches"]}
    build_kernels_ms = {k: v["ms"] for k, v in prof_build.items() if v["launches"]}

    out = {
        "metric": "speculation trees/sec (batch %d, %s-token corpus)" % (B, format(n_tokens, ",")),
        "value": B * K / elapsed, "unit": "trees/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": elapsed / K * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int32+f64", "data": "synthetic",
        "launch": ("hip-graph replay, %d step%s per graph" % (S, "" if S == 1 else "s"))
                  if graph is not None else "host enqueue",
        "config": {"workload": w.name, "batch": B, "ctx_len": ctx_len, "corpus_tokens": n_tokens,
                   "corpus_docs": n_docs, "vocab": w.vocab, "D": w.D, "P": w.P, "alpha": w.alpha,
                   "min_score": w.min_score, "max_nodes": mn, "seed": args.seed,
                   "generator": {k: v for k, v in w.params.items()
                                 if k in ("kind", "n_templates", "template_len", "span", "mut",
                                          "doc_len", "zipf_s")},
                   "step": ("sd_speculate + simulated verifier + sd_accept + sd_index_append"
                            if args.separate_calls else
                            "sd_speculate + simulated verifier + sd_accept_append"
                            if args.two_launches else
                            "simulated verifier + sd_accept_append_speculate (verification of "
                            "the current drafts, acceptance, append, next drafts)")},
        "index_build_tokens_per_s": n_tokens / (g_build_ms * 1e-3),
        "index_build_ms": g_build_ms, "request_build_ms": r_build_ms,
        "request_build_tokens_per_s": B * ctx_len / (r_build_ms * 1e-3),
        "step_latency_ms": step_latency,
        "speculate_only_ms_median": spec_ms, "speculate_only_trees_per_s": B / (spec_ms * 1e-3),
        "speculate_latency_us_by_batch": latency_by_batch,
        "speculate_kernel_us_by_context_tokens": us_by_context,
        "speculate_latency_profile": latency_profile,
        "stream_copy_gbs": achievable_gbs,
        "mean_tree_nodes": mean_nodes, "mean_accept_len": mean_accept,
        "kernel_ms_per_launch": kernels_ms, "build_kernel_ms_total": build_kernels_ms,
        "roofline": roofline, "roofline_build": roofline_build,
        "index_bytes": stats["index_bytes"], "scratch_bytes": stats["scratch_bytes"],
    }
    # ---- empirical entropy of the global index (the paper's effectiveness predictor) -------
    t0 = time.perf_counter()
    ent_bits, ent_weight = sd.sd_index_entropy(ctx)
    ent_ms = (time.perf_counter() - t0) * 1e3
    t0 = time.perf_counter()
    sd.sd_index_entropy(ctx)
    ent_ms = min(ent_ms, (time.perf_counter() - t0) * 1e3)
    out["index_entropy"] = {"mean_bits": ent_bits, "weight": ent_weight, "ms": ent_ms}

    # ---- online insertion: the outputs of one batch (B documents of max_nodes + 1 tokens) are
    # added to the global index; done last because it grows the index.  The context was sized
    # for the corpus alone, so a second context with room for the insertions does this leg.
    ins_docs, ins_len, ins_reps = B, mn + 1, 3
    ctx2 = sd.sd_create(w.vocab, w.D, w.P, w.alpha, w.min_score, 1, 64,
                        n_tokens + n_docs + ins_reps * ins_docs * (ins_len + 1), 0)
    sd.sd_index_build(ctx2, sd.SD_SCOPE_GLOBAL, None, d_corpus, d_doc_off, n_tokens)
    d_ins = d_future[:, :ins_len * ins_reps].contiguous()
    d_ins_off = torch.arange(0, (ins_docs + 1) * ins_len, ins_len, dtype=torch.int64, device=dev)
    ins_ms = []
    for r in range(ins_reps):
        chunk = d_ins[:, r * ins_len:(r + 1) * ins_len].contiguous().reshape(-1)
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        sd.sd_index_insert(ctx2, chunk, d_ins_off, ins_docs * ins_len)
        e1.record()
        torch.cuda.synchronize()
        ins_ms.append(e0.elapsed_time(e1))
    ins_ms.sort()
    out["index_insert"] = {"documents": ins_docs, "tokens": ins_docs * ins_len,
                           "ms_median": ins_ms[len(ins_ms) // 2],
                           "tokens_per_s": ins_docs * ins_len / (ins_ms[len(ins_ms) // 2] * 1e-3)}
    sd.sd_destroy(ctx2)
    sd.sd_destroy(ctx)

    # ---- sd_speculate as throughput work: batches of several workgroups per compute unit ----
    # The workload's own batch is one workgroup per compute unit and bound by its slowest
    # request; these batches show what the same kernel sustains once the compute units have
    # requests to overlap.  1024 further contexts are drawn like the workload's; slot i holds
    # context i % 1024 rotated by (i / 1024) eighths of its length, so every slot asks about
    # another place of the text.
    wide = sorted({int(v) for v in args.throughput_batches.split(",") if v.strip()})
    wide = [nb for nb in wide if nb > B]
    if wide:
        drawn = extra_contexts(cfg, args.seed, 1024)
        nmax = wide[-1]
        reps = (nmax + 1023) // 1024
        allc = np.concatenate([np.roll(drawn, -(r * ctx_len // 8) % ctx_len, axis=1) for r in range(reps)])[:nmax]
        d_wctx = torch.from_numpy(np.ascontiguousarray(allc).reshape(-1)).to(dev)
        del allc, drawn
        d_woff = torch.arange(0, (nmax + 1) * ctx_len, ctx_len, dtype=torch.int64, device=dev)
        d_wslots = torch.arange(nmax, dtype=i32, device=dev)
        ctx3 = sd.sd_create(w.vocab, w.D, w.P, w.alpha, w.min_score, nmax, ctx_len + 1,
                            n_tokens + n_docs, 0)
        sd.sd_index_build(ctx3, sd.SD_SCOPE_GLOBAL, None, d_corpus, d_doc_off, n_tokens)
        sd.sd_index_build(ctx3, sd.SD_SCOPE_REQUESTS, d_wslots, d_wctx, d_woff, nmax * ctx_len)
        torch.cuda.synchronize()
        by_batch = {}
        for nb in wide:
            tr = sd.Trees(nb, mn, dev)
            sl = d_wslots[:nb].contiguous()
            for _ in range(3):
                sd.sd_speculate(ctx3, sl, tr)
            torch.cuda.synchronize()
            gw = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gw):
                for _ in range(10):
                    sd.sd_speculate(ctx3, sl, tr)
            torch.cuda.synchronize()
            ts = []
            for _ in range(6):
                e0, e1 = ev(), ev()
                e0.record()
                gw.replay()
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1) / 10)
            ms = min(ts[1:])
            sd.sd_debug_profile(ctx3, 2)
            sd.sd_debug_profile_read(ctx3)
            sd.sd_speculate(ctx3, sl, tr)
            nbytes = sd.sd_debug_profile_read(ctx3)["speculate"]["algo_bytes"]
            sd.sd_debug_profile(ctx3, 0)
            gbs = nbytes / (ms * 1e-3) / 1e9
            by_batch[str(nb)] = {"us_per_launch": ms * 1e3, "trees_per_s": nb / (ms * 1e-3),
                                 "algo_bytes_per_launch": nbytes, "achieved_gbs": gbs,
                                 "frac_of_peak": gbs / HBM_PEAK_GBS,
                                 "frac_of_achievable": gbs / achievable_gbs,
                                 "mean_tree_nodes": float(tr.n_nodes.float().mean().item())}
            del gw, tr
        st3 = sd.sd_get_stats(ctx3)
        assert st3["err_bad_token"] == 0 and st3["err_bad_slot"] == 0, st3
        sd.sd_destroy(ctx3)
        out["speculate_throughput_by_batch"] = by_batch
        # the same kernel with the compute units full: its share of the roofline there
        top_b = str(wide[-1])
        out["roofline"]["sd_speculate_at_batch_%s" % top_b] = {
            "achieved": by_batch[top_b]["achieved_gbs"], "frac": by_batch[top_b]["frac_of_peak"],
            "frac_of_achievable": by_batch[top_b]["frac_of_achievable"],
            "avg_launch_ms": by_batch[top_b]["us_per_launch"] * 1e-3,
            "algo_bytes_per_launch": by_batch[top_b]["algo_bytes_per_launch"]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, n_requests=min(32, B), build_tokens=300_000)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
