#!/usr/bin/env python3
"""Benchmark of the SuffixDecoding draft-generation path on one MI355X.

A step is one decode step over the whole batch: the simulated greedy verifier on the current
drafts, then sd_accept_append_speculate (acceptance, append of the accepted + bonus tokens,
the next drafts): one speculation, one verification, one acceptance and one append per step.
The two index builds (global corpus, request contexts) happen once per run and are timed
separately in the same run (index_build_tokens_per_s).  Inputs are synthetic, resident in HBM
before any timed region starts.

Prints ONE JSON line.  `value` = speculation trees per second over K timed decode steps of the
headline workload (large); `other_workloads` holds the same figures for the agentic,
low-repetition and streaming configurations (streaming: per-step latency over its 64 steps).
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
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), and the
    commit the summary says it was measured at, if a summary for this kernel and workload has
    been committed under profiles/."""
    path = os.path.join(ROOT, "profiles", "%s_%s_pmc.md" % (kernel, workload))
    try:
        txt = open(path).read()
    except OSError:
        return None, None
    m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", txt)
    c = re.search(r"measured_at_commit:\s*([0-9a-f]+)", txt)
    return (float(m.group(1)) if m else None), (c.group(1) if c else None)


def _host_threads() -> int:
    """Threads the oracle's all-cores leg uses: the cores this process may run on, at most 16
    (the share of a one-GPU job on the benchmark machine)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def _cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


_CPU_LEG = {}   # what the forked workers of the all-cores leg inherit: tries, contexts, parameters


def _cpu_leg_chunk(bounds):
    """One worker's share of a pass of the all-cores leg: drafts for requests [lo, hi), `rounds`
    times over (a pass has to last much longer than handing the shares out and back)."""
    import oracle
    g = _CPU_LEG
    lo, hi, rounds = bounds
    n = 0
    for _ in range(rounds):
        n += sum(oracle.generate(g["tg"], g["tries"][i], g["contexts"][i], g["P"], g["alpha"],
                                 g["min_score"])["n_nodes"] for i in range(lo, hi))
    return n


def cpu_baseline(w, n_one: int, n_all: int, build_tokens: int):
    """The oracle as it stands on a bounded sample of the same workload: GenerateCandidateTree
    for the first requests of the batch against the full corpus, on one core and, over disjoint
    requests, on all the host cores this process has: one forked worker process per core, which
    inherits the prebuilt (read-only) tries.  Called before anything touches the GPU, so that
    forking is safe."""
    import concurrent.futures as cf
    import multiprocessing as mp
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
    # (b) draft generation; the global trie holds exactly the suffixes the sample can reach
    threads = _host_threads()
    n_all = max(n_one, min(n_all, w.batch))
    contexts = [w.contexts[b] for b in range(n_all)]
    tg = parity.oracle_global_trie(docs, w.D, w.vocab, contexts, w.P)

    def request_trie(x):
        tr = oracle.Trie(w.D)
        tr.append(x)
        return tr

    with cf.ThreadPoolExecutor(threads) as ex:
        tries = list(ex.map(request_trie, contexts))

        def draft(i):
            return oracle.generate(tg, tries[i], contexts[i], w.P, w.alpha, w.min_score)["n_nodes"]

        reps = []
        for _ in range(5):   # one thread: median of five passes over the first n_one requests
            t0 = time.perf_counter()
            drafted = sum(draft(i) for i in range(n_one))
            reps.append(time.perf_counter() - t0)
        one_s = sorted(reps)[len(reps) // 2]
    # all cores: the requests in as many contiguous shares as there are workers
    _CPU_LEG.update(tg=tg, tries=tries, contexts=contexts, P=w.P, alpha=w.alpha, min_score=w.min_score)
    cuts = [n_all * k // threads for k in range(threads + 1)]
    # rounds per pass: about a quarter of a second of work for each worker
    rounds = max(1, int(0.25 / max(one_s / n_one * (n_all / threads), 1e-6)))
    shares = [(cuts[k], cuts[k + 1], rounds) for k in range(threads) if cuts[k + 1] > cuts[k]]
    reps_all = []
    with mp.get_context("fork").Pool(len(shares)) as pool:
        pool.map(_cpu_leg_chunk, [(a, b, 1) for a, b, _ in shares])   # workers started, pages touched
        for _ in range(5):
            t0 = time.perf_counter()
            drafted_all = sum(pool.map(_cpu_leg_chunk, shares, chunksize=1))
            reps_all.append(time.perf_counter() - t0)
    all_s = sorted(reps_all)[len(reps_all) // 2]
    _CPU_LEG.clear()
    return {
        "value": n_all * rounds / all_s, "unit": "trees/s", "cores": len(shares), "kind": "oracle",
        "sample": "GenerateCandidateTree for the first %d requests of the batch against the full "
                  "%d-token corpus in %d worker processes over disjoint requests (tries prebuilt "
                  "and inherited read-only, median of five passes of %d rounds each); one-core figures: the first %d requests; "
                  "build leg: plain trie over the first %d corpus tokens on one thread"
                  % (n_all, len(w.corpus), len(shares), rounds, n_one, n),
        "cpu_model": _cpu_model(), "host_cpus_visible": os.cpu_count(),
        "us_per_drafted_token": all_s * len(shares) / max(drafted_all, 1) * 1e6,   # core time per token
        "one_thread": {"value": n_one / one_s, "unit": "trees/s", "cores": 1,
                       "us_per_drafted_token": one_s / max(drafted, 1) * 1e6,
                       "first_pass_trees_per_s": n_one / reps[0]},
        "index_build_tokens_per_s": n / build_s,
    }


class Run:
    """One workload on the device: inputs uploaded, context created, the decode step in its
    three forms, and the timing legs every workload gets."""

    def __init__(self, args, name, total_steps):
        import numpy as np
        import torch
        import paper_2411_04975_amd as sd
        from workloads import CONFIGS, make_workload, verifier
        self.np, self.torch, self.sd, self.verifier = np, torch, sd, verifier
        self.args = args
        cfg = CONFIGS[name]
        self.cfg = cfg
        mn = int(np.floor(cfg["alpha"] * cfg["P"]))
        self.mn = mn
        self.w = w = make_workload(name, seed=args.seed,
                                   future_len=(total_steps + 2) * (mn + 1) + mn + 2)
        self.dev = dev = torch.device("cuda", 0)
        torch.cuda.set_device(dev)
        self.B, self.ctx_len = B, ctx_len = w.batch, w.ctx_len
        self.n_tokens, self.n_docs = int(w.corpus.shape[0]), len(w.doc_offsets) - 1
        i32 = torch.int32
        self.d_corpus = torch.from_numpy(w.corpus).to(dev)
        self.d_doc_off = torch.from_numpy(w.doc_offsets).to(dev)
        self.d_ctx = torch.from_numpy(w.contexts.reshape(-1)).to(dev)
        self.d_ctx_off = torch.arange(0, (B + 1) * ctx_len, ctx_len, dtype=torch.int64, device=dev)
        self.d_future = torch.from_numpy(w.future).to(dev)
        self.d_slots = torch.arange(B, dtype=i32, device=dev)
        # request b lives in slot b: the decode step says so by passing no slot ids (which
        # spares every drafting workgroup one dependent load), unless --explicit-slot-ids
        self.step_slots = self.d_slots if args.explicit_slot_ids else None
        max_ctx = ctx_len + (total_steps + 1) * (mn + 1)
        self.ctx = sd.sd_create(w.vocab, w.D, w.P, w.alpha, w.min_score, B, max_ctx,
                                self.n_tokens + self.n_docs, 0)
        self.trees = sd.Trees(B, mn, dev)
        self.d_target = torch.zeros((B, mn + 1), dtype=i32, device=dev)
        self.d_alen = torch.full((B,), -1, dtype=i32, device=dev)
        self.d_apath = torch.zeros((B, mn), dtype=i32, device=dev)
        self.d_bonus = torch.zeros(B, dtype=i32, device=dev)
        self.d_new = torch.zeros(B * (mn + 1), dtype=i32, device=dev)
        self.d_newoff = torch.zeros(B + 1, dtype=i32, device=dev)
        self.d_pos = torch.zeros(B, dtype=i32, device=dev)
        self.one_launch = not (args.separate_calls or args.two_launches)
        self.step = (self.step_separate if args.separate_calls else
                     self.step_fused if args.two_launches else self.step_next)

    def close(self):
        self.sd.sd_destroy(self.ctx)

    def ev(self):
        return self.torch.cuda.Event(enable_timing=True)

    # ---- index builds -----------------------------------------------------------------------
    def build_global(self):
        self.sd.sd_index_build(self.ctx, self.sd.SD_SCOPE_GLOBAL, None, self.d_corpus,
                               self.d_doc_off, self.n_tokens)

    def build_requests(self):
        self.sd.sd_index_build(self.ctx, self.sd.SD_SCOPE_REQUESTS, self.d_slots, self.d_ctx,
                               self.d_ctx_off, self.B * self.ctx_len)

    def time_builds(self, reps):
        """Median of `reps` global builds and one request build, HIP events, inputs in HBM."""
        torch = self.torch
        self.build_global()
        torch.cuda.synchronize()
        ms = []
        for _ in range(reps):
            e0, e1 = self.ev(), self.ev()
            e0.record()
            self.build_global()
            e1.record()
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        ms.sort()
        e0, e1 = self.ev(), self.ev()
        e0.record()
        self.build_requests()
        e1.record()
        torch.cuda.synchronize()
        return ms[len(ms) // 2], e0.elapsed_time(e1)

    # ---- the decode step, three ways --------------------------------------------------------
    def step_separate(self):
        sd, v = self.sd, self.verifier
        sd.sd_speculate(self.ctx, self.step_slots, self.trees)
        v.targets(self.trees.n_nodes, self.trees.parents, self.d_future, self.d_pos, self.d_target)
        sd.sd_accept(self.ctx, self.trees, self.B, self.d_target, self.d_alen, self.d_apath, self.d_bonus)
        v.collect(self.trees.tokens, self.d_alen, self.d_apath, self.d_bonus, self.d_new,
                  self.d_newoff, self.d_pos)
        sd.sd_index_append(self.ctx, self.step_slots, self.d_new, self.d_newoff)

    def step_fused(self):
        # the verifier stand-in moves its positions on by what the previous step produced;
        # sd_accept_append does sd_accept and sd_index_append of the result in one launch
        sd, v = self.sd, self.verifier
        sd.sd_speculate(self.ctx, self.step_slots, self.trees)
        v.targets(self.trees.n_nodes, self.trees.parents, self.d_future, self.d_pos, self.d_target,
                  advance=self.d_alen)
        sd.sd_accept_append(self.ctx, self.trees, self.step_slots, self.d_target, self.d_alen,
                            self.d_apath, self.d_bonus)

    def step_next(self):
        # One library launch per step: the trees hold the current drafts; the verifier stand-in
        # produces their target tokens; sd_accept_append_speculate ends the step (acceptance,
        # append) and drafts the next trees from the extended contexts.
        self.verifier.targets(self.trees.n_nodes, self.trees.parents, self.d_future, self.d_pos,
                              self.d_target, advance=self.d_alen)
        self.sd.sd_accept_append_speculate(self.ctx, self.trees, self.step_slots, self.d_target,
                                           self.d_alen, self.d_apath, self.d_bonus)

    def reset(self):
        self.build_requests()
        self.d_pos.zero_()
        self.d_alen.fill_(-1)
        if self.one_launch:  # the first drafts: every later step leaves the next ones behind
            self.sd.sd_speculate(self.ctx, self.step_slots, self.trees)

    def warm(self, W):
        self.reset()
        for _ in range(W):
            self.step()
        self.torch.cuda.synchronize()

    def capture(self, n_steps):
        g = self.torch.cuda.CUDAGraph()
        with self.torch.cuda.graph(g):
            for _ in range(n_steps):
                self.step()
        self.torch.cuda.synchronize()
        return g

    def timed_steps(self, K, W, steps_per_graph):
        """Wall clock between device synchronisations over K steps that follow W warm-up steps
        from a fresh state.  The steps are replayed from a HIP graph captured through the same
        C-ABI calls (steps_per_graph <= 0: all K in one graph, one launch for the timed region;
        1: one launch per step), or enqueued from the host with --no-graph."""
        torch = self.torch
        self.warm(W)                  # also loads every kernel before capture
        S = 0
        graphs = None
        if not self.args.no_graph:
            S = K if steps_per_graph <= 0 else max(1, min(steps_per_graph, K))
            graphs = (self.capture(S), self.capture(1) if K % S else None)
            self.warm(W)              # capture ran no work: start again from a known state
        t0 = time.perf_counter()
        if graphs is not None:
            for _ in range(K // S):
                graphs[0].replay()
            for _ in range(K % S):
                graphs[1].replay()
        else:
            for _ in range(K):
                self.step()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, S

    def step_latency(self, K, W):
        """Every step its own launch (a one-step graph, or host enqueue), bracketed by events
        and synchronised: what a serving loop that waits for each step sees."""
        torch = self.torch
        self.warm(max(W, 1))
        run = self.step
        if not self.args.no_graph:
            run = self.capture(1).replay
            self.warm(W)
        lat = []
        for _ in range(K):
            e0, e1 = self.ev(), self.ev()
            e0.record()
            run()
            e1.record()
            torch.cuda.synchronize()
            lat.append(e0.elapsed_time(e1))
        lat.sort()
        return {"median": lat[len(lat) // 2], "p99": lat[min(len(lat) - 1, int(0.99 * len(lat)))],
                "max": lat[-1], "steps": K}

    def common_figures(self, K, W, build_reps):
        """The figures every workload reports."""
        B = self.B
        g_build_ms, r_build_ms = self.time_builds(build_reps)
        elapsed, S = self.timed_steps(K, W, self.args.steps_per_graph)
        mean_nodes = float(self.trees.n_nodes.float().mean().item())
        mean_accept = float(self.d_alen.float().mean().item())
        st = self.sd.sd_get_stats(self.ctx)
        assert st["err_bad_token"] == 0 and st["err_bad_slot"] == 0 and st["err_ctx_overflow"] == 0, st
        elapsed1, _ = self.timed_steps(K, W, 1)
        out = {
            "batch": B, "ctx_len": self.ctx_len, "corpus_tokens": self.n_tokens,
            "steps": K, "warmup": W,
            "ms_per_step": elapsed / K * 1e3, "trees_per_s": B * K / elapsed,
            "launch": ("hip-graph replay, %d step%s per graph" % (S, "" if S == 1 else "s"))
                      if S else "host enqueue",
            "ms_per_step_one_launch_per_step": elapsed1 / K * 1e3,
            "step_latency_ms": self.step_latency(K, W),
            "index_build_ms": g_build_ms,
            "index_build_tokens_per_s": self.n_tokens / (g_build_ms * 1e-3),
            "request_build_ms": r_build_ms,
            "request_build_tokens_per_s": B * self.ctx_len / (r_build_ms * 1e-3),
            "mean_tree_nodes": mean_nodes, "mean_accept_len": mean_accept,
            "index_bytes": st["index_bytes"], "scratch_bytes": st["scratch_bytes"],
        }
        # what the library's own counters say about all drafting calls so far
        if st["spec_requests"]:
            out["counters"] = {
                "requests_with_a_tree": st["spec_trees"] / st["spec_requests"],
                "mean_winning_p": st["spec_match_len"] / max(st["spec_trees"], 1),
                "mean_nodes_per_tree": st["spec_nodes"] / max(st["spec_trees"], 1),
                "trees_from_request_index": st["spec_from_request"] / max(st["spec_trees"], 1),
                "global_matches_by_per_p_search": st["spec_global_search"] / st["spec_requests"],
                "requests_with_long_request_lists": st["spec_request_wide"] / st["spec_requests"],
                "mean_accept_len": st["accept_len"] / max(st["accept_requests"], 1),
            }
        return out, elapsed, S


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64,
                    help="timed decode steps (default: as many as the streaming configuration "
                         "runs; the one graph launch and the closing synchronisation of the timed "
                         "region, some 50 us together, are spread over them)")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--others", default="agentic,lowrep,streaming",
                    help="further workloads whose step time, step latency and build rates go into "
                         "other_workloads (streaming always runs its 64 decode steps); empty: none")
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
    ap.add_argument("--explicit-slot-ids", action="store_true",
                    help="pass an array of slot ids (0, 1, 2, ...) to the calls of the decode step "
                         "instead of NULL, which stands for the same identity mapping")
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

    # The oracle's leg runs first: its all-cores part forks worker processes, which a process
    # that has initialised the GPU must not do.
    cpu_leg = None
    if not args.no_cpu_baseline:
        from workloads import make_workload
        wl = make_workload(args.workload, seed=args.seed)
        cpu_leg = cpu_baseline(wl, n_one=min(32, wl.batch), n_all=min(128, wl.batch), build_tokens=300_000)
        del wl

    import numpy as np
    import torch
    import paper_2411_04975_amd as sd
    from workloads import CONFIGS, verifier
    from workloads.synth import extra_contexts

    K, W = args.steps, args.warmup
    run = Run(args, args.workload, K + W)
    w, cfg, mn, dev = run.w, run.cfg, run.mn, run.dev
    B, ctx_len, n_tokens, n_docs = run.B, run.ctx_len, run.n_tokens, run.n_docs
    ctx, trees, d_slots, d_ctx = run.ctx, run.trees, run.d_slots, run.d_ctx
    ev, step, reset, one_launch = run.ev, run.step, run.reset, run.one_launch
    i32 = torch.int32

    run.build_global()
    torch.cuda.synchronize()
    # The hand-written streaming copy of known size (the corpus: 4 B read + 4 B written per
    # token) lets rocprofv3 counter runs of this script calibrate FETCH_SIZE / WRITE_SIZE; the
    # same kernel over 2 x 512 MiB gives the achievable HBM rate of this run.
    calib = torch.empty_like(run.d_corpus)
    if n_tokens % 4 == 0:
        verifier.stream_copy(run.d_corpus, calib)
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

    # what a load costs whose address comes from the load before it (one lane, random lines):
    # working sets that fit the L2, the memory-side cache, and neither
    dep_ns = {name: verifier.dependent_load_ns(lines, 20000, dev)
              for name, lines in (("2 MB", 1 << 14), ("64 MB", 1 << 19), ("2 GB", 1 << 24))}
    torch.cuda.empty_cache()

    head, elapsed, S = run.common_figures(K, W, args.build_reps)
    mean_nodes, mean_accept = head["mean_tree_nodes"], head["mean_accept_len"]
    sd.sd_debug_profile(ctx, 1)
    run.build_global()
    prof_build = sd.sd_debug_profile_read(ctx)
    sd.sd_debug_profile(ctx, 0)

    # ---- sd_speculate alone: median over 50 calls from one fixed state, and against batch ---
    run.warm(W)

    def time_speculate(slots_t, reps):
        for _ in range(5):
            sd.sd_speculate(ctx, slots_t, trees)
        torch.cuda.synchronize()
        if not args.no_graph:
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2):
                sd.sd_speculate(ctx, slots_t, trees)
            torch.cuda.synchronize()
            go = g2.replay
        else:
            go = lambda: sd.sd_speculate(ctx, slots_t, trees)
        ts = []
        for _ in range(reps):
            e0, e1 = ev(), ev()
            e0.record()
            go()
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
    run.build_requests()

    # ---- per-kernel durations (HIP events on the launch stream) over the same K steps -----
    run.warm(W)
    sd.sd_debug_profile(ctx, 1)
    sd.sd_debug_profile_read(ctx)
    for _ in range(K):
        step()
    prof = sd.sd_debug_profile_read(ctx)
    # ---- algorithmic bytes of the same launches (counting variants, untimed) --------------
    run.warm(W)
    sd.sd_debug_profile(ctx, 2)
    sd.sd_debug_profile_read(ctx)
    for _ in range(K):
        step()
    cnt = sd.sd_debug_profile_read(ctx)
    sd.sd_debug_profile(ctx, 0)

    # ---- latency profile of sd_speculate: wall-clock marks inside the timing variant --------
    run.warm(W)
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
    traffic, traffic_commit = _traffic_from_profiles("k_speculate", w.name)
    roofline = {"bound": "hbm",
                "kernel": "k_speculate<accept and append first>" if one_launch else "k_speculate",
                "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": traffic, "traffic_measured_at_commit": traffic_commit,
                "algo_bytes_per_launch": exp_bytes, "avg_launch_ms": exp_ms,
                "achievable": achievable_gbs, "frac_of_achievable": achieved / achievable_gbs}
    N = n_tokens + n_docs
    sc = prof_build["sort_scatter"]
    sc_ms = sc["ms"] / max(sc["launches"], 1)
    sc_ach = 24.0 * N / (sc_ms * 1e-3) / 1e9 if sc_ms > 0 else 0.0
    traffic_b, traffic_b_commit = _traffic_from_profiles("k_radix_scatter", w.name)
    roofline_build = {"bound": "hbm", "kernel": "k_radix_scatter", "achieved": sc_ach,
                      "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": sc_ach / HBM_PEAK_GBS,
                      "traffic": traffic_b, "traffic_measured_at_commit": traffic_b_commit,
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
        "value_is": "requests drafted for per second of whole decode steps (verifier stand-in, "
                    "acceptance, append, next drafts), all timed steps in one graph launch; "
                    "sd_speculate alone: speculate_only_trees_per_s; one launch per step: "
                    "ms_per_step_one_launch_per_step",
        "launch": head["launch"],
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
                            "the current drafts, acceptance, append, next drafts)"),
                   "slot_ids": "explicit array" if args.explicit_slot_ids else
                               "NULL (request b is slot b)"},
        "ms_per_step_one_launch_per_step": head["ms_per_step_one_launch_per_step"],
        "index_build_tokens_per_s": head["index_build_tokens_per_s"],
        "index_build_ms": head["index_build_ms"], "request_build_ms": head["request_build_ms"],
        "request_build_tokens_per_s": head["request_build_tokens_per_s"],
        "step_latency_ms": head["step_latency_ms"],
        "speculate_only_ms_median": spec_ms, "speculate_only_trees_per_s": B / (spec_ms * 1e-3),
        "speculate_latency_us_by_batch": latency_by_batch,
        "speculate_kernel_us_by_context_tokens": us_by_context,
        "speculate_latency_profile": latency_profile,
        "stream_copy_gbs": achievable_gbs, "dependent_load_ns_by_working_set": dep_ns,
        "mean_tree_nodes": mean_nodes, "mean_accept_len": mean_accept,
        "counters": head.get("counters"),
        "kernel_ms_per_launch": kernels_ms, "build_kernel_ms_total": build_kernels_ms,
        "roofline": roofline, "roofline_build": roofline_build,
        "index_bytes": head["index_bytes"], "scratch_bytes": head["scratch_bytes"],
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
    d_corpus, d_doc_off, d_future = run.d_corpus, run.d_doc_off, run.d_future
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
    run.close()

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
        by_batch["scratch_bytes_of_the_%d_slot_context" % nmax] = st3["scratch_bytes"]
        sd.sd_destroy(ctx3)
        out["speculate_throughput_by_batch"] = by_batch
        # the same kernel with the compute units full: its share of the roofline there (a
        # batch no configuration names: context, never the headline fraction)
        top_b = str(wide[-1])
        out["roofline"]["sd_speculate_at_batch_%s" % top_b] = {
            "achieved": by_batch[top_b]["achieved_gbs"], "frac": by_batch[top_b]["frac_of_peak"],
            "frac_of_achievable": by_batch[top_b]["frac_of_achievable"],
            "avg_launch_ms": by_batch[top_b]["us_per_launch"] * 1e-3,
            "algo_bytes_per_launch": by_batch[top_b]["algo_bytes_per_launch"]}
        del d_wctx, d_woff, d_wslots
    del run, d_corpus, d_doc_off, d_future, d_ctx, trees, d_slots, ctx2d, ev, step, reset, ctx
    torch.cuda.empty_cache()

    # ---- the other configurations: step time, per-step latency, build rates -----------------
    others = {}
    for name in [v.strip() for v in args.others.split(",") if v.strip()]:
        if name == args.workload or name not in CONFIGS:
            continue
        # the streaming configuration is defined as a run of 64 decode steps from the given
        # contexts: its latency figures are over those 64 steps, no warm-up steps before them
        Ko, Wo = (CONFIGS[name]["steps"], 0) if name == "streaming" else (K, W)
        r = Run(args, name, Ko + Wo)
        fig, _, _ = r.common_figures(Ko, Wo, args.build_reps)
        fig["config"] = {k: r.cfg[k] for k in ("vocab", "D", "P", "alpha", "min_score")}
        r.close()
        del r
        torch.cuda.empty_cache()
        others[name] = fig
    out["other_workloads"] = others

    if cpu_leg is not None:
        out["cpu_baseline"] = cpu_leg
    print(json.dumps(out))


if __name__ == "__main__":
    main()
