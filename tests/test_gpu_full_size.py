"""GPU parity at the benchmark configurations' full sizes, in the launch configuration
bench.py times (whole batch, full corpus): sd_speculate over the batch, sd_accept, then the
fused sd_accept_append_speculate step.  EVERY request of the batch is compared element by
element with the oracle (first drafts, acceptance, next drafts on the extended contexts); the
oracle runs in worker processes over chunks of requests, each with a global trie that holds
exactly the suffixes its chunk can reach.  The streaming workload runs all of its 64 decode
steps with two samples of requests followed by the oracle step by step.

Each test also says which routes of the kernel its batch took (counters of sd_get_stats): how
many trees came from the per-request index, how many requests had request-side suffix lists
of more than 64 occurrences, how the global matches were found.  The templated workloads
never take the long-list route on their own (a context's last token occurs once or twice in
it), so a few requests of the same batch get contexts with a planted repeated pair of tokens
and are run, in the same batch shape, against the oracle as well."""
import math

import numpy as np
import pytest

import oracle
from tests import oracle_jobs, parity
from workloads import make_workload

pytestmark = pytest.mark.gpu

JOB_TIMEOUT = 900
TREE_KEYS = ("n_nodes", "match_len", "source", "tokens", "parents", "scores", "tree_score")
COUNTERS = ("spec_requests", "spec_trees", "spec_from_request", "spec_global_list",
            "spec_global_search", "spec_request_wide", "spec_occ_in_memory", "spec_list_rounds")


def _check_properties(got, w):
    """Invariants of any valid result (Section 3 definitions + the size cap)."""
    n, ml = got["n_nodes"], got["match_len"]
    assert np.all(n <= np.floor(w.alpha * ml)) and np.all(n <= w.max_nodes) and np.all(n >= 0)
    assert np.all((n == 0) == (got["source"] == -1))
    idx = np.arange(w.max_nodes)[None, :]
    live = idx < n[:, None]
    assert np.all(got["tokens"][~live] == -1) and np.all(got["parents"][~live] == -1)
    assert np.all(got["scores"][~live] == 0.0)
    assert np.all(got["parents"][live] < np.broadcast_to(idx, live.shape)[live])
    assert np.all(got["parents"][live] >= -1)
    sc = got["scores"]
    assert np.all(sc[live] >= w.min_score) and np.all(sc[live] <= 1.0)
    # best-first on a monotone tree: scores never increase in insertion order
    assert np.all((sc[:, 1:] <= sc[:, :-1]) | ~live[:, 1:])
    for b in range(len(n)):
        k = int(n[b])
        assert float(np.cumsum(sc[b, :k])[-1] if k else 0.0) == pytest.approx(
            got["tree_score"][b], rel=1e-12)
        assert len({(int(got["parents"][b, j]), int(got["tokens"][b, j])) for j in range(k)}) == k
        d = parity.node_depths(got["parents"][b], k)
        assert k == 0 or d.max() <= w.D - ml[b]


def _planted(w, ids, n_plant=320):
    """Contexts of the workload that end with a pair of tokens the corpus is unlikely to hold,
    which also stands at n_plant earlier places of the context, each time followed by the same
    token, then by tokens that repeat with periods 2 and 4: the request-side lists of pattern
    lengths 1 and 2 hold hundreds of occurrences, with children of half and a quarter of them
    below, and the tree of pattern length 2 outscores what the global index has to offer."""
    out = {}
    for b in ids:
        x = w.contexts[b].copy()
        a = int((int(x[-2]) * 7919 + 13) % w.vocab)
        c = int((int(x[-1]) * 104729 + 7) % w.vocab)
        fill = x[7:7 + 8].copy()
        stride = max(8, (len(x) - 16) // (n_plant + 1))
        for i in range(n_plant):
            p = 16 + i * stride
            if p + 6 >= len(x) - 2:
                break
            x[p], x[p + 1] = a, c
            x[p + 2], x[p + 3], x[p + 4] = fill[0], fill[1 + i % 2], fill[3 + i % 4]
        x[-2], x[-1] = a, c
        out[int(b)] = x
    return out


def _gather(results, B, mn, step):
    """Chunk results of oracle_jobs.decode_steps -> arrays over the whole batch (rows of
    requests no job covered keep a marker that can match nothing)."""
    want = dict(n_nodes=np.full(B, -9, np.int32), tokens=np.full((B, mn), -9, np.int32),
                parents=np.full((B, mn), -9, np.int32), scores=np.full((B, mn), -9.0),
                tree_score=np.full(B, -9.0), match_len=np.full(B, -9, np.int32),
                source=np.full(B, -9, np.int32))
    acc = dict(accept_len=np.full(B, -9, np.int32), bonus=np.full(B, -9, np.int32), paths={})
    for r in results:
        ids = np.asarray(r["ids"])
        rec = r["steps"][step]
        for k in TREE_KEYS:
            want[k][ids] = rec["trees"][k]
        if "accept_len" in rec:
            acc["accept_len"][ids] = rec["accept_len"]
            acc["bonus"][ids] = rec["bonus"]
            for b, pth in zip(r["ids"], rec["paths"]):
                acc["paths"][b] = pth
    return want, acc


def _delta(st1, st0):
    return {k: int(st1[k] - st0[k]) for k in COUNTERS}


def _run_full(name, seed=0, chunk=32, cap=oracle_jobs.MAX_WORKERS, plant=()):
    w = make_workload(name, seed=seed)
    docs = w.docs()
    B, mn = w.batch, w.max_nodes
    contexts = [w.contexts[b] for b in range(B)]
    chunks = [range(i, min(i + chunk, B)) for i in range(0, B, chunk)]
    planted = _planted(w, plant)
    ex = oracle_jobs.pool(len(chunks) + 1, cap)
    g = None
    try:
        jobs = oracle_jobs.submit(ex, name, seed, chunks, 1, window=0)
        jobs_p = oracle_jobs.submit(ex, name, seed, [sorted(planted)], 1, overrides=planted,
                                    window=0) if planted else []
        g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, w.ctx_len + 4 * (mn + 1),
                           len(w.corpus) + len(docs))
        g.build_global(docs)
        g.build_requests(range(B), contexts)
        st0 = g.stats()
        got = g.speculate(range(B))
        st1 = g.stats()
        routes = _delta(st1, st0)
        assert routes["spec_requests"] == B
        assert st1["err_bad_token"] == 0 and st1["err_bad_slot"] == 0
        _check_properties(got, w)
        tgt = parity.targets_from_future(got, w.future, mn)
        al, ap, bo = g.accept(tgt)
        assert np.all(al <= got["n_nodes"])
        # the decode step as bench.py runs it: the same acceptance, the append and the next
        # drafts in one launch over the whole batch
        al2, ap2, bo2, nxt = g.accept_append_speculate(range(B), tgt)
        assert np.array_equal(al2, al) and np.array_equal(bo2, bo) and np.array_equal(ap2, ap)
        _check_properties(nxt, w)
        # ---- every request against the oracle ------------------------------------------
        results = [j.result(timeout=JOB_TIMEOUT) for j in jobs]
        want, acc = _gather(results, B, mn, 0)
        bad = parity.compare_trees(got, want, name)
        assert not bad, "\n".join(bad)
        assert np.array_equal(al, acc["accept_len"]) and np.array_equal(bo, acc["bonus"])
        for b in range(B):
            L = int(al[b])
            assert list(ap[b, :L]) == list(acc["paths"][b]) and np.all(ap[b, L:] == -1)
        want2, _ = _gather(results, B, mn, 1)
        bad = parity.compare_trees(nxt, want2, name + " next drafts")
        assert not bad, "\n".join(bad)
        routes["checked_requests"] = B
        routes["oracle_trees_from_request_index"] = int((want["source"] == 1).sum()) + \
            int((want2["source"] == 1).sum())
        assert routes["spec_from_request"] == int((want["source"] == 1).sum())
        # ---- the planted requests, in the same batch shape --------------------------------
        if planted:
            ids = sorted(planted)
            g.build_requests(ids, [planted[b] for b in ids])
            st0 = g.stats()
            got_p = g.speculate(range(B))
            rp = _delta(g.stats(), st0)
            rest = np.setdiff1d(np.arange(B), ids)
            for k in TREE_KEYS:     # the other requests: their next drafts once more
                assert np.array_equal(got_p[k][rest], nxt[k][rest]), k
            res_p = [j.result(timeout=JOB_TIMEOUT) for j in jobs_p]
            want_p, acc_p = _gather(res_p, B, mn, 0)
            bad = parity.compare_trees({k: got_p[k][ids] for k in TREE_KEYS},
                                       {k: want_p[k][ids] for k in TREE_KEYS}, name + " planted")
            assert not bad, "\n".join(bad)
            # (the other requests' targets are their first futures once more: any tokens do)
            tgt_p = parity.targets_from_future(got_p, w.future, mn)
            al_p, ap_p, bo_p, nxt_p = g.accept_append_speculate(range(B), tgt_p)
            assert np.array_equal(al_p[ids], acc_p["accept_len"][ids])
            assert np.array_equal(bo_p[ids], acc_p["bonus"][ids])
            want_p2, _ = _gather(res_p, B, mn, 1)
            bad = parity.compare_trees({k: nxt_p[k][ids] for k in TREE_KEYS},
                                       {k: want_p2[k][ids] for k in TREE_KEYS},
                                       name + " planted, next drafts")
            assert not bad, "\n".join(bad)
            _check_properties(nxt_p, w)
            routes["planted_requests"] = len(ids)
            routes["planted_request_wide"] = rp["spec_request_wide"]
            routes["planted_trees_from_request_index"] = int((want_p["source"][ids] == 1).sum())
            assert rp["spec_request_wide"] >= len(ids)
            assert routes["planted_trees_from_request_index"] >= 1
        st = g.stats()
        assert st["err_bad_token"] == 0 and st["err_bad_slot"] == 0 and st["err_ctx_overflow"] == 0
        print("\nroutes %s seed %d: %s" % (name, seed, routes))
        return got, want, routes
    finally:
        ex.shutdown(wait=True, cancel_futures=True)
        if g is not None:
            g.close()


def test_large_insert_then_speculate_sampled():
    """Headline corpus built from 95% of its documents, the rest inserted online in two batches
    (about 250k tokens each): sampled requests against the oracle trie over all documents."""
    w = make_workload("large", seed=0)
    docs = w.docs()
    B = w.batch
    contexts = [w.contexts[b] for b in range(B)]
    n0 = int(len(docs) * 0.95)
    n1 = n0 + (len(docs) - n0) // 2
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, w.ctx_len + 128,
                       len(w.corpus) + len(docs))
    try:
        g.build_global(docs[:n0])
        g.build_requests(range(B), contexts)
        g.insert_global(docs[n0:n1])
        g.insert_global(docs[n1:])
        got = g.speculate(range(B))
        st = g.stats()
        assert st["err_bad_token"] == 0 and st["err_bad_slot"] == 0
        _check_properties(got, w)
        rng = np.random.default_rng(4)
        pick = sorted(rng.choice(B, size=16, replace=False).tolist())
        sub = [contexts[b] for b in pick]
        tg = parity.oracle_global_trie(docs, w.D, w.vocab, sub, w.P)
        want = parity.oracle_speculate_batch(tg, sub, w.D, w.P, w.alpha, w.min_score, w.max_nodes)
        bad = parity.compare_trees({k: v[pick] for k, v in got.items()}, want, "large+insert")
        assert not bad, "\n".join(bad)
        # the entropy of the index at full size: its weight has a closed form (every position
        # weighs min(D, tokens left in its document)), and the index after the insertions must
        # give what a build over all documents gives
        h, wt = g.entropy()
        lens = np.array([len(d) for d in docs], np.int64)
        full = np.minimum(lens, w.D)                       # positions with fewer than D tokens left
        closed = int(np.sum(full * (full + 1) // 2 + (lens - full) * w.D))
        assert wt == float(closed)
        assert 0.0 < h < math.log2(w.vocab)
        g.build_global(docs)
        h2, wt2 = g.entropy()
        assert wt2 == wt and h2 == pytest.approx(h, rel=1e-9, abs=1e-12)
    finally:
        g.close()


def test_entropy_templated_mid_size_against_oracle():
    """The headline recipe at 200k tokens and the full depth bound (D = 64): long unary chains,
    runs of many suffixes at every depth, documents that end inside templates.  Tolerance as in
    the small entropy cases: summation order and log2 routines differ."""
    from workloads.synth import scaled
    w = make_workload(scaled("large", total=200_000, n_templates=60, batch=2, ctx=64), seed=5)
    docs = w.docs()
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, 1, 16, len(w.corpus) + len(docs) + 8)
    try:
        g.build_global(docs)
        h, wt = g.entropy()
    finally:
        g.close()
    t = oracle.Trie(w.D)
    for d in docs:
        t.add_doc(d)
    ho, wo = t.entropy()
    assert wt == wo
    assert h == pytest.approx(ho, rel=1e-9, abs=1e-12)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_agentic_full(seed):
    got, want, routes = _run_full("agentic", seed=seed, chunk=16, plant=(5, 40))
    assert (got["n_nodes"] > 0).mean() > 0.5
    assert routes["spec_global_list"] == 64


def test_large_full():
    """All 256 requests of the headline configuration."""
    got, want, routes = _run_full("large", chunk=32, plant=(1, 85, 128, 254))
    assert (got["n_nodes"] > 0).mean() > 0.5 and got["n_nodes"].max() > 32
    # on this corpus the last two tokens of a context start a handful of suffixes: the global
    # matches of every request come from that list
    assert routes["spec_global_list"] == 256 and routes["spec_global_search"] == 0


def test_lowrep_full():
    """All 256 requests of the low-repetition configuration: frequent last tokens (hundreds of
    occurrences in the context, first-token buckets of up to a million suffixes) take every
    route the templated workloads do not.  Eight tries of about 150 million nodes each."""
    got, want, routes = _run_full("lowrep", chunk=32, cap=8)
    assert (got["n_nodes"] > 0).mean() > 0.3
    assert routes["spec_global_search"] >= 32 and routes["spec_global_list"] >= 32
    assert routes["spec_request_wide"] >= 32
    assert routes["oracle_trees_from_request_index"] >= 1


def test_streaming_all_decode_steps():
    """100M-token corpus, 512 requests, all 64 decode steps with the simulated verifier:
    speculate, accept, append.  Two samples of eight requests (two of them with planted
    repeats) are followed by the oracle through every step (global trie restricted to the
    suffixes a sample can reach, extended as the contexts grow; per-request tries extended
    online); invariants are checked for the whole batch at every step, and every request's
    appended tokens must be its ground-truth future."""
    w = make_workload("streaming", seed=0)
    docs = w.docs()
    B, mn, steps = w.batch, w.max_nodes, w.steps
    assert steps == 64
    contexts = [w.contexts[b].copy() for b in range(B)]
    samples = [sorted(np.random.default_rng(s).choice(B, size=8, replace=False).tolist())
               for s in (2, 5)]
    assert not set(samples[0]) & set(samples[1])
    planted = _planted(w, [samples[0][3], samples[1][6]])
    for b, x in planted.items():
        contexts[b] = x
    pick = sorted(samples[0] + samples[1])
    ex = oracle_jobs.pool(2)
    g = None
    try:
        jobs = oracle_jobs.submit(ex, "streaming", 0, samples, steps, overrides=planted, window=96)
        g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, w.ctx_len + steps * (mn + 1),
                           len(w.corpus) + len(docs))
        g.build_global(docs)
        g.build_requests(range(B), contexts)
        st0 = g.stats()
        pos = np.zeros(B, np.int64)
        accepted = 0
        got_next = None
        seen = []        # per step: the sampled requests' trees and acceptance
        for step in range(steps):
            got = got_next if got_next is not None else g.speculate(range(B))
            got_next = None
            _check_properties(got, w)
            fut = np.stack([w.future[b, pos[b]:pos[b] + mn + 2] for b in range(B)])
            tgt = parity.targets_from_future(got, fut, mn)
            # the three ways to end a step take turns: separate accept and append; both in one
            # launch; and, as bench.py's step does, both plus the next step's drafts in one launch
            mode = step % 3
            if mode == 2:
                al, ap, bo, got_next = g.accept_append_speculate(range(B), tgt)
            else:
                al, ap, bo = g.accept_append(range(B), tgt) if mode == 1 else g.accept(tgt)
            new = []
            for b in range(B):
                L = int(al[b])
                toks = [int(got["tokens"][b, j]) for j in ap[b, :L]] + [int(bo[b])]
                assert toks == [int(v) for v in w.future[b, pos[b]:pos[b] + L + 1]]
                new.append(np.array(toks, np.int32))
                pos[b] += L + 1
                accepted += L
            if mode == 0:
                g.append(range(B), new)
            seen.append(dict(trees={k: got[k][pick].copy() for k in TREE_KEYS},
                             accept_len=al[pick].copy(), bonus=bo[pick].copy(),
                             paths=[ap[b, :int(al[b])].copy() for b in pick]))
        last = got_next if got_next is not None else g.speculate(range(B))
        seen.append(dict(trees={k: last[k][pick].copy() for k in TREE_KEYS}))
        routes = _delta(g.stats(), st0)
        assert accepted > B          # the drafts do get accepted on this workload
        assert g.stats()["err_ctx_overflow"] == 0
        # ---- the sampled requests against the oracle, step by step ----------------------------
        results = [j.result(timeout=JOB_TIMEOUT) for j in jobs]
        row = {b: i for i, b in enumerate(pick)}
        from_request = 0
        for r in results:
            rows = [row[b] for b in r["ids"]]
            for step in range(steps + 1):
                rec, mine = r["steps"][step], seen[step]
                bad = parity.compare_trees({k: mine["trees"][k][rows] for k in TREE_KEYS},
                                           rec["trees"], "streaming step %d" % step)
                assert not bad, "\n".join(bad)
                from_request += int((rec["trees"]["source"] == 1).sum())
                if step < steps:
                    assert np.array_equal(mine["accept_len"][rows], rec["accept_len"]), step
                    assert np.array_equal(mine["bonus"][rows], rec["bonus"]), step
                    for i, pth in zip(rows, rec["paths"]):
                        assert list(mine["paths"][i]) == list(pth), step
        routes["checked_requests_x_steps"] = "%d x %d" % (len(pick), steps + 1)
        routes["oracle_trees_from_request_index"] = from_request
        print("\nroutes streaming: %s" % routes)
        assert routes["spec_request_wide"] >= len(planted) and from_request >= 1
    finally:
        ex.shutdown(wait=True, cancel_futures=True)
        if g is not None:
            g.close()
