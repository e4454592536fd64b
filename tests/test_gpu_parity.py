"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Structure (parents, tokens, sizes, match length, source, acceptance) must be
bit-exact; fp64 scores within 1e-12 relative."""
import numpy as np
import pytest

import oracle
from tests import parity
from workloads import make_workload, scaled

pytestmark = pytest.mark.gpu


def sd_read_global(g):
    import paper_2411_04975_amd as sd
    return sd.sd_debug_read_global(g.ctx)


def _run_workload(w, check_accept=True, slots=None):
    docs = w.docs()
    contexts = [w.contexts[b] for b in range(w.batch)]
    slots = list(range(w.batch)) if slots is None else slots
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, max(slots) + 1,
                       w.ctx_len + 4 * (w.max_nodes + 1), len(w.corpus) + len(docs))
    try:
        g.build_global(docs)
        g.build_requests(slots, contexts)
        got = g.speculate(slots)
        tg = parity.oracle_global_trie(docs, w.D, w.vocab, contexts, w.P)
        want = parity.oracle_speculate_batch(tg, contexts, w.D, w.P, w.alpha, w.min_score,
                                             w.max_nodes)
        bad = parity.compare_trees(got, want, w.name)
        assert not bad, "\n".join(bad)
        st = g.stats()
        assert st["err_bad_token"] == 0 and st["err_bad_slot"] == 0 and st["err_ctx_overflow"] == 0
        if check_accept:
            tgt = parity.targets_from_future(want, w.future, w.max_nodes)
            al, ap, bo = g.accept(tgt)
            for b in range(w.batch):
                n = int(want["n_nodes"][b])
                L, path, bonus = oracle.accept(want["tokens"][b, :n], want["parents"][b, :n],
                                               tgt[b])
                assert al[b] == L and bo[b] == bonus, (b, al[b], L)
                assert list(ap[b, :L]) == list(path) and np.all(ap[b, L:] == -1)
        return got, want
    finally:
        g.close()


@pytest.mark.parametrize("size", ["5-sort-tiles", "11-sort-tiles"])
def test_global_index_is_a_sorted_suffix_array(size, tiny_workload):
    w = tiny_workload if size == "5-sort-tiles" else make_workload(scaled("tiny", n_docs=90), seed=2)
    import paper_2411_04975_amd as sd
    docs = w.docs()
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, 4, 64, len(w.corpus) + len(docs))
    try:
        g.build_global(docs)
        text, sa = sd.sd_debug_read_global(g.ctx)
    finally:
        g.close()
    N = len(w.corpus) + len(docs)
    assert len(sa) == N and np.array_equal(np.sort(sa), np.arange(N))
    # the text is the documents back to back with -1 after each
    want_text = np.concatenate([np.concatenate([d, [-1]]) for d in docs]).astype(np.int32)
    assert np.array_equal(text, want_text)
    # D-truncated, end-marker-terminated keys are non-decreasing along the suffix array
    pad = np.concatenate([text, np.full(w.D, -1, np.int32)])
    keys = np.stack([pad[sa + k] for k in range(w.D)], axis=1).astype(np.int64)
    ended = np.cumsum(keys == -1, axis=1) > 0        # everything after the first marker ...
    keys[ended] = -1                                 # ... does not take part in the comparison
    a, b = keys[:-1], keys[1:]
    diff = a != b
    first = diff.argmax(axis=1)
    rows = np.arange(N - 1)
    ok = ~diff.any(axis=1) | (a[rows, first] < b[rows, first])
    assert ok.all(), "suffix array out of order at %s" % np.nonzero(~ok)[0][:5]
    # interval widths equal oracle counts for sampled paths
    t = oracle.Trie(w.D)
    for d in docs:
        t.add_doc(d)
    rng = np.random.default_rng(3)
    for _ in range(300):
        i = int(rng.integers(0, len(w.corpus)))
        k = int(rng.integers(1, w.D + 1))
        path = w.corpus[i:i + k]
        m = np.ones(N, bool)
        for q, tok in enumerate(path):
            m &= keys[:, q] == tok
        idx = np.nonzero(m)[0]
        assert len(idx) == t.lookup(path)[0]
        if len(idx):
            assert idx[-1] - idx[0] + 1 == len(idx)       # contiguous range


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tiny_parity(seed):
    w = make_workload("tiny", seed=seed)
    got, want = _run_workload(w)
    assert (want["n_nodes"] > 0).sum() >= w.batch // 2


def test_agentic_scaled_parity():
    w = make_workload(scaled("agentic", n_docs=300, batch=32, ctx=2048), seed=0, name="agentic-s")
    got, want = _run_workload(w)
    assert (want["n_nodes"] > 0).sum() >= w.batch // 2
    # (which index the winners came from is asserted at full size, through the library's own
    # counters: tests/test_gpu_full_size.py)


def test_large_scaled_parity():
    w = make_workload(scaled("large", n_templates=300, total=400_000, batch=48, ctx=3000), seed=0,
                      name="large-s")
    got, want = _run_workload(w)
    assert want["n_nodes"].max() > 32


def test_lowrep_scaled_parity():
    w = make_workload(scaled("lowrep", n_docs=150, batch=64, ctx=4096), seed=0, name="lowrep-s")
    got, want = _run_workload(w)


def test_non_identity_slots_and_partial_batch(tiny_workload):
    w = tiny_workload
    slots = [(3 * b + 1) % 40 for b in range(w.batch)]
    assert len(set(slots)) == w.batch
    _run_workload(w, slots=slots)



def test_null_slot_ids_mean_the_identity(tiny_workload):
    """Every call that takes slot ids accepts NULL for "request i is slot i": builds, appends,
    drafts and fused steps made that way give what the same calls with the ids 0, 1, 2, ...
    give."""
    import torch
    import paper_2411_04975_amd as sd
    w = tiny_workload
    docs = w.docs()
    B, mn = w.batch, w.max_nodes
    contexts = [w.contexts[b] for b in range(B)]
    rng = np.random.default_rng(17)
    results = []
    for explicit in (True, False):
        g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, w.ctx_len + 4 * (mn + 1),
                           len(w.corpus) + len(docs))
        try:
            ids = torch.arange(B, dtype=torch.int32, device=g.dev) if explicit else None
            g.build_global(docs)
            d_tok, d_off, n = g._seqs(contexts)
            sd.sd_index_build(g.ctx, sd.SD_SCOPE_REQUESTS, ids, d_tok, d_off, n)
            new = [w.future[b, :1 + b % 3] for b in range(B)]
            d_new, d_noff, _ = g._seqs(new)
            sd.sd_index_append(g.ctx, ids, d_new, d_noff.to(torch.int32))
            tr = g._trees(B, mn)
            sd.sd_speculate(g.ctx, ids, tr)
            torch.cuda.synchronize()
            first = {k: getattr(tr, k).cpu().numpy().copy() for k in ("n_nodes", "tokens", "parents", "scores")}
            tgt = parity.targets_from_future(first, w.future[:, 3:], mn)
            d_t = torch.from_numpy(tgt).to(g.dev)
            al, ap, bo = g._accept_outputs(B, mn)
            sd.sd_accept_append_speculate(g.ctx, tr, ids, d_t, al, ap, bo)
            torch.cuda.synchronize()
            g.check_guards()
            al2, ap2, bo2 = g._accept_outputs(B, mn)
            sd.sd_accept_append(g.ctx, tr, ids, d_t, al2, ap2, bo2)
            torch.cuda.synchronize()
            g.check_guards()
            tr3 = g._trees(B, mn)
            sd.sd_speculate_static(g.ctx, ids, tr3)
            torch.cuda.synchronize()
            st = g.stats()
            assert st["err_bad_slot"] == 0 and st["err_bad_token"] == 0 and st["err_ctx_overflow"] == 0
            results.append([first["n_nodes"], first["tokens"], first["parents"], first["scores"],
                            al.cpu().numpy(), bo.cpu().numpy(), tr.tokens.cpu().numpy(),
                            tr.n_nodes.cpu().numpy(), al2.cpu().numpy(), tr3.tokens.cpu().numpy(),
                            tr3.parents.cpu().numpy(), tr3.scores.cpu().numpy()])
        finally:
            g.close()
    for a_, b_ in zip(*results):
        assert np.array_equal(a_, b_)
    assert results[0][0].sum() > 0 and results[0][7].sum() > 0


def _more_minis():
    """Cases aimed at the chain merge (token ties, more chains than one call merges, chains
    longer than one window), at the depth bound inside runs of equal counts, and at the
    largest tree size."""
    out = []
    # three symbols, deep bound, big trees: long single-occurrence chains full of token ties
    rng = np.random.default_rng(21)
    doc = list(rng.integers(0, 3, 700))
    ctxs = [doc[a:a + ln] for a, ln in ((100, 40), (333, 25), (10, 12), (600, 9), (250, 60))]
    out.append(("ties-deep-window", 3, 200, 8, 8.0, 0.01, [doc, doc[50:400]], ctxs))
    # one pattern followed by many different one-off continuations (10 and 14 tied chains)
    docs = []
    for fan in (10, 14):
        for i in range(fan):
            docs.append([7, 8, 50 + fan] + [1000 * fan + 40 * i + k for k in range(30)])
    out.append(("many-tied-chains", 20000, 40, 4, 8.0, 0.01, docs,
                [[3, 7, 8, 60], [5, 7, 8, 64], [7, 8, 60, 10000], [8, 64]]))
    # periodic text: every pattern length has the same chain below it and the depth bound cuts it
    per = [4, 9, 2, 7, 5]
    out.append(("periodic-depth-bound", 16, 14, 8, 3.0, 0.05, [per * 30, per * 3 + [1, 2, 3]],
                [per * 4, (per * 4)[:-2], per * 2 + [4, 9], [9, 2, 7]]))
    # forty tied chains: the step-by-step merge works in bursts of six nodes between refills of
    # its token windows
    docs = [[7, 8, 90] + [2000 + 37 * i + k for k in range(10)] for i in range(40)]
    out.append(("forty-tied-chains", 20000, 40, 4, 8.0, 0.01, docs,
                [[1, 7, 8, 90], [8, 90], [90]]))
    # a wide node with three hundred children of one or two occurrences each: every probe of a
    # group opens a run of its own; and the same with eight occurrences per child (several
    # groups of probes, a handful of runs in each)
    docs = [[5, 1000 + i, 7, i % 3] for i in range(300)] + [[5, 1000 + i, 9] for i in range(0, 300, 7)]
    out.append(("fan-out-singles", 20000, 12, 3, 8.0, 0.001, docs, [[5], [2, 5], [7, 1]]))
    docs = [[6, 500 + i % 100, i % 5, i % 2] for i in range(800)]
    out.append(("fan-out-eights", 20000, 12, 3, 8.0, 0.001, docs, [[6], [3, 6], [6, 510]]))
    # largest tree size the library accepts
    rng = np.random.default_rng(22)
    doc = list(rng.integers(0, 4, 3000))
    ctxs = [doc[a:a + ln] for a, ln in ((500, 300), (1200, 80), (2500, 150), (40, 70))]
    out.append(("largest-trees", 4, 255, 64, 4.0, 0.001, [doc], ctxs))
    return out


MINIS = [
    # vocab, D, P, alpha, min_score, docs, contexts
    ("all-equal", 2, 6, 3, 2.0, 0.05, [[1] * 50], [[1] * 20, [1], [0, 1, 1]]),
    ("single-token-docs", 3, 4, 2, 2.0, 0.1, [[0], [1], [1], [2]], [[1], [2, 1], [0, 0, 0]]),
    ("ctx-shorter-than-P", 4, 10, 8, 1.0, 0.1, [[0, 1, 2, 3] * 10], [[2, 3], [3], [0, 1, 2]]),
    ("empty-context", 4, 5, 3, 1.0, 0.1, [[0, 1, 2, 3, 0, 1, 2]], [[], [0, 1], []]),
    ("min-score-zero", 3, 8, 4, 4.0, 0.0, [[0, 1, 2, 0, 1, 1, 0, 2, 2, 1, 0, 1] * 4],
     [[2, 0, 1], [1, 1, 0], [0]]),
    ("min-score-one", 3, 8, 4, 4.0, 1.0, [[0, 1, 2, 0, 1, 2, 0, 1, 2]], [[0, 1], [2, 0, 1, 2]]),
    ("binary-wide", 2, 12, 6, 4.0, 0.02,
     [list(np.random.default_rng(11).integers(0, 2, 400))], None),
    ("alpha-below-one", 5, 9, 6, 0.5, 0.1, [[0, 1, 2, 3, 4] * 12], [[3, 4, 0, 1, 2, 3]]),
] + _more_minis()


@pytest.mark.parametrize("name,vocab,D,P,alpha,ms,docs,contexts", MINIS,
                         ids=[m[0] for m in MINIS])
def test_adversarial_minis(name, vocab, D, P, alpha, ms, docs, contexts):
    rng = np.random.default_rng(5)
    if contexts is None:
        contexts = [list(rng.integers(0, vocab, int(rng.integers(1, 300)))) for _ in range(12)]
    docs = [np.asarray(d, np.int32) for d in docs]
    contexts = [np.asarray(c, np.int32) for c in contexts]
    B = len(contexts)
    g = parity.GpuPath(vocab, D, P, alpha, ms, B, 512, sum(len(d) for d in docs) + len(docs))
    try:
        g.build_global(docs)
        g.build_requests(range(B), contexts)
        got = g.speculate(range(B))
        tg = parity.oracle_global_trie(docs, D, vocab)
        want = parity.oracle_speculate_batch(tg, contexts, D, P, alpha, ms, g.max_nodes)
        bad = parity.compare_trees(got, want, name)
        assert not bad, "\n".join(bad)
    finally:
        g.close()


def test_empty_global_index_and_unbuilt_slots():
    g = parity.GpuPath(100, 8, 4, 2.0, 0.1, 4, 64, 100)
    try:
        # nothing built at all: every slot is an empty context
        got = g.speculate([0, 1])
        assert np.all(got["n_nodes"] == 0) and np.all(got["source"] == -1)
        assert np.all(got["tokens"] == -1) and np.all(got["scores"] == 0)
        g.build_global([])
        ctxs = [np.array([5, 6, 7, 5, 6], np.int32)]
        g.build_requests([2], ctxs)
        got = g.speculate([2, 3])
        want = parity.oracle_speculate_batch(None, [ctxs[0], np.zeros(0, np.int32)], 8, 4, 2.0, 0.1,
                                             g.max_nodes)
        assert not parity.compare_trees(got, want)
        assert got["source"][0] == 1 and got["n_nodes"][0] > 0
    finally:
        g.close()


def test_append_equals_rebuild_and_streaming_loop():
    """Decode loop with the simulated verifier: speculate, accept, append accepted + bonus
    tokens; each step is compared with the oracle whose per-request tries are extended online."""
    w = make_workload(scaled("tiny", batch=12, steps=6), seed=4)
    docs = w.docs()
    B, mn = w.batch, w.max_nodes
    contexts = [w.contexts[b].copy() for b in range(B)]
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, w.ctx_len + 6 * (mn + 1),
                       len(w.corpus) + len(docs))
    try:
        g.build_global(docs)
        g.build_requests(range(B), contexts)
        tg = parity.oracle_global_trie(docs, w.D, w.vocab)
        tries = []
        for x in contexts:
            t = oracle.Trie(w.D)
            t.append(x)
            tries.append(t)
        pos = np.zeros(B, np.int64)
        total_acc = 0
        for step in range(6):
            got = g.speculate(range(B))
            want = parity.oracle_speculate_batch(tg, contexts, w.D, w.P, w.alpha, w.min_score, mn,
                                                 request_tries=tries)
            bad = parity.compare_trees(got, want, "step %d" % step)
            assert not bad, "\n".join(bad)
            fut = np.stack([w.future[b, pos[b]:pos[b] + mn + 2] for b in range(B)])
            tgt = parity.targets_from_future(want, fut, mn)
            # odd steps end with the fused call (accept + append in one launch), even steps
            # with the two separate calls: the contexts must come out the same either way
            fused = step % 2 == 1
            al, ap, bo = g.accept_append(range(B), tgt) if fused else g.accept(tgt)
            new = []
            for b in range(B):
                n = int(want["n_nodes"][b])
                L, path, bonus = oracle.accept(want["tokens"][b, :n], want["parents"][b, :n], tgt[b])
                assert al[b] == L and bo[b] == bonus and list(ap[b, :L]) == list(path)
                toks = [int(want["tokens"][b, j]) for j in path] + [int(bonus)]
                assert toks == [int(v) for v in w.future[b, pos[b]:pos[b] + L + 1]]
                new.append(np.array(toks, np.int32))
                tries[b].append(new[-1])
                contexts[b] = np.concatenate([contexts[b], new[-1]])
                pos[b] += L + 1
                total_acc += L
            if not fused:
                g.append(range(B), new)
        assert total_acc > 0
        # a context rebuilt from scratch gives the same trees as the appended one
        got_app = g.speculate(range(B))
        g.build_requests(range(B), contexts)
        got_reb = g.speculate(range(B))
        assert not parity.compare_trees(got_app, got_reb, "append vs rebuild")
        st = g.stats()
        assert st["err_ctx_overflow"] == 0
    finally:
        g.close()


def test_fused_step_end_and_next_draft_in_one_launch():
    """Decode loop in which every step ends with sd_accept_append_speculate: the acceptance, the
    appended context and the next trees must be those of the oracle, step after step; and a full
    context makes the fused call raise the overflow flag and draft from the unchanged context."""
    w = make_workload(scaled("tiny", batch=12, steps=6), seed=9)
    docs = w.docs()
    B, mn = w.batch, w.max_nodes
    contexts = [w.contexts[b].copy() for b in range(B)]
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, w.ctx_len + 6 * (mn + 1),
                       len(w.corpus) + len(docs))
    try:
        g.build_global(docs)
        g.build_requests(range(B), contexts)
        tg = parity.oracle_global_trie(docs, w.D, w.vocab)
        tries = []
        for x in contexts:
            t = oracle.Trie(w.D)
            t.append(x)
            tries.append(t)
        pos = np.zeros(B, np.int64)
        got = g.speculate(range(B))
        total_acc = 0
        for step in range(6):
            want = parity.oracle_speculate_batch(tg, contexts, w.D, w.P, w.alpha, w.min_score, mn,
                                                 request_tries=tries)
            bad = parity.compare_trees(got, want, "step %d" % step)
            assert not bad, "\n".join(bad)
            fut = np.stack([w.future[b, pos[b]:pos[b] + mn + 2] for b in range(B)])
            tgt = parity.targets_from_future(want, fut, mn)
            al, ap, bo, got = g.accept_append_speculate(range(B), tgt)
            for b in range(B):
                n = int(want["n_nodes"][b])
                L, path, bonus = oracle.accept(want["tokens"][b, :n], want["parents"][b, :n], tgt[b])
                assert al[b] == L and bo[b] == bonus and list(ap[b, :L]) == list(path)
                assert list(ap[b, L:]) == [-1] * (mn - L)
                new = np.array([int(want["tokens"][b, j]) for j in path] + [int(bonus)], np.int32)
                tries[b].append(new)
                contexts[b] = np.concatenate([contexts[b], new])
                pos[b] += L + 1
                total_acc += L
        assert total_acc > 0
        want = parity.oracle_speculate_batch(tg, contexts, w.D, w.P, w.alpha, w.min_score, mn,
                                             request_tries=tries)
        assert not parity.compare_trees(got, want, "after the last step")
        # the separate calls see the same contexts
        assert not parity.compare_trees(g.speculate(range(B)), want, "separate speculate")
        assert g.stats()["err_ctx_overflow"] == 0
    finally:
        g.close()
    g = parity.GpuPath(10, 6, 3, 1.0, 0.1, 2, 16, 100)
    try:
        g.build_global([np.array([1, 2, 3, 0, 4], np.int32)])
        g.build_requests([1], [np.arange(16, dtype=np.int32) % 10])     # slot 1 is full
        g.speculate([1])
        tgt = np.zeros((1, g.max_nodes + 1), np.int32)
        al, ap, bo, got = g.accept_append_speculate([1], tgt)
        assert g.stats()["err_ctx_overflow"] == 1 and bo[0] == 0
        want = parity.oracle_speculate_batch(
            parity.oracle_global_trie([np.array([1, 2, 3, 0, 4], np.int32)], 6, 10),
            [np.arange(16, dtype=np.int32) % 10], 6, 3, 1.0, 0.1, g.max_nodes)
        assert not parity.compare_trees(got, want)
        # a bad slot id: flag raised, empty draft
        g.speculate([1])
        al, ap, bo, got = g.accept_append_speculate([7], tgt)
        assert g.stats()["err_bad_slot"] == 1 and got["n_nodes"][0] == 0
    finally:
        g.close()


@pytest.mark.parametrize("mn", [256, 64, 16])
def test_accept_on_synthetic_trees(mn):
    """sd_accept against the oracle's walk on trees that sd_speculate would not produce by
    itself: chains of every length up to the largest tree, bushy random trees, targets that
    stop the walk anywhere, empty trees; for trees of up to 256 nodes (pointer jumping in LDS)
    and of up to 64 and 16 (one node per lane, in registers; a chain of 64 accepted to the
    end takes its bonus token from target position 64)."""
    import torch
    import paper_2411_04975_amd as sd
    rng = np.random.default_rng(17 + mn)
    cases = []
    for L in (0, 1, 2, 7, 8, 9, 10, 15, 16, 63, 64, 65, 200, 256):  # a chain accepted up to node L
        if L > mn:
            continue
        n = mn
        tok = rng.integers(0, 50, n).astype(np.int32)
        par = np.arange(-1, n - 1, dtype=np.int32)
        tgt = np.empty(n + 1, np.int32)
        tgt[:n] = tok                                               # target at node j-1 = token of j
        tgt[n] = 3
        if L < n:
            tgt[L] = tok[L] + 1                                     # node L is refused
        cases.append((n, tok, par, tgt))
    for _ in range(40):                                             # random trees, distinct siblings
        n = int(rng.integers(0, mn + 1))
        par = np.array([int(rng.integers(-1, j)) for j in range(n)], np.int32)
        tok = np.zeros(n, np.int32)
        seen = {}
        for j in range(n):
            k = seen.get(int(par[j]), 0)
            seen[int(par[j])] = k + 1
            tok[j] = 100 * k + int(rng.integers(0, 100))            # distinct among siblings
        tgt = rng.integers(0, 300, mn + 1).astype(np.int32)
        v = -1                                                      # lay a path of random length
        for _ in range(int(rng.integers(0, 40))):
            kids = [j for j in range(n) if par[j] == v]
            if not kids:
                break
            j = kids[int(rng.integers(0, len(kids)))]
            tgt[v + 1] = tok[j]
            v = j
        cases.append((n, tok, par, tgt))
    B = len(cases)
    dev = torch.device("cuda", 0)
    ctx = sd.sd_create(1000, 8, 4, mn / 4.0, 0.1, B, 16, 16, 0)    # floor(alpha P) = mn
    try:
        tr = sd.Trees(B, mn, dev)
        toks = np.full((B, mn), -1, np.int32)
        pars = np.full((B, mn), -1, np.int32)
        tgts = np.zeros((B, mn + 1), np.int32)
        nn = np.zeros(B, np.int32)
        for b, (n, tok, par, tgt) in enumerate(cases):
            toks[b, :n] = tok; pars[b, :n] = par; nn[b] = n
            tgts[b, :len(tgt)] = tgt
        tr.tokens.copy_(torch.from_numpy(toks)); tr.parents.copy_(torch.from_numpy(pars))
        tr.n_nodes.copy_(torch.from_numpy(nn))
        al = torch.full((B,), -7, dtype=torch.int32, device=dev)
        ap = torch.full((B, mn), -7, dtype=torch.int32, device=dev)
        bo = torch.full((B,), -7, dtype=torch.int32, device=dev)
        sd.sd_accept(ctx, tr, B, torch.from_numpy(tgts).to(dev), al, ap, bo)
        torch.cuda.synchronize()
        al, ap, bo = al.cpu().numpy(), ap.cpu().numpy(), bo.cpu().numpy()
        for b, (n, tok, par, tgt) in enumerate(cases):
            L, path, bonus = oracle.accept(tok, par, tgts[b])
            assert al[b] == L and bo[b] == bonus, (b, n, al[b], L)
            assert list(ap[b, :L]) == list(path) and list(ap[b, L:]) == [-1] * (mn - L)
    finally:
        sd.sd_destroy(ctx)


def test_verifier_stand_in_matches_its_definition():
    """The simulated target model of the serving-loop glue (the token after a draft node of
    depth k is the k-th ground-truth token) against the plain numpy statement of the same
    thing, on chains, bushy trees and empty trees, with and without moving the positions on."""
    import torch
    from workloads import verifier
    rng = np.random.default_rng(23)
    B, mn, flen = 40, 256, 700
    dev = torch.device("cuda", 0)
    pars = np.full((B, mn), -1, np.int32)
    nn = np.zeros(B, np.int32)
    for b in range(B):
        n = int(rng.integers(0, mn + 1)) if b % 4 else (0 if b == 0 else mn)
        nn[b] = n
        if b % 3 == 0:
            pars[b, :n] = np.arange(-1, n - 1)                         # one long chain
        else:
            pars[b, :n] = [int(rng.integers(-1, j)) for j in range(n)]
    future = rng.integers(0, 1000, (B, flen)).astype(np.int32)
    pos = rng.integers(0, 100, B).astype(np.int32)
    adv = rng.integers(-1, 20, B).astype(np.int32)
    for use_adv in (False, True):
        d_pos = torch.from_numpy(pos.copy()).to(dev)
        d_tgt = torch.full((B, mn + 1), -7, dtype=torch.int32, device=dev)
        verifier.targets(torch.from_numpy(nn).to(dev), torch.from_numpy(pars).to(dev),
                         torch.from_numpy(future).to(dev), d_pos, d_tgt,
                         advance=torch.from_numpy(adv).to(dev) if use_adv else None)
        torch.cuda.synchronize()
        p0 = pos + (adv + 1 if use_adv else 0)
        assert np.array_equal(d_pos.cpu().numpy(), p0)
        want = parity.targets_from_future({"n_nodes": nn, "parents": pars},
                                          np.stack([future[b, p0[b]:p0[b] + mn + 2] for b in range(B)]),
                                          mn)
        assert np.array_equal(d_tgt.cpu().numpy(), want)


def test_device_flags_bad_token_slot_and_overflow():
    g = parity.GpuPath(10, 6, 3, 1.0, 0.1, 2, 16, 100)
    try:
        g.build_global([np.array([1, 2, 3, 11, 4], np.int32)])          # token 11 >= vocab
        assert g.stats()["err_bad_token"] == 1
        g.build_requests([5], [np.array([1, 2], np.int32)])             # slot 5 out of range
        assert g.stats()["err_bad_slot"] == 1
        g.build_requests([0], [np.arange(8, dtype=np.int32) % 10])
        g.append([0], [np.arange(9, dtype=np.int32) % 10])              # 8 + 9 > 16
        assert g.stats()["err_ctx_overflow"] == 1
        got = g.speculate([0])                                          # context unchanged
        want = parity.oracle_speculate_batch(
            parity.oracle_global_trie([np.array([1, 2, 3, 0, 4], np.int32)], 6, 10),
            [np.arange(8, dtype=np.int32) % 10], 6, 3, 1.0, 0.1, g.max_nodes)
        assert not parity.compare_trees(got, want)
        # the fused accept + append raises the same flags and leaves the context alone
        g.build_requests([1], [np.arange(16, dtype=np.int32) % 10])     # slot 1 is full
        g.speculate([1])
        tgt = np.zeros((1, g.max_nodes + 1), np.int32)
        al, ap, bo = g.accept_append([1], tgt)
        assert g.stats()["err_ctx_overflow"] == 1 and bo[0] == 0
        got = g.speculate([1])
        want = parity.oracle_speculate_batch(
            parity.oracle_global_trie([np.array([1, 2, 3, 0, 4], np.int32)], 6, 10),
            [np.arange(16, dtype=np.int32) % 10], 6, 3, 1.0, 0.1, g.max_nodes)
        assert not parity.compare_trees(got, want)
    finally:
        g.close()


def test_decode_step_in_a_hip_graph_matches_eager():
    """A decode step (speculate, verifier glue, accept, append) captured into a HIP graph and
    replayed several times, with eager work and synchronisations in between, must give the
    results of the same steps enqueued eagerly on a second context."""
    import torch
    import paper_2411_04975_amd as sd
    from workloads import verifier
    w = make_workload(scaled("tiny", batch=16), seed=3)
    dev = torch.device("cuda", 0)
    i32 = torch.int32
    B, mn, steps = w.batch, w.max_nodes, 5
    docs_tok = torch.from_numpy(w.corpus).to(dev)
    docs_off = torch.from_numpy(w.doc_offsets).to(dev)
    ctx_tok = torch.from_numpy(w.contexts.reshape(-1)).to(dev)
    ctx_off = torch.arange(0, (B + 1) * w.ctx_len, w.ctx_len, dtype=torch.int64, device=dev)
    future = torch.from_numpy(w.future).to(dev)
    slots = torch.arange(B, dtype=i32, device=dev)

    class Loop:
        def __init__(self, fused=False, one_launch=False):
            self.ctx = sd.sd_create(w.vocab, w.D, w.P, w.alpha, w.min_score, B,
                                    w.ctx_len + (steps + 3) * (mn + 1), len(w.corpus) + 64, 0)
            sd.sd_index_build(self.ctx, sd.SD_SCOPE_GLOBAL, None, docs_tok, docs_off, len(w.corpus))
            sd.sd_index_build(self.ctx, sd.SD_SCOPE_REQUESTS, slots, ctx_tok, ctx_off,
                              B * w.ctx_len)
            self.trees = sd.Trees(B, mn, dev)
            self.target = torch.zeros((B, mn + 1), dtype=i32, device=dev)
            self.alen = torch.zeros(B, dtype=i32, device=dev)
            self.apath = torch.zeros((B, mn), dtype=i32, device=dev)
            self.bonus = torch.zeros(B, dtype=i32, device=dev)
            self.new = torch.zeros(B * (mn + 1), dtype=i32, device=dev)
            self.newoff = torch.zeros(B + 1, dtype=i32, device=dev)
            self.pos = torch.zeros(B, dtype=i32, device=dev)
            self.fused = fused
            self.one_launch = one_launch
            if fused or one_launch:
                self.alen.fill_(-1)
            if one_launch:   # the first drafts; every step leaves the next ones behind
                sd.sd_speculate(self.ctx, slots, self.trees)

        def step(self):
            if self.one_launch:   # the step bench.py times
                verifier.targets(self.trees.n_nodes, self.trees.parents, future, self.pos,
                                 self.target, advance=self.alen)
                sd.sd_accept_append_speculate(self.ctx, self.trees, slots, self.target, self.alen,
                                              self.apath, self.bonus)
                return
            sd.sd_speculate(self.ctx, slots, self.trees)
            if self.fused:
                verifier.targets(self.trees.n_nodes, self.trees.parents, future, self.pos,
                                 self.target, advance=self.alen)
                sd.sd_accept_append(self.ctx, self.trees, slots, self.target, self.alen,
                                    self.apath, self.bonus)
                return
            verifier.targets(self.trees.n_nodes, self.trees.parents, future, self.pos, self.target)
            sd.sd_accept(self.ctx, self.trees, B, self.target, self.alen, self.apath, self.bonus)
            verifier.collect(self.trees.tokens, self.alen, self.apath, self.bonus, self.new,
                             self.newoff, self.pos)
            sd.sd_index_append(self.ctx, slots, self.new, self.newoff)

        def snapshot(self):
            torch.cuda.synchronize()
            t = self.trees
            return [x.clone() for x in (t.n_nodes, t.tokens, t.parents, t.scores, t.tree_score,
                                        t.match_len, t.source, self.alen, self.apath, self.bonus,
                                        self.pos)]

    eager, graphed, fused, one = Loop(), Loop(), Loop(fused=True), Loop(one_launch=True)
    try:
        torch.cuda.synchronize()
        first = one.snapshot()
        g1 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g1):
            one.step()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            graphed.step()
        gf = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gf):
            fused.step()
        torch.cuda.synchronize()
        moved = 0
        for i in range(steps):
            eager.step()
            want = eager.snapshot()
            g.replay()
            got = graphed.snapshot()
            for a, b in zip(got, want):
                assert torch.equal(a, b), "replay %d differs from the eager step" % i
            # the three-launch step: same trees and acceptance (its positions lag by one step)
            gf.replay()
            gotf = fused.snapshot()
            for a, b in zip(gotf[:10], want[:10]):
                assert torch.equal(a, b), "fused replay %d differs from the eager step" % i
            # the step with one library launch: this step's acceptance, and the next step's drafts
            g1.replay()
            got1 = one.snapshot()
            for a, b in zip(first[:7], want[:7]):
                assert torch.equal(a, b), "one-launch step %d: drafts differ from the eager step" % i
            for a, b in zip(got1[7:10], want[7:10]):
                assert torch.equal(a, b), "one-launch step %d: acceptance differs" % i
            first = got1
            moved += int(want[7].sum())
            # unrelated eager work between replays
            _ = (torch.arange(1000, device=dev) * 2).sum().item()
        assert moved > 0
    finally:
        sd.sd_destroy(eager.ctx)
        sd.sd_destroy(graphed.ctx)
        sd.sd_destroy(fused.ctx)
        sd.sd_destroy(one.ctx)


VARIANTS = [(1, 0), (0, 1), (1, 1)]


@pytest.mark.parametrize("den_mode,linear", VARIANTS)
@pytest.mark.parametrize("cfg", ["tiny", "agentic-s", "lowrep-s"])
def test_variants_sibling_denominator_and_linear(cfg, den_mode, linear):
    """The printed sibling-sum denominator and the chain-only ("linear") variant, alone and
    together, against the oracle run with the same switches."""
    if cfg == "tiny":
        w = make_workload("tiny", seed=5)
    elif cfg == "agentic-s":
        w = make_workload(scaled("agentic", n_docs=300, batch=32, ctx=2048), seed=1, name=cfg)
    else:
        w = make_workload(scaled("lowrep", n_docs=150, batch=48, ctx=4096), seed=1, name=cfg)
    docs = w.docs()
    contexts = [w.contexts[b] for b in range(w.batch)]
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, w.batch, w.ctx_len + 64,
                       len(w.corpus) + len(docs), den_mode=den_mode, linear=linear, tau=2.5)
    try:
        g.build_global(docs)
        g.build_requests(range(w.batch), contexts)
        got = g.speculate(range(w.batch))
        tg = parity.oracle_global_trie(docs, w.D, w.vocab, contexts, w.P)
        want = parity.oracle_speculate_batch(tg, contexts, w.D, w.P, w.alpha, w.min_score,
                                             w.max_nodes, den_mode=den_mode, linear=linear)
        bad = parity.compare_trees(got, want, "%s den=%d linear=%d" % (cfg, den_mode, linear))
        assert not bad, "\n".join(bad)
        # hybrid gate (Section 3): the draft is used iff SCORE > tau
        assert np.array_equal(got["use_draft"], (want["tree_score"] > 2.5).astype(np.int32))
        if linear:
            n = want["n_nodes"]
            for b in range(w.batch):
                assert list(got["parents"][b, :n[b]]) == list(range(-1, n[b] - 1))
        # the switches change results on these inputs (otherwise the test proves nothing)
        base = parity.oracle_speculate_batch(tg, contexts, w.D, w.P, w.alpha, w.min_score,
                                             w.max_nodes)
        if cfg == "tiny":
            assert any(not np.array_equal(base[k], want[k]) for k in ("tokens", "parents", "scores"))
    finally:
        g.close()


@pytest.mark.parametrize("den_mode,linear", VARIANTS)
def test_variants_on_adversarial_minis(den_mode, linear):
    rng = np.random.default_rng(8)
    for name, vocab, D, P, alpha, ms, docs, contexts in MINIS:
        if contexts is None:
            contexts = [list(rng.integers(0, vocab, int(rng.integers(1, 300)))) for _ in range(8)]
        docs_a = [np.asarray(d, np.int32) for d in docs]
        ctx_a = [np.asarray(c, np.int32) for c in contexts]
        B = len(ctx_a)
        g = parity.GpuPath(vocab, D, P, alpha, ms, B, 512, sum(len(d) for d in docs_a) + len(docs_a),
                           den_mode=den_mode, linear=linear)
        try:
            g.build_global(docs_a)
            g.build_requests(range(B), ctx_a)
            got = g.speculate(range(B))
            tg = parity.oracle_global_trie(docs_a, D, vocab)
            want = parity.oracle_speculate_batch(tg, ctx_a, D, P, alpha, ms, g.max_nodes,
                                                 den_mode=den_mode, linear=linear)
            bad = parity.compare_trees(got, want, name)
            assert not bad, "\n".join(bad)
        finally:
            g.close()


# ---- online insertion into the global index -------------------------------------------------
def _sorted_on_D(text, sa, D):
    N = len(sa)
    pad = np.concatenate([text, np.full(D, -1, np.int32)])
    keys = np.stack([pad[sa + k] for k in range(D)], axis=1).astype(np.int64)
    ended = np.cumsum(keys == -1, axis=1) > 0
    keys[ended] = -1
    a, b = keys[:-1], keys[1:]
    diff = a != b
    first = diff.argmax(axis=1)
    rows = np.arange(N - 1)
    return bool((~diff.any(axis=1) | (a[rows, first] < b[rows, first])).all()), keys


def test_insert_equals_build_over_all_documents(tiny_workload):
    """Documents inserted in uneven batches (one of them empty, one with an empty document):
    afterwards text, suffix-array order, interval widths and speculation results are those of one
    build over all documents, and of the oracle trie that received the same documents."""
    w = tiny_workload
    import paper_2411_04975_amd as sd
    docs = [np.asarray(d, np.int32) for d in w.docs()]
    docs.insert(7, np.zeros(0, np.int32))
    N = sum(len(d) for d in docs) + len(docs)
    cuts = [0, 5, 5, 6, 20, len(docs)]
    contexts = [w.contexts[i] for i in range(w.batch)]
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, w.batch, w.ctx_len + 8, N)
    h = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, w.batch, w.ctx_len + 8, N)
    try:
        g.build_requests(range(w.batch), contexts)
        h.build_requests(range(w.batch), contexts)
        tg = oracle.Trie(w.D)
        for a, b in zip(cuts[:-1], cuts[1:]):
            if a == 0:
                g.build_global(docs[a:b])
            else:
                g.insert_global(docs[a:b])
            for d in docs[a:b]:
                tg.add_doc(d)
            got = g.speculate(range(w.batch))
            want = parity.oracle_speculate_batch(tg, contexts, w.D, w.P, w.alpha, w.min_score,
                                                 g.max_nodes)
            bad = parity.compare_trees(got, want, "after documents [%d, %d)" % (a, b))
            assert not bad, "\n".join(bad)
        text, sa = sd.sd_debug_read_global(g.ctx)
        h.build_global(docs)
        text2, sa2 = sd.sd_debug_read_global(h.ctx)
        st = g.stats()
    finally:
        g.close()
        h.close()
    assert st["err_bad_token"] == 0
    assert len(sa) == N and np.array_equal(np.sort(sa), np.arange(N))
    assert np.array_equal(text, text2)
    ok, keys = _sorted_on_D(text, sa, w.D)
    assert ok
    ok2, keys2 = _sorted_on_D(text2, sa2, w.D)
    assert ok2 and np.array_equal(keys, keys2)   # same D-token key at every rank


def test_insert_into_empty_index_and_capacity():
    import paper_2411_04975_amd as sd
    docs = [np.array([3, 1, 4, 1, 5, 9, 2, 6, 5, 3, 5], np.int32), np.array([1, 5, 9, 2], np.int32)]
    ctxs = [np.array([4, 1, 5], np.int32), np.array([9, 2], np.int32)]
    g = parity.GpuPath(10, 8, 4, 2.0, 0.05, 2, 32, 40)
    try:
        g.build_requests(range(2), ctxs)
        g.insert_global(docs[:1])                    # nothing built before
        g.insert_global([])                           # no documents: no change
        g.insert_global(docs[1:])
        got = g.speculate(range(2))
        tg = parity.oracle_global_trie(docs, 8, 10)
        want = parity.oracle_speculate_batch(tg, ctxs, 8, 4, 2.0, 0.05, g.max_nodes)
        assert not parity.compare_trees(got, want)
        with pytest.raises(sd.SdError):               # 17 positions held, 40 allowed
            g.insert_global([np.arange(30, dtype=np.int32) % 10])
        got2 = g.speculate(range(2))                  # the refused call changed nothing
        assert not parity.compare_trees(got2, want)
    finally:
        g.close()


# ---- empirical entropy of the global index ----------------------------------------------------
# Tolerance: both sides add up to ~1e7 terms of size <= 2^40 in different orders and with
# different log2 routines; 1e-9 relative is far above that noise and far below any real error.
ENTROPY_RTOL = 1e-9
# The mean is a difference of two such sums divided by the weight: where it cancels to (nearly)
# nothing, what is left is rounding noise of the sums, a few ulps of log2(N) <= 40 bits.
ENTROPY_ATOL = 1e-12


@pytest.mark.parametrize("case", ["tiny", "tiny-D3", "binary", "all-equal", "distinct", "zipf",
                                  "empty-docs", "many-stops", "deep-D", "wide-runs"])
def test_entropy_matches_oracle(case, tiny_workload):
    rng = np.random.default_rng(31)
    if case == "tiny":
        D, vocab, docs = tiny_workload.D, tiny_workload.vocab, tiny_workload.docs()
    elif case == "tiny-D3":
        D, vocab, docs = 3, tiny_workload.vocab, tiny_workload.docs()[:7]
    elif case == "binary":
        D, vocab, docs = 12, 2, [rng.integers(0, 2, int(n)).astype(np.int32) for n in (300, 1, 77, 500)]
    elif case == "all-equal":
        D, vocab, docs = 9, 3, [np.full(400, 1, np.int32), np.full(5, 1, np.int32), np.full(30, 2, np.int32)]
    elif case == "distinct":
        D, vocab, docs = 6, 1000, [np.arange(700, dtype=np.int32)]
    elif case == "zipf":
        w = make_workload(scaled("lowrep", n_docs=40, doc_len=(500, 500), batch=2, ctx=64), seed=3)
        D, vocab, docs = w.D, w.vocab, w.docs()
    elif case == "many-stops":
        # hundreds of documents end in the same tokens (many suffixes stop at one depth of one
        # run), others run on past them
        D, vocab = 8, 50
        docs = [np.array([int(rng.integers(10, 50)), 5, 6], np.int32) for _ in range(300)]
        docs += [np.array([7, 5, 6, 7, 8, 5, 6], np.int32) for _ in range(37)]
        docs += [np.array([5], np.int32)] * 70 + [rng.integers(0, 50, 400).astype(np.int32)]
    elif case == "deep-D":
        # the largest depth bound: lengths and shared prefixes up to 255, documents shorter and
        # longer than D, repeated so that runs reach the bound
        D, vocab = 255, 9
        a, b = rng.integers(0, 9, 700).astype(np.int32), rng.integers(0, 9, 300).astype(np.int32)
        docs = [a, b, a[100:], np.concatenate([b, a[:280]]), a[:255], a[:254], b[40:296]]
    elif case == "wide-runs":
        # runs of thousands of suffixes at depths 2, 3 and beyond (one phrase in every document),
        # with tails that differ
        D, vocab = 16, 400
        phrase = np.array([1, 2, 3, 4, 5, 6, 7], np.int32)
        docs = [np.concatenate([rng.integers(8, 400, int(rng.integers(0, 4))).astype(np.int32), phrase,
                                rng.integers(8, 400, int(rng.integers(0, 6))).astype(np.int32)])
                for _ in range(3000)]
    else:
        D, vocab, docs = 5, 7, [np.zeros(0, np.int32), np.array([3], np.int32), np.zeros(0, np.int32),
                                np.array([3, 3, 4], np.int32)]
    docs = [np.asarray(d, np.int32) for d in docs]
    N = sum(len(d) for d in docs) + len(docs)
    g = parity.GpuPath(vocab, D, min(4, D - 1), 1.0, 0.1, 1, 16, N + 8)
    try:
        assert g.entropy() == (0.0, 0.0)             # nothing built yet
        g.build_global(docs)
        h, wt = g.entropy()
        h2, wt2 = g.entropy()                        # repeatable, and leaves the index alone
    finally:
        g.close()
    t = oracle.Trie(D)
    for d in docs:
        t.add_doc(d)
    ho, wo = t.entropy()
    assert wt == wo and wt2 == wo
    assert h == pytest.approx(ho, rel=ENTROPY_RTOL, abs=ENTROPY_ATOL)
    assert h2 == pytest.approx(ho, rel=ENTROPY_RTOL, abs=ENTROPY_ATOL)


def test_entropy_fuzz_small_corpora():
    """Seeded corpora of four shapes (random tokens; slices of one text: deep shared prefixes
    and many suffixes that stop together; runs of one token; common endings) over the range of
    vocabularies and depth bounds, capacity with and without slack."""
    for seed in range(120):
        rng = np.random.default_rng(1000 + seed)
        vocab = int(rng.choice([2, 3, 5, 17, 300]))
        D = int(rng.choice([2, 3, 5, 9, 16, 33, 64, 130, 255]))
        kind = int(rng.integers(0, 4))
        base = rng.integers(0, vocab, int(rng.integers(1, 600))).astype(np.int32)
        docs = []
        for _ in range(int(rng.integers(1, 40))):
            if kind == 0:
                d = rng.integers(0, vocab, int(rng.integers(0, 300))).astype(np.int32)
            elif kind == 1:
                a = int(rng.integers(0, len(base)))
                d = base[a:int(rng.integers(a, len(base) + 1))].copy()
            elif kind == 2:
                d = np.full(int(rng.integers(0, 400)), int(rng.integers(0, vocab)), np.int32)
            else:
                tail = base[-int(rng.integers(1, min(len(base), 12) + 1)):]
                d = np.concatenate([rng.integers(0, vocab, int(rng.integers(0, 20))).astype(np.int32), tail])
            docs.append(d)
        N = sum(len(d) for d in docs) + len(docs)
        g = parity.GpuPath(vocab, D, min(4, D - 1), 1.0, 0.1, 1, 16, N + int(rng.integers(0, 9)))
        try:
            g.build_global(docs)
            h, wt = g.entropy()
        finally:
            g.close()
        t = oracle.Trie(D)
        for d in docs:
            t.add_doc(d)
        ho, wo = t.entropy()
        assert wt == wo, (seed, wt, wo)
        assert h == pytest.approx(ho, rel=ENTROPY_RTOL, abs=ENTROPY_ATOL), (seed, vocab, D, kind)


def test_profiling_variants_give_the_same_trees(tiny_workload):
    """The counting (mode 2) and timing (mode 3) variants of the speculation kernel are the
    measured kernel plus bookkeeping: same trees, plausible counters and marks."""
    import paper_2411_04975_amd as sd
    w = tiny_workload
    docs = w.docs()
    B = w.batch
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, w.ctx_len + 8,
                       len(w.corpus) + len(docs))
    try:
        g.build_global(docs)
        g.build_requests(range(B), [w.contexts[b] for b in range(B)])
        base = g.speculate(range(B))
        sd.sd_debug_profile(g.ctx, 2)
        sd.sd_debug_profile_read(g.ctx)
        counted = g.speculate(range(B))
        prof = sd.sd_debug_profile_read(g.ctx)
        sd.sd_debug_profile(g.ctx, 3)
        timed = g.speculate(range(B))
        rt, khz = sd.sd_debug_read_request_ticks(g.ctx, B)
        ut = sd.sd_debug_read_unit_ticks(g.ctx, B)
        sd.sd_debug_profile(g.ctx, 0)
    finally:
        g.close()
    for other in (counted, timed):
        for k in base:
            assert np.array_equal(base[k], other[k]), k
    assert prof["speculate"]["launches"] == 1 and prof["speculate"]["ms"] > 0
    # at least the context scan (4 B per token) and the emitted trees are counted
    assert prof["speculate"]["algo_bytes"] >= B * w.ctx_len * 4
    assert khz > 0
    nw = int(rt[0, 0, 7])
    assert 1 <= nw <= 16
    m = rt[:, :nw, :].astype(np.int64)
    assert np.all(m[:, :, 1] <= m[:, :, 2]) and np.all(m[:, :, 2] <= m[:, :, 3])
    assert np.all(m[:, :, 3] <= m[:, :, 4])
    assert np.all(m[:, 0, 6] >= 1)                     # the context's own last token
    assert ut.shape == (B, 2, w.P, 4)


def test_fused_step_under_profiling_modes_and_bad_arguments(tiny_workload):
    """sd_accept_append_speculate gives the same results whatever the profiling mode (the
    counting and timing variants exist for the separate kernels, which it then runs), is
    timed under its own name in mode 1, and turns bad arguments into errors on the host."""
    import torch
    import paper_2411_04975_amd as sd
    w = tiny_workload
    docs = w.docs()
    B, mn = w.batch, w.max_nodes
    results = []
    for mode in (0, 1, 2, 3):
        g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, w.ctx_len + 2 * (mn + 1),
                           len(w.corpus) + len(docs))
        try:
            g.build_global(docs)
            g.build_requests(range(B), [w.contexts[b] for b in range(B)])
            got = g.speculate(range(B))
            fut = np.stack([w.future[b, :mn + 2] for b in range(B)])
            tgt = parity.targets_from_future(got, fut, mn)
            sd.sd_debug_profile(g.ctx, mode)
            sd.sd_debug_profile_read(g.ctx)
            al, ap, bo, nxt = g.accept_append_speculate(range(B), tgt)
            prof = sd.sd_debug_profile_read(g.ctx)
            sd.sd_debug_profile(g.ctx, 0)
            results.append((al, ap, bo, nxt))
            if mode == 1:
                assert prof["accept_speculate"]["launches"] == 1 and prof["speculate"]["launches"] == 0
            if mode >= 2:
                assert prof["accept"]["launches"] == 1 and prof["speculate"]["launches"] == 1
            if mode == 0:
                dev = g.dev
                i32 = torch.int32
                slots = torch.arange(B, dtype=i32, device=dev)
                d_t = torch.zeros((B, mn + 1), dtype=i32, device=dev)
                al_, ap_, bo_ = (torch.zeros(B, dtype=i32, device=dev),
                                 torch.zeros((B, mn), dtype=i32, device=dev),
                                 torch.zeros(B, dtype=i32, device=dev))
                small = sd.Trees(B, mn - 1, dev) if mn > 1 else None
                if small is not None:
                    with pytest.raises(sd.SdError):        # fewer nodes than floor(alpha P)
                        sd.sd_accept_append_speculate(g.ctx, small, slots, d_t[:, :mn].contiguous(),
                                                      al_, ap_[:, :mn - 1].contiguous(), bo_)
                many = torch.arange(B + 1, dtype=i32, device=dev)
                big = sd.Trees(B + 1, mn, dev)
                with pytest.raises(sd.SdError):            # more requests than slots
                    sd.sd_accept_append_speculate(
                        g.ctx, big, many, torch.zeros((B + 1, mn + 1), dtype=i32, device=dev),
                        torch.zeros(B + 1, dtype=i32, device=dev),
                        torch.zeros((B + 1, mn), dtype=i32, device=dev),
                        torch.zeros(B + 1, dtype=i32, device=dev))
                assert g.stats()["err_bad_slot"] == 0      # nothing was launched
        finally:
            g.close()
    base = results[0]
    for other in results[1:]:
        for a, b in zip(base[:3], other[:3]):
            assert np.array_equal(a, b)
        for k in base[3]:
            assert np.array_equal(base[3][k], other[3][k]), k


@pytest.mark.parametrize("D", [5, 16, 40])
def test_suffix_array_with_long_and_short_groups(D):
    """Runs of one token (groups of hundreds of equal prefixes, which need the device-wide sort
    rounds) next to random text (groups of one or two, reordered inside LDS tiles), a group that
    straddles tile boundaries, documents of one token and empty ones: the result must be a
    permutation ordered on D tokens, and insertion must keep it so."""
    import paper_2411_04975_amd as sd
    rng = np.random.default_rng(77)
    docs = [np.full(300, 7, np.int32), rng.integers(0, 50, 3000).astype(np.int32),
            np.tile(np.array([1, 2, 3], np.int32), 400), np.zeros(0, np.int32),
            np.array([9], np.int32), rng.integers(0, 3, 2500).astype(np.int32),
            np.full(70, 7, np.int32)]
    more = [np.full(130, 7, np.int32), rng.integers(0, 50, 500).astype(np.int32)]
    N = sum(len(d) for d in docs + more) + len(docs) + len(more)
    g = parity.GpuPath(64, D, 4, 1.0, 0.1, 1, 16, N)
    try:
        g.build_global(docs)
        text, sa = sd.sd_debug_read_global(g.ctx)
        n0 = sum(len(d) for d in docs) + len(docs)
        assert len(sa) == n0 and np.array_equal(np.sort(sa), np.arange(n0))
        assert _sorted_on_D(text, sa, D)[0]
        g.insert_global(more)
        text, sa = sd.sd_debug_read_global(g.ctx)
        assert len(sa) == N and np.array_equal(np.sort(sa), np.arange(N))
        assert _sorted_on_D(text, sa, D)[0]
        want_text = np.concatenate([np.concatenate([d, [-1]]) for d in docs + more]).astype(np.int32)
        assert np.array_equal(text, want_text)
    finally:
        g.close()


def test_global_build_captured_into_a_graph():
    """A build enqueued on a stream that is being captured cannot wait for the stream to see
    which sorting rounds need their device-wide fall-back: it enqueues every round with its
    fall-back behind a device-side switch.  The corpus has runs of one token (rounds that fall
    back) next to random text; the graph is replayed twice, with other work in between, and the
    index must be sorted on D tokens and draft like the oracle each time."""
    import torch
    import paper_2411_04975_amd as sd
    rng = np.random.default_rng(78)
    D, P, alpha, ms, vocab = 16, 6, 2.0, 0.05, 64
    docs = [np.full(300, 7, np.int32), rng.integers(0, 50, 3000).astype(np.int32),
            np.tile(np.array([1, 2, 3], np.int32), 400), np.zeros(0, np.int32),
            np.array([9], np.int32), rng.integers(0, 3, 2500).astype(np.int32)]
    ctxs = [np.concatenate([rng.integers(0, 50, 20), d[5:5 + 12]]).astype(np.int32)
            for d in (docs[1], docs[2], docs[5], docs[0])]
    N = sum(len(d) for d in docs) + len(docs)
    g = parity.GpuPath(vocab, D, P, alpha, ms, len(ctxs), 64, N)
    try:
        d_tok, d_off, n = g._seqs(docs)
        g.build_global([np.array([5, 5, 5], np.int32)])       # something else first
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            sd.sd_index_build(g.ctx, sd.SD_SCOPE_GLOBAL, None, d_tok, d_off, n)
        tg = oracle.Trie(D)
        for d in docs:
            tg.add_doc(d)
        want = parity.oracle_speculate_batch(tg, ctxs, D, P, alpha, ms, g.max_nodes)
        g.build_requests(range(len(ctxs)), ctxs)
        for rep in range(2):
            gr.replay()
            torch.cuda.synchronize()
            text, sa = sd.sd_debug_read_global(g.ctx)
            assert len(sa) == N and np.array_equal(np.sort(sa), np.arange(N))
            assert _sorted_on_D(text, sa, D)[0]
            bad = parity.compare_trees(g.speculate(range(len(ctxs))), want, "replay %d" % rep)
            assert not bad, "\n".join(bad)
            _ = (torch.arange(1000, device=g.dev) * 2).sum().item()
    finally:
        g.close()


@pytest.mark.parametrize("n", [255, 256, 257, 640, 1023, 1024, 1025, 2500, 4095, 4096, 4097, 6000])
def test_first_token_buckets_around_the_scan_limits(n):
    """The second pattern token is located inside the first token's bucket by one of three
    routes, chosen by the bucket's size (up to 256 entries, up to 1024, beyond): token 0 gets
    exactly n occurrences here, other tokens about n / 5 or n / 3, and patterns of every length
    up to 20 (so that both the one-pattern and the two-patterns-at-once stages run) must match
    as in the oracle."""
    rng = np.random.default_rng(n)
    body = []
    for i in range(n):
        body += [0, 1 + int(rng.integers(0, 5)), 6 + int(rng.integers(0, 3))]
        if rng.random() < 0.3:
            body.append(9 + int(rng.integers(0, 3)))
    doc = np.array(body, np.int32)
    assert int((doc == 0).sum()) == n
    docs = [doc[:len(doc) // 2], doc[len(doc) // 2:]]
    ctxs = []
    for _ in range(12):
        a = int(rng.integers(0, len(doc) - 30))
        x = doc[a:a + int(rng.integers(2, 30))].copy()
        k = int(rng.integers(0, 3))
        if k == 1:
            x = np.concatenate([x, [0]])                         # ends with the wide bucket's token
        elif k == 2:
            x = np.concatenate([x, [0, 1 + int(rng.integers(0, 5))]])
        ctxs.append(x.astype(np.int32))
    vocab, D, P, alpha, ms = 12, 24, 20, 1.0, 0.02
    B = len(ctxs)
    g = parity.GpuPath(vocab, D, P, alpha, ms, B, 64, len(doc) + 4)
    try:
        g.build_global(docs)
        g.build_requests(range(B), ctxs)
        got = g.speculate(range(B))
        tg = oracle.Trie(D)
        for d in docs:
            tg.add_doc(d)
        want = parity.oracle_speculate_batch(tg, ctxs, D, P, alpha, ms, g.max_nodes)
        bad = parity.compare_trees(got, want, "bucket of %d" % n)
        assert not bad, "\n".join(bad)
        assert int((want["source"] == 0).sum()) >= B // 2
    finally:
        g.close()


def test_largest_vocabulary_and_depth():
    """vocab = 2^24 and D = 255, the largest the library takes: token codes of 25 bits (the
    first sort's keys hold two of them; the occurrence sort's keys then hold two tokens instead
    of three), suffixes compared on 255 tokens.  A handful of token ids from the top of the
    range, in contexts whose last token occurs a few hundred times (several sorted runs that
    are merged; equal keys that the tokens beyond the key must order) and a corpus that repeats
    a long piece, so that matches and chains run deep."""
    rng = np.random.default_rng(224)
    vocab, D, P, alpha, ms = 1 << 24, 255, 8, 2.0, 0.02
    ids = np.array([vocab - 1, vocab - 2, vocab - 77, 1 << 23, (1 << 23) + 1, 3, 0], np.int32)
    piece = ids[rng.integers(0, len(ids), 400)]
    docs = [piece[a:a + 300].copy() for a in (0, 20, 50, 90)]
    docs.append(ids[rng.integers(0, 3, 500)])
    ctxs = []
    for i in range(10):
        body = ids[rng.integers(0, 3 if i % 2 else len(ids), int(rng.integers(150, 900)))]
        e = int(rng.integers(100, 390))
        if i % 3 == 0:      # a context that repeats a piece of its own, which the corpus does not hold
            unit = ids[rng.integers(0, len(ids), 37)]
            ctxs.append(np.concatenate([body, np.tile(unit, 9)[:-int(rng.integers(1, 30))]]).astype(np.int32))
        else:
            ctxs.append(np.concatenate([body, piece[e - 60:e]]).astype(np.int32))
    B = len(ctxs)
    n_pos = sum(len(d) for d in docs) + len(docs)
    g = parity.GpuPath(vocab, D, P, alpha, ms, B, 1400, n_pos)
    try:
        g.build_global(docs)
        text, sa = sd_read_global(g)
        assert _sorted_on_D(text, sa, D)[0]
        g.build_requests(range(B), ctxs)
        got = g.speculate(range(B))
        tg = oracle.Trie(D)
        for d in docs:
            tg.add_doc(d)
        want = parity.oracle_speculate_batch(tg, ctxs, D, P, alpha, ms, g.max_nodes)
        bad = parity.compare_trees(got, want, "vocab 2^24, D 255")
        assert not bad, "\n".join(bad)
        assert int((want["source"] == 1).sum()) >= 1 and int((want["source"] == 0).sum()) >= 1
    finally:
        g.close()


@pytest.mark.parametrize("copies,alphabet,alpha", [(3, 50, 1.5), (90, 50, 1.5), (90, 3, 1.5), (6000, 3, 1.5),
                                                   (90, 50, 4.0), (6000, 3, 4.0)])
def test_longest_patterns(copies, alphabet, alpha):
    """P = 64, the largest pattern length the library takes, with D = 140 and alpha 1.5 (trees
    of up to 96 nodes) or 4 (256 nodes, the largest tree; fewer waves per workgroup then, for
    the LDS their frontiers take): contexts end inside text that the corpus holds `copies` times, so that
    patterns of every length up to 64 match, at once from the suffixes that start with the last
    two tokens (few copies) or one pattern length at a time, singly above length 32 (many
    copies; a three-letter alphabet makes the first tokens' buckets wide and the ranges long),
    and the request's own index sees left-extensions of up to 64 tokens."""
    rng = np.random.default_rng(64000 + copies + alphabet)
    vocab, D, P, ms = 60, 140, 64, 0.02
    piece = rng.integers(0, alphabet, 200).astype(np.int32)
    docs = []
    for i in range(copies):
        a = int(rng.integers(0, 60))
        d = piece[a:a + int(rng.integers(100, 140))].copy()
        if i % 3 == 0:
            d[int(rng.integers(0, len(d)))] = int(rng.integers(0, alphabet))    # a mutation
        docs.append(np.concatenate([rng.integers(0, alphabet, int(rng.integers(0, 9))).astype(np.int32), d]))
    docs.append(rng.integers(0, alphabet, 300).astype(np.int32))
    ctxs = []
    for i in range(12):
        e = int(rng.integers(70, 190))
        x = piece[max(0, e - int(rng.integers(1, 150))):e].copy()
        if i % 4 == 1:                                   # the context repeats its own tail further up
            x = np.concatenate([x, rng.integers(0, alphabet, 5).astype(np.int32), x[-70:]])
        if i % 4 == 2 and len(x) > 40:                   # a break 40 tokens before the end
            x[-40] = (int(x[-40]) + 1) % alphabet
        ctxs.append(x.astype(np.int32))
    B = len(ctxs)
    n_pos = sum(len(d) for d in docs) + len(docs)
    g = parity.GpuPath(vocab, D, P, alpha, ms, B, 400, n_pos)
    try:
        g.build_global(docs)
        g.build_requests(range(B), ctxs)
        got = g.speculate(range(B))
        tg = oracle.Trie(D)
        for d in docs:
            tg.add_doc(d)
        want = parity.oracle_speculate_batch(tg, ctxs, D, P, alpha, ms, g.max_nodes)
        bad = parity.compare_trees(got, want, "P = 64, %d copies, alphabet %d" % (copies, alphabet))
        assert not bad, "\n".join(bad)
        assert int(want["match_len"].max()) > 32, "a pattern longer than 32 tokens wins somewhere"
        assert int((want["n_nodes"] > 0).sum()) >= B // 2
        # a fused step on these trees (more than 64 nodes: the acceptance settles them in LDS):
        # the targets follow each draft's first-child chain for some nodes, then differ
        mn = g.max_nodes
        tgt = np.full((B, mn + 1), vocab - 1, np.int32)
        tries, ctx2, exp = [], [], []
        for b in range(B):
            n = int(want["n_nodes"][b])
            v = -1
            for _ in range(int(rng.integers(0, 90))):
                kids = [j for j in range(n) if want["parents"][b, j] == v]
                if not kids:
                    break
                tgt[b, v + 1] = want["tokens"][b, kids[0]]
                v = kids[0]
            L, path, bonus = oracle.accept(want["tokens"][b, :n], want["parents"][b, :n], tgt[b])
            new = np.array([int(want["tokens"][b, j]) for j in path] + [int(bonus)], np.int32)
            exp.append((L, list(path), bonus))
            ctx2.append(np.concatenate([ctxs[b], new]))
            tr = oracle.Trie(D)
            tr.append(ctx2[b])
            tries.append(tr)
        al, ap, bo, got2 = g.accept_append_speculate(range(B), tgt)
        for b in range(B):
            L, path, bonus = exp[b]
            assert al[b] == L and bo[b] == bonus and list(ap[b, :L]) == path, b
        assert max(e[0] for e in exp) > 40
        want2 = parity.oracle_speculate_batch(tg, ctx2, D, P, alpha, ms, mn, request_tries=tries)
        bad = parity.compare_trees(got2, want2, "fused step at P = 64")
        assert not bad, "\n".join(bad)
    finally:
        g.close()


@pytest.mark.parametrize("n,filler", [(1, 0), (2, 0), (63, 0), (64, 0), (65, 0), (130, 0), (40, 5000),
                                      (64, 4000), (0, 0)])
def test_two_token_anchor_around_the_list_limits(n, filler):
    """All pattern lengths of the global index are settled from the suffixes that start with
    the context's last two tokens when there are at most 64 of them (and their first token's
    bucket is within the sampled lookup's reach), and searched for one by one otherwise.  Here
    the pair (7, 8) occurs exactly n times, each time behind a piece of the context's tail of
    another length (so every pattern length has its own count), at the very start of a document
    and behind other documents' ends; `filler` further occurrences of 7 widen its bucket.  Both
    routes must give the oracle's trees, for contexts of every length from 0 on."""
    rng = np.random.default_rng(1000 * n + filler)
    vocab, D, P, alpha, ms = 40, 14, 9, 2.0, 0.01
    tailtok = rng.integers(10, 40, P - 2).astype(np.int32)          # the context's tail before (7, 8)
    docs = []
    for i in range(n):
        keep = int(rng.integers(0, P - 1))                           # tokens of the tail in front
        pre = rng.integers(10, 40, int(rng.integers(0, 6))).astype(np.int32) if i % 5 else np.zeros(0, np.int32)
        cont = rng.integers(0, 4, int(rng.integers(0, 8))).astype(np.int32)   # few distinct tokens: ties
        docs.append(np.concatenate([pre, tailtok[len(tailtok) - keep:], [7, 8], cont]).astype(np.int32))
    if filler:
        docs.append(np.tile(np.array([7, 9], np.int32), filler))
    docs.append(rng.integers(0, 40, 50).astype(np.int32))
    order = rng.permutation(len(docs))
    docs = [docs[i] for i in order]
    full = np.concatenate([rng.integers(10, 40, 5).astype(np.int32), tailtok, [7, 8]]).astype(np.int32)
    ctxs = [full[len(full) - k:] for k in range(0, len(full) + 1)]    # lengths 0 .. all
    ctxs += [np.concatenate([full, [7]]).astype(np.int32), np.concatenate([full[:-1], [9]]).astype(np.int32)]
    B = len(ctxs)
    N = sum(len(d) for d in docs) + len(docs)
    g = parity.GpuPath(vocab, D, P, alpha, ms, B, 64, N + 4)
    try:
        g.build_global(docs)
        g.build_requests(range(B), ctxs)
        got = g.speculate(range(B))
        tg = oracle.Trie(D)
        for d in docs:
            tg.add_doc(d)
        want = parity.oracle_speculate_batch(tg, ctxs, D, P, alpha, ms, g.max_nodes)
        bad = parity.compare_trees(got, want, "pair occurs %d times, filler %d" % (n, filler))
        assert not bad, "\n".join(bad)
        if n:
            assert int(want["match_len"].max()) >= 2
    finally:
        g.close()


def test_wide_batches_on_thinner_workgroups():
    """Batches of several workgroups per compute unit run on workgroups of fewer waves (the
    library sizes them by the batch): 775 and 3329 requests must give the trees of the oracle
    row by row, and so must a fused step at 775.  The requests are 114 distinct contexts,
    repeated over the slots: 16 drawn ones, each with 0..6 tokens cut off its end, and two of
    three tokens only whose last token occurs about 1400 and 1650 times: thinner workgroups
    have less LDS, so these are sorted in LDS at one width and in device memory at another."""
    import paper_2411_04975_amd as sd
    w = make_workload(scaled("tiny", alpha=2.0, min_score=0.05), seed=5)
    docs = w.docs()
    mn = w.max_nodes
    variants = [w.contexts[i % 16][:w.ctx_len - (i // 16)] for i in range(112)]
    rng = np.random.default_rng(77)
    for share in (0.74, 0.86):
        x = np.where(rng.random(1900) < share, 7, rng.integers(8, 10, 1900)).astype(np.int32)
        x[-1] = 7
        variants.append(x)
    NV = len(variants)
    tg = parity.oracle_global_trie(docs, w.D, w.vocab)
    tries = []
    for x in variants:
        t = oracle.Trie(w.D)
        t.append(x)
        tries.append(t)
    want_v = parity.oracle_speculate_batch(tg, variants, w.D, w.P, w.alpha, w.min_score, mn,
                                           request_tries=tries)
    assert len(set(want_v["n_nodes"].tolist())) > 3

    def rows(want, B):
        idx = np.arange(B) % NV
        return {k: v[idx] for k, v in want.items()}

    B = 3329
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, 1900 + mn + 1,
                       len(w.corpus) + len(docs))
    try:
        g.build_global(docs)
        g.build_requests(range(B), [variants[b % NV] for b in range(B)])
        for nb in (3329, 775):
            got = g.speculate(range(nb))
            bad = parity.compare_trees(got, rows(want_v, nb), "batch %d" % nb)
            assert not bad, "\n".join(bad)
            if nb > sd.SD_TICK_SLOTS:      # the timing variant keeps marks for that many requests
                continue
            sd.sd_debug_profile(g.ctx, 3)
            timed = g.speculate(range(nb))
            rt, _ = sd.sd_debug_read_request_ticks(g.ctx, nb)
            sd.sd_debug_profile(g.ctx, 0)
            assert 1 <= int(rt[0, 0, 7]) < 8, "the batch ran on full-width workgroups"
            assert not parity.compare_trees(timed, rows(want_v, nb), "timing variant, batch %d" % nb)
        # the fused step at 775: the targets follow each draft's first-child chain for a
        # number of nodes that depends on the variant, then differ
        nb = 775
        tgt_v = np.full((NV, mn + 1), w.vocab - 1, np.int32)
        new_v = []
        for i in range(NV):
            n = int(want_v["n_nodes"][i])
            v = -1
            for _ in range(i % 5):
                kids = [j for j in range(n) if want_v["parents"][i, j] == v]
                if not kids:
                    break
                tgt_v[i, v + 1] = want_v["tokens"][i, kids[0]]
                v = kids[0]
            L, path, bonus = oracle.accept(want_v["tokens"][i, :n], want_v["parents"][i, :n], tgt_v[i])
            new = np.array([int(want_v["tokens"][i, j]) for j in path] + [int(bonus)], np.int32)
            new_v.append((L, list(path), bonus))
            tries[i].append(new)
            variants[i] = np.concatenate([variants[i], new])
        al, ap, bo, got = g.accept_append_speculate(range(nb), tgt_v[np.arange(nb) % NV])
        for b in range(nb):
            L, path, bonus = new_v[b % NV]
            assert al[b] == L and bo[b] == bonus and list(ap[b, :L]) == path, b
        assert sum(v[0] for v in new_v) > 50
        want2 = parity.oracle_speculate_batch(tg, variants, w.D, w.P, w.alpha, w.min_score, mn,
                                              request_tries=tries)
        bad = parity.compare_trees(got, rows(want2, nb), "fused step, batch %d" % nb)
        assert not bad, "\n".join(bad)
        st = g.stats()
        assert st["err_bad_token"] == 0 and st["err_bad_slot"] == 0 and st["err_ctx_overflow"] == 0
    finally:
        g.close()


def _fuzz_case(seed):
    """A small random configuration: vocabulary, bounds, thresholds, variants, document and
    context shapes all drawn from the seed (repetitive and random text mixed)."""
    rng = np.random.default_rng(1000 + seed)
    vocab = int(rng.choice([2, 3, 5, 17, 300]))
    P = int(rng.integers(1, 13))
    D = int(P + rng.integers(1, 30))
    alpha = float(rng.choice([0.5, 1.0, 1.5, 2.0, 4.0, 7.3]))
    if np.floor(alpha * P) < 1:
        alpha = 1.0
    ms = float(rng.choice([0.0, 0.01, 0.05, 0.2, 0.5, 1.0]))
    den_mode, linear = int(rng.integers(0, 2)), int(rng.integers(0, 4) == 0)
    base = rng.integers(0, vocab, int(rng.integers(5, 60)))

    def seq(n):
        parts, total = [], 0
        while total < n:
            if rng.random() < 0.6:                       # a copy of a piece of the base text
                a = int(rng.integers(0, len(base)))
                piece = base[a:a + int(rng.integers(1, 25))]
            else:
                piece = rng.integers(0, vocab, int(rng.integers(1, 12)))
            parts.append(piece)
            total += len(piece)
        return np.concatenate(parts)[:n].astype(np.int32) if n else np.zeros(0, np.int32)

    docs = [seq(int(rng.integers(0, 400))) for _ in range(int(rng.integers(1, 9)))]
    ctxs = [seq(int(rng.integers(0, 200))) for _ in range(int(rng.integers(1, 6)))]
    return vocab, D, P, alpha, ms, den_mode, linear, docs, ctxs


@pytest.mark.parametrize("chunk", range(6))
def test_fuzz_small_configurations(chunk):
    """60 random small configurations (10 per test), every switch of the library drawn at
    random, each compared with the oracle after build, after an insertion and after an append."""
    for seed in range(chunk * 10, chunk * 10 + 10):
        vocab, D, P, alpha, ms, den_mode, linear, docs, ctxs = _fuzz_case(seed)
        rng = np.random.default_rng(5000 + seed)
        cut = int(rng.integers(0, len(docs) + 1))
        B = len(ctxs)
        N = sum(len(d) for d in docs) + len(docs)
        g = parity.GpuPath(vocab, D, P, alpha, ms, B, 256, N + 4, den_mode=den_mode, linear=linear)
        label = "fuzz seed %d (vocab %d D %d P %d alpha %g ms %g den %d lin %d)" % (
            seed, vocab, D, P, alpha, ms, den_mode, linear)
        try:
            g.build_global(docs[:cut])
            g.build_requests(range(B), ctxs)
            tg = oracle.Trie(D)
            for d in docs[:cut]:
                tg.add_doc(d)
            tries = []
            for x in ctxs:
                t = oracle.Trie(D)
                t.append(x)
                tries.append(t)

            def check(tag):
                got = g.speculate(range(B))
                want = parity.oracle_speculate_batch(tg, ctxs, D, P, alpha, ms, g.max_nodes,
                                                     request_tries=tries, den_mode=den_mode,
                                                     linear=linear)
                bad = parity.compare_trees(got, want, label + " " + tag)
                assert not bad, "\n".join(bad)
                return want

            check("after build")
            g.insert_global(docs[cut:])
            for d in docs[cut:]:
                tg.add_doc(d)
            want = check("after insert")
            # append a few tokens per request: the best tree's first tokens, or random ones
            new = []
            for b in range(B):
                k = int(rng.integers(0, 4))
                toks = [int(v) for v in want["tokens"][b, :min(k, int(want["n_nodes"][b]))]]
                toks += [int(v) for v in rng.integers(0, vocab, k - len(toks))]
                new.append(np.array(toks, np.int32))
                tries[b].append(new[-1])
                ctxs[b] = np.concatenate([ctxs[b], new[-1]])
            g.append(range(B), new)
            check("after append")
            st = g.stats()
            assert st["err_bad_token"] == 0 and st["err_bad_slot"] == 0 and st["err_ctx_overflow"] == 0
        finally:
            g.close()


@pytest.mark.parametrize("vocab,D,P,alpha,copies", [
    (50000, 64, 32, 2.0, 3), (50000, 64, 32, 2.0, 4), (50000, 64, 32, 2.0, 6),
    (3, 64, 32, 2.0, 3), (3, 64, 24, 2.0, 5), (7, 48, 16, 4.0, 3),
    (50000, 200, 32, 2.0, 3), (5, 200, 32, 2.0, 4), (50000, 255, 60, 1.0, 9),
])
def test_tied_chain_merges(vocab, D, P, alpha, copies):
    """Trees whose top scores tie between several single-occurrence chains: a template occurs
    `copies` times, every copy with one token of its own a few places behind the pattern, and
    goes on alike afterwards (equal tokens at equal offsets: the tie rule decides all along).
    Large and tiny vocabularies, depth bounds that the staged windows reach (64) and do not
    reach (200, 255), two to nine chains, trees cut by K and trees that end by themselves."""
    rng = np.random.default_rng(vocab * 1000 + D + copies)
    docs, ctxs = [], []
    for case in range(6):
        L = int(rng.integers(P + 8, P + 140))
        tmpl = rng.integers(0, vocab, L).astype(np.int32)
        head = int(rng.integers(P, P + 6))          # the pattern and a few tokens all copies share
        for c in range(copies):
            d = tmpl.copy()
            at = head + int(rng.integers(0, 4)) + (c % 2)
            if at < L:
                d[at] = (d[at] + 1 + c) % vocab       # this copy's own token (may tie with another's)
            cut = L if rng.random() < 0.6 else int(rng.integers(head + 1, L + 1))
            docs.append(d[:cut])
        pre = rng.integers(0, vocab, int(rng.integers(0, 20))).astype(np.int32)
        ctxs.append(np.concatenate([pre, tmpl[:head - int(rng.integers(0, 5))]]).astype(np.int32))
    B = len(ctxs)
    N = sum(len(d) for d in docs) + len(docs)
    g = parity.GpuPath(vocab, D, P, alpha, 0.01, B, 512, N + 4)
    try:
        g.build_global(docs)
        g.build_requests(range(B), ctxs)
        tg = oracle.Trie(D)
        for d in docs:
            tg.add_doc(d)
        got = g.speculate(range(B))
        want = parity.oracle_speculate_batch(tg, ctxs, D, P, alpha, 0.01, g.max_nodes)
        bad = parity.compare_trees(got, want, "tied chains vocab %d D %d copies %d" % (vocab, D, copies))
        assert not bad, "\n".join(bad)
        # the case is what it claims to be: trees that branch into several chains
        branching = 0
        for b in range(B):
            n = int(want["n_nodes"][b])
            par = [int(v) for v in want["parents"][b, :n]]
            kids = {}
            for v in par:
                kids[v] = kids.get(v, 0) + 1
            branching += any(k >= 2 for k in kids.values())
        assert branching >= 3, branching
    finally:
        g.close()


@pytest.mark.parametrize("chunk", [0, 1, 2, 3, 460])
def test_fuzz_fused_decode_loops(chunk):
    """50 random small configurations (10 per test), four decode steps each, every step ended by
    sd_accept_append_speculate: acceptance, appended contexts and next drafts against the
    oracle.  The targets follow a random draft path for a random number of nodes, so accepted
    lengths of every size occur; contexts start at every length from empty on.  (Chunk 460 holds
    a step in which the request's own tree and the global one tie node for node: the earlier
    one must win, which a bound on a tree's reachable SCORE must not get in the way of.)"""
    accepted = 0
    for seed in range(chunk * 10, chunk * 10 + 10):
        vocab, D, P, alpha, ms, den_mode, linear, docs, ctxs = _fuzz_case(1000 + seed)
        rng = np.random.default_rng(9000 + seed)
        ctxs = [c[:int(rng.integers(0, len(c) + 1))] if rng.random() < 0.3 else c for c in ctxs]
        B = len(ctxs)
        N = sum(len(d) for d in docs) + len(docs)
        g = parity.GpuPath(vocab, D, P, alpha, ms, B, 256 + 5 * 260, N + 4, den_mode=den_mode,
                           linear=linear)
        mn = g.max_nodes
        label = "fused fuzz seed %d (vocab %d D %d P %d alpha %g ms %g den %d lin %d)" % (
            seed, vocab, D, P, alpha, ms, den_mode, linear)
        try:
            g.build_global(docs)
            g.build_requests(range(B), ctxs)
            tg = oracle.Trie(D)
            for d in docs:
                tg.add_doc(d)
            tries = []
            for x in ctxs:
                t = oracle.Trie(D)
                t.append(x)
                tries.append(t)
            ctxs = [np.asarray(c, np.int32) for c in ctxs]
            got = g.speculate(range(B))
            for step in range(4):
                want = parity.oracle_speculate_batch(tg, ctxs, D, P, alpha, ms, mn,
                                                     request_tries=tries, den_mode=den_mode,
                                                     linear=linear)
                bad = parity.compare_trees(got, want, label + " step %d" % step)
                assert not bad, "\n".join(bad)
                # targets: random tokens, then a random root path of the draft made to agree
                tgt = rng.integers(0, vocab, (B, mn + 1)).astype(np.int32)
                for b in range(B):
                    n = int(want["n_nodes"][b])
                    v = -1
                    for _ in range(int(rng.integers(0, n + 2))):
                        kids = [j for j in range(n) if want["parents"][b, j] == v]
                        if not kids:
                            break
                        j = kids[int(rng.integers(0, len(kids)))]
                        tgt[b, v + 1] = want["tokens"][b, j]
                        v = j
                al, ap, bo, got = g.accept_append_speculate(range(B), tgt)
                for b in range(B):
                    n = int(want["n_nodes"][b])
                    L, path, bonus = oracle.accept(want["tokens"][b, :n], want["parents"][b, :n], tgt[b])
                    assert al[b] == L and bo[b] == bonus and list(ap[b, :L]) == list(path), label
                    assert list(ap[b, L:]) == [-1] * (mn - L), label
                    new = np.array([int(want["tokens"][b, j]) for j in path] + [int(bonus)], np.int32)
                    tries[b].append(new)
                    ctxs[b] = np.concatenate([ctxs[b], new])
                    accepted += L
            want = parity.oracle_speculate_batch(tg, ctxs, D, P, alpha, ms, mn, request_tries=tries,
                                                 den_mode=den_mode, linear=linear)
            bad = parity.compare_trees(got, want, label + " after the last step")
            assert not bad, "\n".join(bad)
            st = g.stats()
            assert st["err_ctx_overflow"] == 0 and st["err_bad_token"] == 0, label
        finally:
            g.close()
    assert accepted > 20
