"""GPU parity at the benchmark configurations' full sizes, in the launch configuration
bench.py times (whole batch, full corpus).  The oracle checks a sample of requests one by one
(its global trie holds exactly the suffixes those requests can reach); properties that hold
at any size are checked for every request."""
import math

import numpy as np
import pytest

import oracle
from tests import parity
from workloads import make_workload

pytestmark = pytest.mark.gpu


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


def _run_full(name, sample, seed=0):
    w = make_workload(name, seed=seed)
    docs = w.docs()
    B = w.batch
    contexts = [w.contexts[b] for b in range(B)]
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, w.ctx_len + 128,
                       len(w.corpus) + len(docs))
    try:
        g.build_global(docs)
        g.build_requests(range(B), contexts)
        got = g.speculate(range(B))
        st = g.stats()
        assert st["err_bad_token"] == 0 and st["err_bad_slot"] == 0
        _check_properties(got, w)
        rng = np.random.default_rng(1)
        pick = sorted(rng.choice(B, size=min(sample, B), replace=False).tolist())
        sub = [contexts[b] for b in pick]
        tg = parity.oracle_global_trie(docs, w.D, w.vocab, sub, w.P)
        want = parity.oracle_speculate_batch(tg, sub, w.D, w.P, w.alpha, w.min_score, w.max_nodes)
        got_sub = {k: v[pick] for k, v in got.items()}
        bad = parity.compare_trees(got_sub, want, name)
        assert not bad, "\n".join(bad)
        # acceptance on the whole batch, oracle on the sample
        tgt = parity.targets_from_future(got, w.future, w.max_nodes)
        al, ap, bo = g.accept(tgt)
        for i, b in enumerate(pick):
            k = int(want["n_nodes"][i])
            L, path, bonus = oracle.accept(want["tokens"][i, :k], want["parents"][i, :k], tgt[b])
            assert al[b] == L and bo[b] == bonus and list(ap[b, :L]) == list(path)
        assert np.all(al <= got["n_nodes"])
        # the decode step as bench.py runs it: the same acceptance, the append and the next
        # drafts in one launch over the whole batch; sampled requests against the oracle on
        # their extended contexts
        al2, ap2, bo2, nxt = g.accept_append_speculate(range(B), tgt)
        assert np.array_equal(al2, al) and np.array_equal(bo2, bo) and np.array_equal(ap2, ap)
        _check_properties(nxt, w)
        ext = []
        for i, b in enumerate(pick):
            k = int(want["n_nodes"][i])
            L, path, bonus = oracle.accept(want["tokens"][i, :k], want["parents"][i, :k], tgt[b])
            new = np.array([int(want["tokens"][i, j]) for j in path] + [int(bonus)], np.int32)
            ext.append(np.concatenate([contexts[b], new]))
        tg2 = parity.oracle_global_trie(docs, w.D, w.vocab, ext, w.P)
        want2 = parity.oracle_speculate_batch(tg2, ext, w.D, w.P, w.alpha, w.min_score, w.max_nodes)
        bad = parity.compare_trees({k: v[pick] for k, v in nxt.items()}, want2, name + " next drafts")
        assert not bad, "\n".join(bad)
        st = g.stats()
        assert st["err_bad_token"] == 0 and st["err_bad_slot"] == 0 and st["err_ctx_overflow"] == 0
        return got, want
    finally:
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


def test_agentic_full():
    got, want = _run_full("agentic", sample=64)
    assert (got["n_nodes"] > 0).mean() > 0.5


def test_large_full_sampled():
    got, want = _run_full("large", sample=24)
    assert (got["n_nodes"] > 0).mean() > 0.5 and got["n_nodes"].max() > 32


def test_lowrep_full_sampled():
    got, want = _run_full("lowrep", sample=24)
    assert (got["n_nodes"] > 0).mean() > 0.3


def test_streaming_full_sampled_decode_loop():
    """100M-token corpus, 512 requests, decode steps with the simulated verifier: speculate,
    accept, append.  Every step the sampled requests are compared with the oracle (global trie
    restricted to the suffixes those requests can reach, per-request tries extended online);
    invariants are checked for the whole batch."""
    w = make_workload("streaming", seed=0)
    docs = w.docs()
    B, mn, steps = w.batch, w.max_nodes, 6
    contexts = [w.contexts[b].copy() for b in range(B)]
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, w.ctx_len + steps * (mn + 1),
                       len(w.corpus) + len(docs))
    try:
        g.build_global(docs)
        g.build_requests(range(B), contexts)
        rng = np.random.default_rng(2)
        pick = sorted(rng.choice(B, size=8, replace=False).tolist())
        # first tokens the sampled requests can ask about over all steps: context tail + futures
        reach = [np.concatenate([contexts[b][-w.P:], w.future[b, :steps * (mn + 1)]]) for b in pick]
        allowed = np.zeros(w.vocab, np.uint8)
        for r in reach:
            allowed[r] = 1
        tg = oracle.Trie(w.D)
        for d in docs:
            tg.add_doc(d, allowed)
        tries = {}
        for b in pick:
            tries[b] = oracle.Trie(w.D)
            tries[b].append(contexts[b])
        pos = np.zeros(B, np.int64)
        accepted = 0
        got_next = None
        for step in range(steps):
            got = got_next if got_next is not None else g.speculate(range(B))
            got_next = None
            _check_properties(got, w)
            sub = [contexts[b] for b in pick]
            want = parity.oracle_speculate_batch(tg, sub, w.D, w.P, w.alpha, w.min_score, mn,
                                                 request_tries=[tries[b] for b in pick])
            bad = parity.compare_trees({k: v[pick] for k, v in got.items()}, want,
                                       "streaming step %d" % step)
            assert not bad, "\n".join(bad)
            fut = np.stack([w.future[b, pos[b]:pos[b] + mn + 2] for b in range(B)])
            tgt = parity.targets_from_future(got, fut, mn)
            # the three ways to end a step take turns: separate accept and append; both in one
            # launch; and, as bench.py's step does, both plus the next step's drafts in one launch
            mode = step % 3
            fused = mode != 0
            if mode == 2:
                al, ap, bo, got_next = g.accept_append_speculate(range(B), tgt)
            else:
                al, ap, bo = g.accept_append(range(B), tgt) if fused else g.accept(tgt)
            new = []
            for b in range(B):
                L = int(al[b])
                toks = [int(got["tokens"][b, j]) for j in ap[b, :L]] + [int(bo[b])]
                assert toks == [int(v) for v in w.future[b, pos[b]:pos[b] + L + 1]]
                new.append(np.array(toks, np.int32))
                contexts[b] = np.concatenate([contexts[b], new[-1]])
                pos[b] += L + 1
                accepted += L
            for i, b in enumerate(pick):
                k = int(want["n_nodes"][i])
                L, path, bonus = oracle.accept(want["tokens"][i, :k], want["parents"][i, :k], tgt[b])
                assert al[b] == L and bo[b] == bonus and list(ap[b, :L]) == list(path)
                tries[b].append(new[b])
            if not fused:
                g.append(range(B), new)
        assert accepted > B          # the drafts do get accepted on this workload
        assert g.stats()["err_ctx_overflow"] == 0
    finally:
        g.close()
