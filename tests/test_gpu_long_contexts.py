"""GPU parity on contexts whose last token occurs thousands of times: the per-request side of
MatchPattern then has occurrence lists too long for the in-LDS sort (they are sorted in device
memory by the whole workgroup), suffix lists of many pattern lengths that are written to the
request's scratch row, and, when those do not fit the row together, several rounds of lists.
The counters of sd_get_stats say which of these routes the kernel took."""
import numpy as np
import pytest

import oracle
from tests import parity

pytestmark = pytest.mark.gpu


def _cases():
    rng = np.random.default_rng(31)
    out = {}
    # name -> (vocab, D, P, alpha, min_score, docs, contexts)
    doc2 = rng.integers(0, 2, 4000)
    out["binary-3000"] = (2, 12, 6, 4.0, 0.02, [doc2], [rng.integers(0, 2, 3000), rng.integers(0, 2, 2900)])
    out["binary-6000"] = (2, 12, 6, 4.0, 0.02, [doc2], [rng.integers(0, 2, 6000), rng.integers(0, 2, 5000),
                                                       rng.integers(0, 2, 700)])
    doc3 = rng.integers(0, 3, 3000)
    out["ternary-6000"] = (3, 10, 5, 3.0, 0.03, [doc3, doc3[100:900]],
                           [rng.integers(0, 3, 6000), rng.integers(0, 3, 6100)])
    # four tokens in five are the same one: every pattern length has a long list, and together
    # they exceed the scratch row several times over
    def biased(n):
        x = (rng.random(n) < 0.8).astype(np.int64)
        x[-1] = 1           # the context ends with the frequent token
        return x

    out["biased-binary-6000"] = (2, 20, 10, 2.0, 0.02, [biased(3000)], [biased(6000), biased(4500)])
    # one repeated token: the list of pattern length p holds all but p - 1 of the positions
    out["one-token-5000"] = (3, 16, 8, 2.0, 0.05, [[1] * 300, [1, 1, 2, 1, 1, 1, 0]],
                             [[1] * 5000, [1] * 2049, [2] + [1] * 2500, [1] * 70])
    return out


CASES = _cases()


def _future(rng, vocab, B, n):
    return rng.integers(0, vocab, (B, n)).astype(np.int32)


@pytest.mark.parametrize("den_mode", [0, 1])
@pytest.mark.parametrize("name", list(CASES))
def test_long_occurrence_lists(name, den_mode):
    vocab, D, P, alpha, ms, docs, contexts = CASES[name]
    docs = [np.asarray(d, np.int32) for d in docs]
    contexts = [np.asarray(c, np.int32) for c in contexts]
    B = len(contexts)
    longest = max(len(c) for c in contexts)
    mn = int(np.floor(alpha * P))
    g = parity.GpuPath(vocab, D, P, alpha, ms, B, longest + mn + 1, sum(len(d) for d in docs) + len(docs),
                       den_mode=den_mode)
    try:
        g.build_global(docs)
        g.build_requests(range(B), contexts)
        st0 = g.stats()
        got = g.speculate(range(B))
        tg = parity.oracle_global_trie(docs, D, vocab)
        tries = []
        for x in contexts:
            tr = oracle.Trie(D)
            tr.append(x)
            tries.append(tr)
        want = parity.oracle_speculate_batch(tg, contexts, D, P, alpha, ms, mn, request_tries=tries,
                                             den_mode=den_mode)
        bad = parity.compare_trees(got, want, name)
        assert not bad, "\n".join(bad)
        st1 = g.stats()
        assert st1["spec_requests"] - st0["spec_requests"] == B
        assert st1["spec_request_wide"] - st0["spec_request_wide"] >= 1
        # more occurrences of the last token than the in-LDS sort takes (2048 records)
        if max(int(np.sum(c == c[-1])) for c in contexts) > 2048:
            assert st1["spec_occ_in_memory"] - st0["spec_occ_in_memory"] >= 1
        if name in ("biased-binary-6000", "one-token-5000"):
            assert st1["spec_list_rounds"] - st0["spec_list_rounds"] >= 2
        # the end of the step and the next drafts in one launch, on the extended contexts
        rng = np.random.default_rng(7)
        fut = _future(rng, vocab, B, mn + 2)
        # let the verifier agree with the first draft token of every other request
        for b in range(0, B, 2):
            if want["n_nodes"][b] > 0:
                fut[b, 0] = want["tokens"][b, 0]
        tgt = parity.targets_from_future(want, fut, mn)
        al, ap, bo, nxt = g.accept_append_speculate(range(B), tgt)
        ext = []
        for b in range(B):
            k = int(want["n_nodes"][b])
            L, path, bonus = oracle.accept(want["tokens"][b, :k], want["parents"][b, :k], tgt[b])
            assert al[b] == L and bo[b] == bonus and list(ap[b, :L]) == list(path)
            new = np.array([int(want["tokens"][b, j]) for j in path] + [int(bonus)], np.int32)
            tries[b].append(new)
            ext.append(np.concatenate([contexts[b], new]))
        want2 = parity.oracle_speculate_batch(tg, ext, D, P, alpha, ms, mn, request_tries=tries,
                                              den_mode=den_mode)
        bad = parity.compare_trees(nxt, want2, name + " next drafts")
        assert not bad, "\n".join(bad)
        st = g.stats()
        assert st["err_bad_token"] == 0 and st["err_bad_slot"] == 0 and st["err_ctx_overflow"] == 0
    finally:
        g.close()


def test_long_lists_on_thin_workgroups():
    """The same long contexts in a batch of several workgroups per compute unit: thinner
    workgroups have less LDS for the occurrence sort (it goes to device memory from 1024
    records on) and fewer waves to share the rounds of lists."""
    rng = np.random.default_rng(41)
    vocab, D, P, alpha, ms = 2, 12, 6, 2.0, 0.02
    docs = [rng.integers(0, 2, 3000).astype(np.int32)]
    distinct = [rng.integers(0, 2, n).astype(np.int32) for n in (2500, 1900, 3000, 60)]
    distinct.append((rng.random(3000) < 0.85).astype(np.int32))
    distinct[-1][-1] = 1
    B = 1300
    contexts = [distinct[b % len(distinct)] for b in range(B)]
    mn = int(np.floor(alpha * P))
    g = parity.GpuPath(vocab, D, P, alpha, ms, B, 3000 + mn + 1, sum(len(d) for d in docs) + len(docs))
    try:
        g.build_global(docs)
        g.build_requests(range(B), contexts)
        got = g.speculate(range(B))
        tg = parity.oracle_global_trie(docs, D, vocab)
        want_d = parity.oracle_speculate_batch(tg, distinct, D, P, alpha, ms, mn)
        want = {k: v[np.arange(B) % len(distinct)] for k, v in want_d.items()}
        bad = parity.compare_trees(got, want, "thin workgroups")
        assert not bad, "\n".join(bad)
        st = g.stats()
        assert st["spec_occ_in_memory"] >= B // len(distinct)
        assert st["spec_list_rounds"] >= 1
    finally:
        g.close()


@pytest.mark.parametrize("B", [5, 700, 2600])
def test_frequent_last_token_in_the_fused_step(B):
    """The decode step's kernel with last tokens that occur some hundred times in their contexts
    and a global index that sends every pattern length on a search of its own: the waves that
    are done with their searches first take the occurrences in parts of 64 before the barrier.
    One workgroup per compute unit (16 waves) and several (8 to 4 waves), where a part of the
    lists is too long for that route and takes the other one."""
    rng = np.random.default_rng(43 + B)
    vocab, D, P, alpha, ms = 6, 20, 8, 2.0, 0.02
    docs = [rng.integers(0, vocab, 4000).astype(np.int32) for _ in range(3)]
    lens = (70, 300, 700, 1200, 2000)
    distinct = [rng.integers(0, vocab, n).astype(np.int32) for n in lens]
    contexts = [distinct[b % len(distinct)] for b in range(B)]
    mn = int(np.floor(alpha * P))
    g = parity.GpuPath(vocab, D, P, alpha, ms, B, max(lens) + mn + 1,
                       sum(len(d) for d in docs) + len(docs))
    try:
        g.build_global(docs)
        g.build_requests(range(B), contexts)
        st0 = g.stats()
        got = g.speculate(range(B))
        tg = parity.oracle_global_trie(docs, D, vocab)
        tries = []
        for x in distinct:
            tr = oracle.Trie(D)
            tr.append(x)
            tries.append(tr)
        want_d = parity.oracle_speculate_batch(tg, distinct, D, P, alpha, ms, mn, request_tries=tries)
        pick = np.arange(B) % len(distinct)
        want = {k: v[pick] for k, v in want_d.items()}
        bad = parity.compare_trees(got, want, "frequent last token, first drafts")
        assert not bad, "\n".join(bad)
        st1 = g.stats()
        assert st1["spec_global_search"] - st0["spec_global_search"] == B   # no list form here
        fut = rng.integers(0, vocab, (len(distinct), mn + 2)).astype(np.int32)
        for d in range(0, len(distinct), 2):     # the verifier agrees with some first draft tokens
            if want_d["n_nodes"][d] > 0:
                fut[d, 0] = want_d["tokens"][d, 0]
        tgt_d = parity.targets_from_future(want_d, fut, mn)
        al, ap, bo, nxt = g.accept_append_speculate(range(B), tgt_d[pick])
        ext = []
        for d in range(len(distinct)):
            k = int(want_d["n_nodes"][d])
            L, path, bonus = oracle.accept(want_d["tokens"][d, :k], want_d["parents"][d, :k], tgt_d[d])
            assert np.all(al[pick == d] == L) and np.all(bo[pick == d] == bonus)
            new = np.array([int(want_d["tokens"][d, j]) for j in path] + [int(bonus)], np.int32)
            tries[d].append(new)
            ext.append(np.concatenate([distinct[d], new]))
        want2_d = parity.oracle_speculate_batch(tg, ext, D, P, alpha, ms, mn, request_tries=tries)
        want2 = {k: v[pick] for k, v in want2_d.items()}
        bad = parity.compare_trees(nxt, want2, "frequent last token, next drafts")
        assert not bad, "\n".join(bad)
        # the lists are of the lengths meant: from a dozen to some hundred occurrences
        occ = [int(np.sum(x == x[-1])) for x in ext]
        assert min(occ) < 64 and max(occ) > 256, occ
        st = g.stats()
        assert st["err_bad_token"] == 0 and st["err_bad_slot"] == 0 and st["err_ctx_overflow"] == 0
    finally:
        g.close()
