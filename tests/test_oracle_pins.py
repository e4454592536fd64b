"""Pins for the CPU oracle: brute-force scans, closed forms, invariants, special cases.
None of these reuse the oracle's own code; see tests/brute.py."""
import math
import os

import numpy as np
import pytest

import oracle
from tests import brute
from workloads import make_workload, scaled


def _rand_docs(rng, vocab, n_docs, lo, hi):
    return [rng.integers(0, vocab, size=int(rng.integers(lo, hi + 1))).astype(np.int32)
            for _ in range(n_docs)]


def _all_substrings(docs, D):
    seen = set()
    for doc in docs:
        doc = [int(v) for v in doc]
        for i in range(len(doc)):
            for k in range(1, min(D, len(doc) - i) + 1):
                seen.add(tuple(doc[i:i + k]))
    return seen


@pytest.mark.parametrize("seed,vocab,D", [(0, 2, 3), (1, 3, 4), (2, 4, 6), (3, 3, 9), (4, 2, 1)])
def test_counts_children_ends_match_brute_force(seed, vocab, D):
    rng = np.random.default_rng(seed)
    docs = _rand_docs(rng, vocab, 5, 1, 30)
    t = oracle.Trie(D)
    for d in docs:
        t.add_doc(d)
    subs = _all_substrings(docs, D)
    # every node of the trie corresponds to exactly one observed substring of length <= D
    assert t.num_nodes - 1 == len(subs)
    for w in subs:
        c, e, k = t.lookup(list(w))
        assert c == brute.count(docs, w)
        assert e == brute.ends(docs, w, D)
        assert t.children(list(w)) == brute.children(docs, list(w), D)
    # strings that do not occur have count 0
    for _ in range(200):
        w = tuple(int(v) for v in rng.integers(0, vocab + 1, size=int(rng.integers(1, D + 1))))
        if w not in subs:
            assert t.lookup(list(w)) == (0, 0, 0)


def test_trie_invariants_tiny(tiny_workload):
    w = tiny_workload
    t = oracle.Trie(w.D)
    for d in w.docs():
        t.add_doc(d)
    n = t.dump()
    count, ends, parent, depth = n["count"], n["ends"], n["parent"], n["depth"]
    # COUNT(v) = sum of children's COUNT + suffixes that stop at v
    child_sum = np.zeros_like(count, dtype=np.int64)
    np.add.at(child_sum, parent[1:], count[1:])
    assert np.array_equal(child_sum[1:] + ends[1:], count[1:].astype(np.int64))
    # depth-d nodes together count the positions that have at least d tokens left
    lens = np.diff(w.doc_offsets)
    for d in range(1, w.D + 1):
        assert count[depth == d].sum() == np.maximum(lens - d + 1, 0).sum()
    assert count[depth == 1].sum() == w.corpus.shape[0]
    # a child never occurs more often than its parent; depth never exceeds D
    nz = parent[1:] != 0
    assert np.all(count[1:][nz] <= count[parent[1:][nz]])
    assert depth.max() == w.D
    assert ends.sum() == w.corpus.shape[0]


def _canon(t):
    """Trie as {path tuple: (count, ends)} independent of node numbering."""
    n = t.dump()
    paths = {0: ()}
    out = {}
    order = np.argsort(n["depth"], kind="stable")
    for i in order:
        if i == 0:
            continue
        paths[int(i)] = paths[int(n["parent"][i])] + (int(n["token"][i]),)
        out[paths[int(i)]] = (int(n["count"][i]), int(n["ends"][i]))
    return out


@pytest.mark.parametrize("seed,vocab,D,n", [(0, 2, 4, 40), (1, 3, 5, 80), (2, 50, 8, 200),
                                            (3, 2, 1, 10), (4, 3, 12, 7)])
def test_append_equals_rebuild(seed, vocab, D, n):
    rng = np.random.default_rng(seed)
    seq = rng.integers(0, vocab, size=n).astype(np.int32)
    inc = oracle.Trie(D)
    i = 0
    while i < n:
        k = int(rng.integers(1, 6))
        inc.append(seq[i:i + k])
        i += k
        ref = oracle.Trie(D)
        ref.add_doc(seq[:i])
        assert _canon(inc) == _canon(ref)


def test_filtered_trie_equals_full_below_allowed_tokens(tiny_workload):
    w = tiny_workload
    full = oracle.Trie(w.D)
    allowed = np.zeros(w.vocab, np.uint8)
    firsts = np.unique(w.contexts[:, -w.P:])
    allowed[firsts] = 1
    filt = oracle.Trie(w.D)
    for d in w.docs():
        full.add_doc(d)
        filt.add_doc(d, allowed)
    assert filt.num_nodes < full.num_nodes
    cf, cl = _canon(full), _canon(filt)
    assert cl == {k: v for k, v in cf.items() if allowed[k[0]]}


@pytest.mark.parametrize("den_mode", [0, 1])
@pytest.mark.parametrize("seed,vocab,D,P,alpha,ms", [
    (0, 2, 6, 3, 2.0, 0.05), (1, 3, 8, 4, 1.0, 0.1), (2, 4, 10, 5, 3.0, 0.0),
    (3, 3, 5, 4, 1.5, 0.3), (4, 2, 12, 6, 4.0, 0.01), (5, 6, 7, 3, 2.5, 0.2)])
def test_speculation_matches_trie_free_speculator(seed, vocab, D, P, alpha, ms, den_mode):
    rng = np.random.default_rng(100 + seed)
    docs = _rand_docs(rng, vocab, 4, 5, 40)
    tg = oracle.Trie(D)
    for d in docs:
        tg.add_doc(d)
    for q in range(6):
        x = rng.integers(0, vocab, size=int(rng.integers(1, 25))).astype(np.int32)
        tr = oracle.Trie(D)
        tr.append(x)
        for p in range(1, P + 1):
            for trie, coll in ((tg, docs), (tr, [x])):
                got = oracle.speculate_unit(trie, x, p, alpha, ms, den_mode)
                want = brute.speculate_unit(coll, x, p, alpha, ms, D, den_mode)
                if want is None:
                    assert got is None
                    continue
                assert list(got[0]) == want[0]
                assert list(got[1]) == want[1]
                assert [float(s).hex() for s in got[2]] == [float(s).hex() for s in want[2]]
                assert float(got[3]).hex() == float(want[3]).hex()
        got = oracle.generate(tg, tr, x, P, alpha, ms, den_mode)
        want = brute.generate(docs, x, P, alpha, ms, D, den_mode)
        assert list(got["tokens"]) == want["tokens"]
        assert list(got["parents"]) == want["parents"]
        assert got["match_len"] == want["match_len"] and got["source"] == want["source"]
        assert float(got["tree_score"]).hex() == float(want["tree_score"]).hex()


def _node_paths(root, tokens, parents):
    paths = []
    for j in range(len(tokens)):
        base = root if parents[j] < 0 else paths[parents[j]]
        paths.append(base + [int(tokens[j])])
    return paths


def test_scores_closed_form_structure_and_topk(tiny_workload):
    """Under the default denominator the product of ratios telescopes to
    COUNT(N)/COUNT(N_p); trees obey the size cap and ordering rules; the selected counts are
    the K largest among admissible nodes below N_p."""
    w = tiny_workload
    docs = w.docs()
    tg = oracle.Trie(w.D)
    for d in docs:
        tg.add_doc(d)
    n_checked = 0
    for r in range(w.batch):
        x = w.contexts[r]
        for p in range(1, w.P + 1):
            got = oracle.speculate_unit(tg, x, p, w.alpha, w.min_score)
            if got is None:
                continue
            tok, par, sc, total = got
            K = int(math.floor(w.alpha * p))
            assert len(tok) <= K
            root = [int(v) for v in x[-p:]]
            c_root = tg.lookup(root)[0]
            paths = _node_paths(root, tok, par)
            s = 0.0
            for j in range(len(tok)):
                assert par[j] < j and par[j] >= -1
                c = tg.lookup(paths[j])[0]
                assert c > 0
                exact = c / c_root
                assert abs(sc[j] - exact) <= 64 * 2.0 ** -53 * exact
                assert sc[j] >= w.min_score and 0.0 < sc[j] <= 1.0
                if par[j] >= 0:
                    assert sc[j] <= sc[par[j]]
                if j > 0:
                    assert sc[j] <= sc[j - 1]
                assert len(paths[j]) <= w.D
                s += sc[j]
            assert s == total
            # siblings carry distinct tokens
            assert len({(int(par[j]), int(tok[j])) for j in range(len(tok))}) == len(tok)
            # top-K property on counts: enumerate all admissible descendants by scanning
            if len(tok) and p >= 2:
                sel = sorted((tg.lookup(q)[0] for q in paths), reverse=True)
                # `sure`: nodes clearly at or above min_score; `maybe`: those plus the ones
                # within 1e-9 of it, on which rounding may decide either way (fewest
                # occurrences of all, so they sort last)
                sure, maybe = [], []
                stack = [root]
                while stack:
                    cur = stack.pop()
                    for t_, c_ in brute.children(docs, cur, w.D).items():
                        if c_ / c_root >= w.min_score * (1 - 1e-9):
                            maybe.append(c_)
                            stack.append(cur + [t_])
                            if c_ / c_root >= w.min_score * (1 + 1e-9):
                                sure.append(c_)
                maybe.sort(reverse=True)
                assert sel == maybe[:len(sel)]
                assert len(sel) >= min(K, len(sure))
                n_checked += 1
    assert n_checked > 20


def test_periodic_document_gives_chain():
    """One document that repeats a period-q block: every continuation is forced, so the tree
    is the chain that continues the period, min(K, D-p) long, with hand-computable scores."""
    q, reps, D = 5, 8, 12
    block = [7, 3, 9, 1, 4]
    doc = np.array(block * reps, np.int32)          # 40 tokens
    t = oracle.Trie(D)
    t.add_doc(doc)
    x = np.array([11, 12] + block + [7, 3], np.int32)  # ends "... 4 7 3"
    for p, alpha in ((2, 2.0), (3, 5.0), (7, 1.0)):
        tok, par, sc, total = oracle.speculate_unit(t, x, p, alpha, 0.0)
        K = int(alpha * p)
        n = min(K, D - p)
        assert len(tok) == n
        want = [block[(2 + i) % q] for i in range(n)]     # after "... 7 3" comes 9 1 4 7 3 ...
        assert list(tok) == want
        assert list(par) == list(range(-1, n - 1))
        # occurrences of a string of length L starting at phase f: number of starts i == f mod 5
        # with i + L <= 40.  Pattern (length p) ends in "7 3": it starts at phase (2 - p) mod 5.
        f = (2 - p) % q
        def occ(L):
            return len([i for i in range(f, 40, q) if i + L <= 40])
        for i in range(n):
            assert sc[i] == pytest.approx(occ(p + i + 1) / occ(p), rel=1e-15)
    # pattern "12 7 3 9 1 4 7 3" (p=8) does not occur
    assert oracle.speculate_unit(t, x, 8, 1.0, 0.0) is None


def test_no_repeats_and_short_context():
    doc = np.arange(100, dtype=np.int32)
    t = oracle.Trie(8)
    t.add_doc(doc)
    x = np.array([500, 501, 502], np.int32)      # tokens absent from the corpus
    tr = oracle.Trie(8)
    tr.append(x)
    g = oracle.generate(t, tr, x, 4, 2.0, 0.1)
    assert g["n_nodes"] == 0 and g["source"] == -1 and g["match_len"] == 0 and g["tree_score"] == 0
    # p larger than the context never matches
    assert oracle.speculate_unit(tr, x, 4, 1.0, 0.1) is None
    # the request structure always contains its own suffix but has nothing after it
    got = oracle.speculate_unit(tr, x, 2, 1.0, 0.1)
    assert got is not None and len(got[0]) == 0
    # a context that continues a corpus run drafts that run
    x2 = np.array([10, 11, 12], np.int32)
    tok, par, sc, total = oracle.speculate_unit(t, x2, 3, 2.0, 0.1)
    assert list(tok) == [13, 14, 15, 16, 17] and list(par) == [-1, 0, 1, 2, 3]   # D - p = 5
    assert total == 5.0


def test_hand_worked_golden_example():
    """tests/golden/worked_example.txt: a 3-document corpus small enough to count by eye."""
    path = os.path.join(os.path.dirname(__file__), "golden", "worked_example.txt")
    sect = {}
    cur = None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            cur = line.strip("[]")
            sect[cur] = []
        else:
            sect[cur].append(line)
    D = int(sect["D"][0])
    docs = [np.array(l.split(), np.int32) for l in sect["docs"]]
    x = np.array(sect["context"][0].split(), np.int32)
    t = oracle.Trie(D)
    for d in docs:
        t.add_doc(d)
    for line in sect["counts"]:
        lhs, rhs = line.split("=")
        c, e = (int(v) for v in rhs.split())
        assert t.lookup([int(v) for v in lhs.split()])[:2] == (c, e), line
    for line in sect["units"]:
        # p alpha min_score den_mode | tokens | parents | scores as fractions | tree score
        head, toks, pars, scs, tot = [s.strip() for s in line.split("|")]
        p, alpha, ms, dm = head.split()
        got = oracle.speculate_unit(t, x, int(p), float(alpha), float(ms), int(dm))
        assert list(got[0]) == [int(v) for v in toks.split()], line
        assert list(got[1]) == [int(v) for v in pars.split()], line
        fr = [float(a) / float(b) for a, b in (v.split("/") for v in scs.split())]
        assert np.allclose(got[2], fr, rtol=1e-15, atol=0), line
        a, b = tot.split("/")
        assert got[3] == pytest.approx(float(a) / float(b), rel=1e-15), line


def test_select_is_strict_greater_scan(tiny_workload):
    w = tiny_workload
    tg = oracle.Trie(w.D)
    for d in w.docs():
        tg.add_doc(d)
    n_nonempty = 0
    for r in range(w.batch):
        x = w.contexts[r]
        tr = oracle.Trie(w.D)
        tr.append(x)
        g = oracle.generate(tg, tr, x, w.P, w.alpha, w.min_score)
        best, bp, bs, bt = 0.0, 0, -1, None
        for s, trie in enumerate((tg, tr)):
            for p in range(1, w.P + 1):
                u = oracle.speculate_unit(trie, x, p, w.alpha, w.min_score)
                if u is not None and u[3] > best:
                    best, bp, bs, bt = u[3], p, s, u
        assert g["tree_score"] == best and g["match_len"] == bp and g["source"] == bs
        if bt is not None:
            assert list(g["tokens"]) == list(bt[0]) and list(g["parents"]) == list(bt[1])
            assert g["n_nodes"] <= math.floor(w.alpha * bp) <= w.max_nodes
            n_nonempty += 1
    assert n_nonempty >= w.batch // 2


def test_accept_matches_path_enumeration(tiny_workload):
    w = tiny_workload
    rng = np.random.default_rng(7)
    tg = oracle.Trie(w.D)
    for d in w.docs():
        tg.add_doc(d)
    hits = 0
    for r in range(w.batch):
        x = w.contexts[r]
        g = oracle.generate(tg, None, x, w.P, 2.0, 0.02)
        tok, par = g["tokens"], g["parents"]
        n = len(tok)
        depth = np.zeros(n, np.int64)
        for j in range(n):
            depth[j] = 1 if par[j] < 0 else depth[par[j]] + 1
        for trial in range(4):
            target = np.empty(n + 1, np.int32)
            target[0] = w.future[r, 0]
            target[1:] = w.future[r, depth]
            if trial:                       # perturbed targets exercise early stops and branches
                k = rng.integers(0, n + 1, size=3)
                target[k] = rng.integers(0, w.vocab, size=3)
                if n:
                    target[0] = tok[rng.integers(0, n)]
            L, path, bonus = oracle.accept(tok, par, target)
            L2, path2, bonus2 = brute.accept_by_enumeration(list(tok), list(par), list(target))
            assert (L, list(path), bonus) == (L2, path2, bonus2)
            hits += L > 0
            # with the unperturbed target the accepted path is the longest prefix of the future
            if trial == 0 and L:
                assert [int(tok[j]) for j in path] == [int(v) for v in w.future[r, :L]]
    assert hits > 0
    # empty tree
    L, path, bonus = oracle.accept(np.zeros(0, np.int32), np.zeros(0, np.int32),
                                   np.array([5], np.int32))
    assert L == 0 and len(path) == 0 and bonus == 5


def test_planted_mistakes_are_caught():
    """The pins must fail for plausible mistakes.  Each variant below is the brute-force
    speculator with one planted error; it must disagree with the oracle somewhere."""
    rng = np.random.default_rng(5)
    docs = _rand_docs(rng, 3, 4, 10, 40)
    D, P, alpha, ms = 7, 4, 2.0, 0.1
    tg = oracle.Trie(D)
    for d in docs:
        tg.add_doc(d)

    def run(fn):
        bad = 0
        r2 = np.random.default_rng(9)
        for _ in range(30):
            x = r2.integers(0, 3, size=12).astype(np.int32)
            for p in range(1, P + 1):
                got = oracle.speculate_unit(tg, x, p, alpha, ms)
                want = fn(docs, x, p)
                if (got is None) != (want is None):
                    bad += 1
                elif got is not None and (list(got[0]) != want[0] or list(got[1]) != want[1] or
                                          list(got[2]) != want[2]):
                    bad += 1
        return bad

    assert run(lambda d, x, p: brute.speculate_unit(d, x, p, alpha, ms, D)) == 0
    # wrong depth bound, wrong cap, wrong threshold, wrong denominator
    assert run(lambda d, x, p: brute.speculate_unit(d, x, p, alpha, ms, D + 1)) > 0
    assert run(lambda d, x, p: brute.speculate_unit(d, x, p, alpha + 1, ms, D)) > 0
    assert run(lambda d, x, p: brute.speculate_unit(d, x, p, alpha, ms * 2, D)) > 0
    assert run(lambda d, x, p: brute.speculate_unit(d, x, p, alpha, ms, D, 1)) > 0
    # pattern taken from the wrong end of the context
    assert run(lambda d, x, p: brute.speculate_unit(d, x[::-1], p, alpha, ms, D)) > 0


@pytest.mark.parametrize("den_mode", [0, 1])
@pytest.mark.parametrize("seed,vocab,D,P,alpha,ms", [
    (0, 2, 6, 3, 2.0, 0.05), (1, 3, 8, 4, 1.0, 0.1), (2, 4, 10, 5, 3.0, 0.0), (3, 3, 5, 4, 1.5, 0.3)])
def test_linear_variant_matches_trie_free_speculator(seed, vocab, D, P, alpha, ms, den_mode):
    rng = np.random.default_rng(200 + seed)
    docs = _rand_docs(rng, vocab, 4, 5, 40)
    tg = oracle.Trie(D)
    for d in docs:
        tg.add_doc(d)
    differs = 0
    for q in range(6):
        x = rng.integers(0, vocab, size=int(rng.integers(1, 25))).astype(np.int32)
        tr = oracle.Trie(D)
        tr.append(x)
        for p in range(1, P + 1):
            for trie, coll in ((tg, docs), (tr, [x])):
                got = oracle.speculate_unit(trie, x, p, alpha, ms, den_mode, 1)
                want = brute.speculate_unit(coll, x, p, alpha, ms, D, den_mode, 1)
                if want is None:
                    assert got is None
                    continue
                assert list(got[0]) == want[0] and list(got[1]) == want[1]
                assert [float(s).hex() for s in got[2]] == [float(s).hex() for s in want[2]]
                # a chain: every node hangs off the previous one
                assert list(got[1]) == list(range(-1, len(got[0]) - 1))
                tree = oracle.speculate_unit(trie, x, p, alpha, ms, den_mode, 0)
                differs += list(tree[1]) != list(got[1])
        got = oracle.generate(tg, tr, x, P, alpha, ms, den_mode, 1)
        want = brute.generate(docs, x, P, alpha, ms, D, den_mode, 1)
        assert list(got["tokens"]) == want["tokens"] and got["match_len"] == want["match_len"]
        assert got["source"] == want["source"]
        assert float(got["tree_score"]).hex() == float(want["tree_score"]).hex()
    assert differs > 0      # the tree variant does branch on these inputs


def test_linear_variant_follows_the_most_frequent_child(tiny_workload):
    """Closed form for the chain variant: at every step the next token is the most frequent
    continuation of the path so far (ties to the lower token)."""
    w = tiny_workload
    docs = w.docs()
    tg = oracle.Trie(w.D)
    for d in docs:
        tg.add_doc(d)
    seen = 0
    for r in range(w.batch):
        x = w.contexts[r]
        for p in (1, 2, 3, 5, 8):
            got = oracle.speculate_unit(tg, x, p, 2.0, 0.1, 0, 1)
            if got is None:
                continue
            path = [int(v) for v in x[-p:]]
            c_root = tg.lookup(path)[0]
            for j in range(len(got[0])):
                ch = tg.children(path)
                top = max(ch.values())
                best_tok = min(t_ for t_, c_ in ch.items() if c_ == top)
                assert int(got[0][j]) == best_tok
                path.append(best_tok)
                assert got[2][j] == pytest.approx(tg.lookup(path)[0] / c_root, rel=1e-14)
                seen += 1
    assert seen > 30


# ---- empirical entropy (Appendix, "Predicting SuffixDecoding Effectiveness") -------------------
@pytest.mark.parametrize("seed,vocab,D,n_docs", [(0, 2, 3, 3), (1, 3, 5, 4), (2, 5, 8, 6), (3, 4, 1, 3),
                                                 (4, 50, 6, 5)])
def test_entropy_matches_brute_force(seed, vocab, D, n_docs):
    rng = np.random.default_rng(100 + seed)
    docs = _rand_docs(rng, vocab, n_docs, 1, 40)
    docs.append(np.zeros(0, np.int32))
    t = oracle.Trie(D)
    for d in docs:
        t.add_doc(d)
    h, w = t.entropy()
    hb, wb = brute.entropy(docs, D)
    assert w == wb
    assert h == pytest.approx(hb, rel=1e-12, abs=1e-15)


def test_entropy_closed_forms():
    # all tokens distinct: only the root is uncertain (n equally likely first tokens); every
    # other node has one child.  weight = number of (context, next token) observations
    n, D = 37, 6
    t = oracle.Trie(D)
    t.add_doc(np.arange(n, dtype=np.int32))
    h, w = t.entropy()
    weight = sum(n - k for k in range(D))            # contexts of length k = 0..D-1
    assert w == weight
    assert h == pytest.approx(n * math.log2(n) / weight, rel=1e-13)
    # a periodic document: after one token everything is determined
    q, reps, D = 5, 9, 4
    t = oracle.Trie(D)
    t.add_doc(np.tile(np.arange(q, dtype=np.int32), reps))
    h, w = t.entropy()
    n = q * reps
    assert w == sum(n - k for k in range(D))
    assert h == pytest.approx(n * math.log2(q) / w, rel=1e-13)
    # two equally likely continuations after every context of length 1 .. D-1 built by hand:
    # documents "a b" and "a c", D = 2: root sees a (x2), b, c; node a sees b, c
    t = oracle.Trie(2)
    t.add_doc(np.array([0, 1], np.int32))
    t.add_doc(np.array([0, 2], np.int32))
    h, w = t.entropy()
    root = 4 * (-(0.5 * math.log2(0.5) + 2 * 0.25 * math.log2(0.25)))   # weight 4, H = 1.5
    node_a = 2 * 1.0                                                     # weight 2, H = 1
    assert w == 6 and h == pytest.approx((root + node_a) / 6, rel=1e-14)
    # nothing to predict: empty corpus and single-token documents with D = 1 (root only)
    assert oracle.Trie(3).entropy() == (0.0, 0.0)


def test_entropy_orders_structured_below_random(tiny_workload):
    """The use the paper makes of it: repetitive text scores lower than random text."""
    w = tiny_workload
    t = oracle.Trie(w.D)
    for d in w.docs()[:10]:
        t.add_doc(d)
    rng = np.random.default_rng(0)
    r = oracle.Trie(w.D)
    for d in w.docs()[:10]:
        r.add_doc(rng.integers(0, 64, len(d)).astype(np.int32))
    z = oracle.Trie(w.D)
    for d in w.docs()[:10]:
        z.add_doc(rng.integers(0, w.vocab, len(d)).astype(np.int32))
    assert t.entropy()[0] < r.entropy()[0]
    assert t.entropy()[0] < z.entropy()[0]
