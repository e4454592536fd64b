"""Oracle work of the full-size parity tests, done in worker processes while the test's own
process drives the GPU.  Test infrastructure: a worker imports the oracle and the seeded input
generators only (never the HIP library), regenerates the workload from (name, seed) and
returns plain numpy arrays.

Every job restricts the oracle's global trie to the suffixes its requests can reach (first
token among the last P context tokens, see oracle.Trie.add_doc); when contexts grow, the
suffixes that start with tokens not seen before are added by a further pass over the
documents, which gives the same trie as building it for the larger set at once (insertion of
a suffix depends on nothing but its own first token)."""
from __future__ import annotations

import concurrent.futures as cf
import multiprocessing as mp
import os

import numpy as np

MAX_WORKERS = 12    # the GPU machine gives one GPU's job about 16 cores, whatever os.cpu_count() says


def pool(n_jobs: int, cap: int = MAX_WORKERS):
    """An executor of spawned workers (never forked: the parent may hold a GPU context).  A
    worker that dies breaks the executor with an error instead of being started again."""
    n = max(1, min(n_jobs, cap, MAX_WORKERS, max(1, (os.cpu_count() or 2) - 1)))
    return cf.ProcessPoolExecutor(max_workers=n, mp_context=mp.get_context("spawn"))


class _GlobalTrie:
    """The oracle's global trie over `docs`, holding the suffixes whose first token has been
    asked for so far."""

    def __init__(self, docs, D, vocab):
        import oracle
        self.docs, self.vocab = docs, vocab
        self.have = np.zeros(vocab, np.uint8)
        self.trie = oracle.Trie(D)

    def cover(self, tokens):
        need = np.zeros(self.vocab, np.uint8)
        need[np.asarray(tokens, np.int64)] = 1
        need &= ~self.have & 1
        if need.any():
            for d in self.docs:
                if len(d):
                    self.trie.add_doc(d, need)
            self.have |= need


def _pack(rows, mn):
    """List of oracle.generate results -> arrays shaped like the library's outputs."""
    B = len(rows)
    out = dict(n_nodes=np.zeros(B, np.int32), tokens=np.full((B, mn), -1, np.int32),
               parents=np.full((B, mn), -1, np.int32), scores=np.zeros((B, mn), np.float64),
               tree_score=np.zeros(B, np.float64), match_len=np.zeros(B, np.int32),
               source=np.full(B, -1, np.int32))
    for b, g in enumerate(rows):
        n = g["n_nodes"]
        out["n_nodes"][b] = n
        out["tokens"][b, :n] = g["tokens"]
        out["parents"][b, :n] = g["parents"]
        out["scores"][b, :n] = g["scores"]
        out["tree_score"][b] = g["tree_score"]
        out["match_len"][b] = g["match_len"]
        out["source"][b] = g["source"]
    return out


def _depths(parents, n):
    d = np.zeros(n, np.int64)
    for j in range(n):
        d[j] = 1 if parents[j] < 0 else d[parents[j]] + 1
    return d


def _targets(g, fut, mn):
    """The simulated greedy verifier (Section 4.1): the target token at a node of depth k is
    fut[k]; fut[0] at the root."""
    tgt = np.full(mn + 1, fut[0], np.int32)
    n = g["n_nodes"]
    tgt[1:1 + n] = fut[_depths(g["parents"], n)]
    return tgt


def decode_steps(name, seed, ids, steps, overrides=None, window=96):
    """The oracle's decode loop for the requests `ids` of workload (name, seed): per step
    GenerateCandidateTree, the simulated verifier on the request's ground-truth future, the
    acceptance walk, and the append of the accepted tokens plus the bonus token.  `overrides`
    maps a request id to a context that replaces the workload's.  steps = 1 gives the first
    drafts and their acceptance.  Returns, per step, the trees (arrays over ids), accept_len,
    bonus and the accepted paths; the trees of step s + 1 are the "next drafts" of step s."""
    import oracle
    from workloads import make_workload
    w = make_workload(name, seed=seed)
    mn = w.max_nodes
    window = max(window, mn + 1)
    docs = w.docs()
    contexts = {b: np.asarray((overrides or {}).get(b, w.contexts[b]), np.int32) for b in ids}
    tg = _GlobalTrie(docs, w.D, w.vocab)
    tries = {}
    for b in ids:
        tries[b] = oracle.Trie(w.D)
        if len(contexts[b]):
            tries[b].append(contexts[b])
    pos = {b: 0 for b in ids}
    covered = {b: 0 for b in ids}      # future tokens of b already asked of the global trie
    tg.cover(np.concatenate([contexts[b][-w.P:] for b in ids]))
    out = []
    for step in range(steps + 1):      # one more drafting pass: the next drafts of the last step
        if step < steps and any(pos[b] + mn + 1 > covered[b] for b in ids):
            # whatever this and the next few steps append comes from the futures
            more = []
            for b in ids:
                end = min(pos[b] + window, w.future.shape[1])
                more.append(w.future[b, covered[b]:end])
                covered[b] = max(covered[b], end)
            tg.cover(np.concatenate(more))
        rows = [oracle.generate(tg.trie, tries[b], contexts[b], w.P, w.alpha, w.min_score) for b in ids]
        rec = dict(trees=_pack(rows, mn))
        if step == steps:
            out.append(rec)
            break
        al, bo, paths = [], [], []
        for b, g in zip(ids, rows):
            fut = w.future[b, pos[b]:pos[b] + mn + 2]
            L, path, bonus = oracle.accept(g["tokens"], g["parents"], _targets(g, fut, mn))
            new = np.array([int(g["tokens"][j]) for j in path] + [int(bonus)], np.int32)
            tries[b].append(new)
            contexts[b] = np.concatenate([contexts[b], new])
            pos[b] += L + 1
            al.append(L)
            bo.append(bonus)
            paths.append(np.asarray(path, np.int32))
        rec.update(accept_len=np.array(al, np.int32), bonus=np.array(bo, np.int32), paths=paths)
        out.append(rec)
    return dict(ids=list(ids), steps=out)


def submit(p, name, seed, chunks, steps, overrides=None, window=96):
    """Starts decode_steps for every chunk of request ids; returns the futures."""
    res = []
    for ids in chunks:
        ov = {b: overrides[b] for b in ids if overrides and b in overrides} or None
        res.append(p.submit(decode_steps, name, seed, list(ids), steps, ov, window))
    return res
