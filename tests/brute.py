"""Brute-force definitions used to pin the oracle.  No trie, no index: every
count comes from scanning the documents, straight from the definitions in
Section 3 of the paper (COUNT = number of occurrences; C, D, SCORE; Algorithm 1)
with the depth bound D and the tie rules stated in the oracle's header.
Pure Python, for tiny inputs only."""
import math
from collections import Counter


def occurrences(docs, w):
    w = list(w)
    k = len(w)
    out = []
    for d, doc in enumerate(docs):
        doc = list(doc)
        for i in range(0, len(doc) - k + 1):
            if doc[i:i + k] == w:
                out.append((d, i))
    return out


def count(docs, w):
    return len(occurrences(docs, w))


def children(docs, w, D):
    """token -> COUNT(w + [token]) for |w| < D."""
    if len(w) >= D:
        return {}
    c = Counter()
    k = len(w)
    for d, i in occurrences(docs, w):
        if i + k < len(docs[d]):
            c[int(docs[d][i + k])] += 1
    return dict(c)


def ends(docs, w, D):
    if len(w) == D:
        return count(docs, w)
    k = len(w)
    return sum(1 for d, i in occurrences(docs, w) if i + k == len(docs[d]))


def speculate_unit(docs, x, p, alpha, min_score, D, den_mode=0, linear=0):
    """Greedy tree for one (collection, p).  Returns None when the last p tokens of x do not
    occur, else (tokens, parents, scores, tree_score)."""
    x = [int(v) for v in x]
    if p < 1 or p > len(x):
        return None
    root = x[len(x) - p:]
    if count(docs, root) == 0:
        return None
    K = int(math.floor(alpha * p))

    def den(w):
        if den_mode == 0:
            return float(count(docs, w))
        return float(sum(children(docs, w, D).values()))

    frontier = []  # (score, token, parent, path)

    def push_children(w, parent_idx, parent_score):
        ch = children(docs, w, D)
        if not ch:
            return
        dn = den(w)
        for tok, c in ch.items():
            frontier.append((parent_score * (float(c) / dn), tok, parent_idx, w + [tok]))

    push_children(root, -1, 1.0)
    toks, pars, scs = [], [], []
    total = 0.0
    while len(toks) < K and frontier:
        best = min(frontier, key=lambda c: (-c[0], c[1], c[2]))
        if best[0] < min_score:
            break
        frontier.remove(best)
        if linear:
            del frontier[:]
        j = len(toks)
        toks.append(best[1]); pars.append(best[2]); scs.append(best[0])
        total += best[0]
        push_children(best[3], j, best[0])
    return toks, pars, scs, total


def generate(global_docs, request_seq, P, alpha, min_score, D, den_mode=0, linear=0):
    """Best tree over (global, p=1..P) then (request, p=1..P); strictly greater wins."""
    x = [int(v) for v in request_seq]
    best = dict(tokens=[], parents=[], scores=[], tree_score=0.0, match_len=0, source=-1)
    for s, docs in enumerate((global_docs, [x])):
        if docs is None:
            continue
        for p in range(1, P + 1):
            r = speculate_unit(docs, x, p, alpha, min_score, D, den_mode, linear)
            if r is None:
                continue
            if len(r[0]) > 0 and r[3] > best["tree_score"]:
                best = dict(tokens=r[0], parents=r[1], scores=r[2], tree_score=r[3], match_len=p,
                            source=s)
    return best


def accept_by_enumeration(tokens, parents, target):
    """Longest root-to-node path whose every node token equals the target token at the
    node's parent (target[0] belongs to the root)."""
    n = len(tokens)
    best_path = []
    for leaf in range(n):
        path = []
        v = leaf
        while v >= 0:
            path.append(v)
            v = parents[v]
        path.reverse()
        ok = all(tokens[v] == target[parents[v] + 1] for v in path)
        if ok and len(path) > len(best_path):
            best_path = path
    last = best_path[-1] if best_path else -1
    return len(best_path), best_path, target[last + 1]


def entropy(docs, D):
    """Empirical entropy of the depth-bounded suffix tree over `docs` (Appendix, "Predicting
    SuffixDecoding Effectiveness"), from substring counts alone: for every distinct substring w
    with |w| < D (the empty one included) that is followed by some token, the entropy in bits
    of "which token follows w", weighted by how many times something follows w.
    Returns (weighted mean, total weight)."""
    follow = {}
    for doc in docs:
        doc = [int(v) for v in doc]
        for i in range(len(doc)):
            for k in range(0, min(D - 1, i) + 1):   # context = the k tokens before position i
                follow.setdefault(tuple(doc[i - k:i]), Counter())[doc[i]] += 1
    acc = wsum = 0.0
    for w, c in follow.items():
        s = sum(c.values())
        acc += s * -sum((v / s) * math.log2(v / s) for v in c.values())
        wsum += s
    return (acc / wsum if wsum else 0.0), wsum
