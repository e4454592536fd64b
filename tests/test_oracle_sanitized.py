"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: the inputs of the
oracle's pins (the tiny workload, adversarial minis, both denominators, the chain variant) go
through a sanitized build of oracle/suffix_trie.c (tests/oracle_sanitized_driver.c, a
standalone program with the sanitizer runtime linked in statically); it must finish without a
report and print exactly what the ordinary build returns."""
import math
import os
import struct
import subprocess

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-o", exe,
           os.path.join(HERE, "oracle_sanitized_driver.c"), "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        pytest.skip("no sanitizer runtime for gcc here: " + r.stderr[-300:])
    return exe


def _expected(D, P, alpha, ms, den_mode, linear, docs, ctxs, splits, targets):
    """The same lines from the ordinary build, through its Python wrapper."""
    K = max(1, int(math.floor(alpha * P)))
    tg = oracle.Trie(D)
    for d in docs:
        tg.add_doc(d)
    h, wt = tg.entropy()
    out = ["global nodes %d entropy %s weight %s" % (tg.num_nodes, float(h).hex(), float(wt).hex())]
    for c, x in enumerate(ctxs):
        tr = oracle.Trie(D)
        tr.append(x[:splits[c]])
        tr.append(x[splits[c]:])
        for p in range(1, min(P, len(x)) + 1):
            cg, eg, kg = tg.lookup(x[-p:])
            cr, er, kr = tr.lookup(x[-p:])
            out.append("ctx %d p %d global %d count %d ends %d children %d request count %d ends %d "
                       "children %d" % (c, p, tg.match(x, p), cg, eg, kg, cr, er, kr))
        g = oracle.generate(tg, tr, x, P, alpha, ms, den_mode, linear)
        L, path, bonus = oracle.accept(g["tokens"], g["parents"], targets[c])
        nodes = "".join(" (%d %d %s)" % (int(t), int(q), float(s).hex())
                        for t, q, s in zip(g["tokens"], g["parents"], g["scores"]))
        out.append("ctx %d tree n %d p %d source %d score %s:%s accept %d bonus %d path%s" % (
            c, g["n_nodes"], g["match_len"], g["source"], float(g["tree_score"]).hex(), nodes, L,
            bonus, "".join(" %d" % j for j in path)))
    return out


def _hex(line):
    """C prints doubles with %a, Python with float.hex(): compare their values."""
    return [float.fromhex(t.strip("():")) if t.strip("():").lstrip("-").startswith("0x") else t
            for t in line.split()]


def _run(driver, tmp_path, D, P, alpha, ms, den_mode, linear, docs, ctxs, seed=0):
    rng = np.random.default_rng(seed)
    K = max(1, int(math.floor(alpha * P)))
    docs = [np.asarray(d, np.int32) for d in docs]
    ctxs = [np.asarray(c, np.int32) for c in ctxs if len(c)]
    vocab = int(max([int(d.max()) for d in docs if len(d)] + [int(c.max()) for c in ctxs])) + 1
    splits = [int(rng.integers(0, len(c) + 1)) for c in ctxs]
    targets = [rng.integers(0, vocab, K + 1).astype(np.int32) for _ in ctxs]
    words = [np.array([D, P, den_mode, linear], np.int32),
             np.frombuffer(struct.pack("<dd", alpha, ms), np.int32), np.array([len(docs)], np.int32)]
    for d in docs:
        words += [np.array([len(d)], np.int32), d]
    words.append(np.array([len(ctxs)], np.int32))
    for c, s, t in zip(ctxs, splits, targets):
        words += [np.array([len(c)], np.int32), c, np.array([s], np.int32), t]
    case = str(tmp_path / "case.bin")
    np.concatenate(words).astype("<i4").tofile(case)
    r = subprocess.run([driver, case], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stderr == "", r.stderr[-2000:]
    got = r.stdout.strip().split("\n")
    want = _expected(D, P, alpha, ms, den_mode, linear, docs, ctxs, splits, targets)
    assert len(got) == len(want)
    for a, b in zip(got, want):
        assert _hex(a) == _hex(b), (a, b)


@pytest.mark.parametrize("den_mode,linear", [(0, 0), (1, 0), (0, 1)])
def test_sanitized_oracle_on_the_tiny_workload(driver, tmp_path, tiny_workload, den_mode, linear):
    w = tiny_workload
    _run(driver, tmp_path, w.D, w.P, w.alpha, w.min_score, den_mode, linear, w.docs(),
         [w.contexts[b] for b in range(w.batch)])


def test_sanitized_oracle_on_adversarial_minis(driver, tmp_path):
    rng = np.random.default_rng(3)
    cases = [
        (6, 3, 2.0, 0.05, [[1] * 50], [[1] * 20, [1], [0, 1, 1]]),
        (4, 2, 2.0, 0.1, [[0], [1], [1], [2]], [[1], [2, 1], [0, 0, 0]]),
        (10, 8, 1.0, 0.1, [[0, 1, 2, 3] * 10], [[2, 3], [3], [0, 1, 2]]),
        (8, 4, 4.0, 0.0, [[0, 1, 2, 0, 1, 1, 0, 2, 2, 1, 0, 1] * 4], [[2, 0, 1], [1, 1, 0], [0]]),
        (12, 6, 4.0, 0.02, [list(rng.integers(0, 2, 400))],
         [list(rng.integers(0, 2, int(rng.integers(1, 300)))) for _ in range(8)]),
        (9, 6, 0.5, 0.1, [[0, 1, 2, 3, 4] * 12], [[3, 4, 0, 1, 2, 3]]),
        (255, 64, 4.0, 0.001, [list(rng.integers(0, 4, 1500))], [list(rng.integers(0, 4, 300))]),
    ]
    for i, (D, P, alpha, ms, docs, ctxs) in enumerate(cases):
        for den_mode, linear in ((0, 0), (1, 1)):
            _run(driver, tmp_path, D, P, alpha, ms, den_mode, linear, docs, ctxs, seed=i)
