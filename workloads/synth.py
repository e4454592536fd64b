"""Deterministic synthetic token streams shaped like the paper's workloads.

The paper evaluates on traces of agentic applications (long outputs that
repeat spans of earlier outputs with small edits) and on open-ended chat (low
repetition).  Those traces are not available, so two seeded processes stand in
for them:

* templated: a sequence is a concatenation of spans copied from a fixed pool of
  random "template" sequences, after which each token is independently replaced
  by a uniform random token with a small probability (the "mutation" rate);
* zipf: tokens drawn i.i.d. from a Zipf(s) law over token ranks.

Every request context also carries the unmutated continuation of the template
span it stopped in; a simulated greedy verifier (Section 4.1, "Simulated
Ablations") accepts a drafted token iff it equals that continuation.

Only numpy is used.  Nothing here computes anything about suffix trees.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Tuple

import numpy as np


@dataclasses.dataclass
class Workload:
    name: str
    vocab: int
    D: int
    P: int
    alpha: float
    min_score: float
    # global corpus: concatenated documents and their offsets
    corpus: np.ndarray            # int32[n]
    doc_offsets: np.ndarray       # int64[n_docs+1]
    # request contexts: equal length ctx_len each
    contexts: np.ndarray          # int32[B, ctx_len]
    # ground-truth future tokens of each request (what the target model will say)
    future: np.ndarray            # int32[B, future_len]
    seed: int
    steps: int = 0                # decode steps for streaming style runs
    params: Optional[dict] = None

    @property
    def batch(self) -> int:
        return int(self.contexts.shape[0])

    @property
    def ctx_len(self) -> int:
        return int(self.contexts.shape[1])

    @property
    def max_nodes(self) -> int:
        return int(np.floor(self.alpha * self.P))

    def docs(self) -> List[np.ndarray]:
        o = self.doc_offsets
        return [self.corpus[o[i]:o[i + 1]] for i in range(len(o) - 1)]


# Shapes follow the five benchmark configurations; parameters the configuration
# text leaves open (template length, span range, document length law) are fixed
# here and echoed into every results file through Workload.params.
CONFIGS: Dict[str, dict] = {
    "tiny": dict(kind="templated", vocab=32000, n_templates=10, template_len=400,
                 span=(8, 64), mut=0.05, n_docs=40, doc_len=(500, 500), total=None,
                 batch=16, ctx=512, D=24, P=16, alpha=1.0, min_score=0.1, steps=8),
    "agentic": dict(kind="templated", vocab=128256, n_templates=200, template_len=1024,
                    span=(16, 256), mut=0.05, n_docs=2000, doc_len=(200, 2000), total=None,
                    batch=64, ctx=8192, D=64, P=32, alpha=1.0, min_score=0.1, steps=8),
    "large": dict(kind="templated", vocab=128256, n_templates=5000, template_len=1024,
                  span=(16, 256), mut=0.03, n_docs=None, doc_len=(200, 2000), total=10_000_000,
                  batch=256, ctx=16384, D=64, P=32, alpha=2.0, min_score=0.05, steps=8),
    "lowrep": dict(kind="zipf", vocab=152064, zipf_s=1.1, n_docs=5000, doc_len=(2000, 2000),
                   total=None, batch=256, ctx=4096, D=32, P=16, alpha=1.0, min_score=0.1,
                   steps=8),
    "streaming": dict(kind="templated", vocab=128256, n_templates=10000, template_len=1024,
                      span=(16, 256), mut=0.05, n_docs=None, doc_len=(200, 2000),
                      total=100_000_000, batch=512, ctx=8192, D=64, P=32, alpha=1.0,
                      min_score=0.1, steps=64),
}


def scaled(name: str, **over) -> dict:
    """A copy of a named configuration with some fields replaced."""
    c = dict(CONFIGS[name])
    c.update(over)
    return c


def _doc_lengths(rng, n_docs, doc_len, total) -> np.ndarray:
    lo, hi = doc_len
    if total is None:
        return rng.integers(lo, hi + 1, size=n_docs, dtype=np.int64)
    # draw documents until the stream holds exactly `total` tokens
    est = int(total / ((lo + hi) / 2) * 1.1) + 16
    while True:
        lens = rng.integers(lo, hi + 1, size=est, dtype=np.int64)
        cs = np.cumsum(lens)
        if cs[-1] >= total:
            break
        est *= 2
    k = int(np.searchsorted(cs, total, side="left"))
    lens = lens[:k + 1].copy()
    lens[k] -= cs[k] - total
    return lens[lens > 0]


def _templated_sequences(rng, templates: np.ndarray, lens: np.ndarray, span: Tuple[int, int],
                         mut: float, vocab: int):
    """Concatenate copied template spans into sequences of the given lengths.

    Returns (tokens int32[sum(lens)], last_template int64[n_seq], last_next int64[n_seq])
    where (last_template, last_next) name the template position that follows the
    final copied token of each sequence (before mutation)."""
    n_t, t_len = templates.shape
    lo, hi = span
    n_seq = len(lens)
    max_spans = int(np.max(lens) // lo) + 2
    toks_parts = []
    last_tmpl = np.zeros(n_seq, np.int64)
    last_next = np.zeros(n_seq, np.int64)
    # chunk the sequences so that the (n_seq x max_spans) work arrays stay small
    chunk = max(1, int(4_000_000 // max_spans))
    for c0 in range(0, n_seq, chunk):
        L = lens[c0:c0 + chunk]
        m = len(L)
        sl = rng.integers(lo, hi + 1, size=(m, max_spans), dtype=np.int64)
        tid = rng.integers(0, n_t, size=(m, max_spans), dtype=np.int64)
        u = rng.random(size=(m, max_spans))
        start = np.floor(u * (t_len - sl + 1)).astype(np.int64)
        before = np.cumsum(sl, axis=1) - sl
        eff = np.clip(L[:, None] - before, 0, sl)           # truncate the last span
        flat_eff = eff.ravel()
        keep = flat_eff > 0
        e = flat_eff[keep]
        s = start.ravel()[keep]
        t = tid.ravel()[keep]
        tot = int(e.sum())
        span_first = np.cumsum(e) - e                        # output index where each span begins
        within = np.arange(tot, dtype=np.int64) - np.repeat(span_first, e)
        src = np.repeat(t * t_len + s, e) + within
        toks_parts.append(templates.ravel()[src])
        # last span of every sequence in this chunk
        nspan = (eff > 0).sum(axis=1)
        rows = np.arange(m)
        lt = tid[rows, nspan - 1]
        ln = start[rows, nspan - 1] + eff[rows, nspan - 1]
        last_tmpl[c0:c0 + m] = lt
        last_next[c0:c0 + m] = ln
    toks = np.concatenate(toks_parts).astype(np.int32)
    if mut > 0:
        mask = rng.random(toks.shape[0]) < mut
        toks[mask] = rng.integers(0, vocab, size=int(mask.sum()), dtype=np.int32)
    return toks, last_tmpl, last_next


def _zipf_table(vocab: int, s: float) -> np.ndarray:
    w = 1.0 / np.power(np.arange(1, vocab + 1, dtype=np.float64), s)
    cdf = np.cumsum(w)
    return cdf / cdf[-1]


def make_workload(cfg, seed: int = 0, future_len: Optional[int] = None, name: Optional[str] = None
                  ) -> Workload:
    """Build corpus, contexts and ground-truth futures for a configuration.

    `cfg` is a key of CONFIGS or a dict with the same fields."""
    if isinstance(cfg, str):
        name = name or cfg
        cfg = CONFIGS[cfg]
    name = name or "custom"
    rng = np.random.default_rng(np.random.PCG64(seed))
    vocab = int(cfg["vocab"])
    B, ctx = int(cfg["batch"]), int(cfg["ctx"])
    steps = int(cfg.get("steps", 0))
    max_nodes = int(np.floor(cfg["alpha"] * cfg["P"]))
    if future_len is None:
        future_len = max(1, steps) * (max_nodes + 1) + max_nodes + 1
    lens = _doc_lengths(rng, cfg.get("n_docs"), cfg["doc_len"], cfg.get("total"))
    offs = np.zeros(len(lens) + 1, np.int64)
    np.cumsum(lens, out=offs[1:])
    if cfg["kind"] == "templated":
        templates = rng.integers(0, vocab, size=(cfg["n_templates"], cfg["template_len"]),
                                 dtype=np.int32)
        corpus, _, _ = _templated_sequences(rng, templates, lens, cfg["span"], cfg["mut"], vocab)
        cl = np.full(B, ctx, np.int64)
        ctoks, lt, ln = _templated_sequences(rng, templates, cl, cfg["span"], cfg["mut"], vocab)
        contexts = ctoks.reshape(B, ctx)
        t_len = templates.shape[1]
        idx = (ln[:, None] + np.arange(future_len, dtype=np.int64)[None, :]) % t_len
        future = templates[lt[:, None], idx].astype(np.int32)
    elif cfg["kind"] == "zipf":
        cdf = _zipf_table(vocab, cfg["zipf_s"])
        corpus = np.searchsorted(cdf, rng.random(int(offs[-1])), side="left").astype(np.int32)
        contexts = np.searchsorted(cdf, rng.random(B * ctx), side="left").astype(np.int32)
        contexts = contexts.reshape(B, ctx)
        future = np.searchsorted(cdf, rng.random(B * future_len), side="left").astype(np.int32)
        future = future.reshape(B, future_len)
        np.minimum(corpus, vocab - 1, out=corpus)
        np.minimum(contexts, vocab - 1, out=contexts)
        np.minimum(future, vocab - 1, out=future)
    else:
        raise ValueError(cfg["kind"])
    return Workload(name=name, vocab=vocab, D=int(cfg["D"]), P=int(cfg["P"]),
                    alpha=float(cfg["alpha"]), min_score=float(cfg["min_score"]),
                    corpus=np.ascontiguousarray(corpus), doc_offsets=offs,
                    contexts=np.ascontiguousarray(contexts), future=np.ascontiguousarray(future),
                    seed=seed, steps=steps, params=dict(cfg))


def extra_contexts(cfg, seed: int, n: int) -> np.ndarray:
    """`n` further contexts of a configuration, int32[n, ctx]: drawn by the same process as
    make_workload's (for a templated configuration from the very templates that
    make_workload(cfg, seed) copies from), with a generator of their own."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    vocab, ctx = int(cfg["vocab"]), int(cfg["ctx"])
    rng2 = np.random.default_rng(np.random.PCG64([seed, 0x65787472]))
    if cfg["kind"] == "templated":
        rng = np.random.default_rng(np.random.PCG64(seed))       # replay the draws up to the templates
        _doc_lengths(rng, cfg.get("n_docs"), cfg["doc_len"], cfg.get("total"))
        templates = rng.integers(0, vocab, size=(cfg["n_templates"], cfg["template_len"]),
                                 dtype=np.int32)
        toks, _, _ = _templated_sequences(rng2, templates, np.full(n, ctx, np.int64), cfg["span"],
                                          cfg["mut"], vocab)
    else:
        cdf = _zipf_table(vocab, cfg["zipf_s"])
        toks = np.searchsorted(cdf, rng2.random(n * ctx), side="left").astype(np.int32)
        np.minimum(toks, vocab - 1, out=toks)
    return np.ascontiguousarray(toks.reshape(n, ctx))

