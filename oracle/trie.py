"""ctypes wrapper over the C oracle (suffix_trie.c).  Test infrastructure only.

Function names follow Algorithm 1 of the paper: `speculate_unit` is
MatchPattern + ExpandSpeculationTree for one (structure, p); `generate` is
GenerateCandidateTree; `accept` is the greedy verification walk of Section 2
(drafted tokens are kept until the first one the target model disagrees with).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "suffix_trie.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def library_path() -> str:
    return _LIB


def build_library(force: bool = False) -> str:
    """Compile suffix_trie.c with gcc (no GPU code involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build_library()
    L = C.CDLL(_LIB)
    vp, i32p, i64p, f64p, u8p = (C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64),
                                 C.POINTER(C.c_double), C.POINTER(C.c_uint8))
    L.sdo_trie_new.restype = vp
    L.sdo_trie_new.argtypes = [C.c_int]
    L.sdo_trie_free.argtypes = [vp]
    L.sdo_trie_num_nodes.restype = C.c_int64
    L.sdo_trie_num_nodes.argtypes = [vp]
    L.sdo_trie_add_doc.argtypes = [vp, i32p, C.c_int64, u8p]
    L.sdo_trie_append.argtypes = [vp, i32p, C.c_int64]
    L.sdo_trie_lookup.restype = C.c_int
    L.sdo_trie_lookup.argtypes = [vp, i32p, C.c_int, i64p, i64p, i64p]
    L.sdo_trie_children.restype = C.c_int64
    L.sdo_trie_children.argtypes = [vp, i32p, C.c_int, i32p, i64p, C.c_int64]
    L.sdo_trie_dump.argtypes = [vp, i32p, i32p, i32p, i32p, i32p]
    L.sdo_trie_entropy.restype = C.c_double
    L.sdo_trie_entropy.argtypes = [vp, f64p]
    L.sdo_match.restype = C.c_int32
    L.sdo_match.argtypes = [vp, i32p, C.c_int64, C.c_int]
    L.sdo_speculate_unit.restype = C.c_int
    L.sdo_speculate_unit.argtypes = [vp, i32p, C.c_int64, C.c_int, C.c_double, C.c_double, C.c_int,
                                     C.c_int, i32p, i32p, f64p, f64p]
    L.sdo_generate.restype = C.c_int
    L.sdo_generate.argtypes = [vp, vp, i32p, C.c_int64, C.c_int, C.c_double, C.c_double, C.c_int,
                               C.c_int, i32p, i32p, f64p, f64p, i32p, i32p]
    L.sdo_accept.restype = C.c_int
    L.sdo_accept.argtypes = [C.c_int, i32p, i32p, i32p, i32p, i32p]
    _lib = L
    return L


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(C.POINTER(ty))


class Trie:
    """Suffix trie over D-truncated suffixes with per-node COUNT and ENDS."""

    def __init__(self, D: int):
        self._L = _load()
        self.D = int(D)
        self._h = C.c_void_p(self._L.sdo_trie_new(self.D))

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h:
            self._L.sdo_trie_free(h)

    @property
    def num_nodes(self) -> int:
        return int(self._L.sdo_trie_num_nodes(self._h))

    def add_doc(self, tokens, allowed_first: Optional[np.ndarray] = None) -> None:
        """Insert all suffixes of a closed document.  `allowed_first` (uint8[vocab]) restricts
        insertion to suffixes whose first token is flagged; lookups below flagged first tokens
        are unaffected by the restriction."""
        t = _i32(tokens)
        al = None
        if allowed_first is not None:
            al = np.ascontiguousarray(allowed_first, dtype=np.uint8)
        self._L.sdo_trie_add_doc(self._h, _p(t, C.c_int32), t.shape[0],
                                 _p(al, C.c_uint8) if al is not None else None)

    def append(self, tokens) -> None:
        """Extend the one open sequence of this trie (per-request use)."""
        t = _i32(np.atleast_1d(tokens))
        self._L.sdo_trie_append(self._h, _p(t, C.c_int32), t.shape[0])

    def lookup(self, w) -> Tuple[int, int, int]:
        """(COUNT, ENDS, number of children) of the path w; zeros if absent."""
        w = _i32(w)
        c, e, k = C.c_int64(), C.c_int64(), C.c_int64()
        self._L.sdo_trie_lookup(self._h, _p(w, C.c_int32), w.shape[0], C.byref(c), C.byref(e),
                                C.byref(k))
        return c.value, e.value, k.value

    def children(self, w) -> dict:
        w = _i32(w)
        n = self._L.sdo_trie_children(self._h, _p(w, C.c_int32), w.shape[0], None, None, 0)
        tok = np.zeros(max(n, 1), np.int32)
        cnt = np.zeros(max(n, 1), np.int64)
        self._L.sdo_trie_children(self._h, _p(w, C.c_int32), w.shape[0], _p(tok, C.c_int32),
                                  _p(cnt, C.c_int64), n)
        return {int(tok[i]): int(cnt[i]) for i in range(n)}

    def dump(self):
        """Node table: token, count, ends, parent, depth (node 0 is the root)."""
        n = self.num_nodes
        arrs = [np.zeros(n, np.int32) for _ in range(5)]
        self._L.sdo_trie_dump(self._h, *[_p(a, C.c_int32) for a in arrs])
        return dict(token=arrs[0], count=arrs[1], ends=arrs[2], parent=arrs[3], depth=arrs[4])

    def entropy(self) -> Tuple[float, float]:
        """(weighted mean entropy in bits, total weight): Appendix, "Predicting SuffixDecoding
        Effectiveness"."""
        w = C.c_double()
        h = self._L.sdo_trie_entropy(self._h, C.byref(w))
        return float(h), float(w.value)

    def match(self, x, p: int) -> int:
        x = _i32(x)
        return int(self._L.sdo_match(self._h, _p(x, C.c_int32), x.shape[0], p))


def speculate_unit(trie: Trie, x, p: int, alpha: float, min_score: float, den_mode: int = 0,
                   linear: int = 0):
    """One (structure, p) unit.  Returns None if the pattern does not match, else
    (tokens, parents, scores, tree_score).  den_mode 1 = the printed sibling-sum denominator;
    linear 1 = the chain-only variant."""
    L = _load()
    x = _i32(x)
    K = max(1, int(np.floor(alpha * p)))
    tok = np.zeros(K, np.int32)
    par = np.zeros(K, np.int32)
    sc = np.zeros(K, np.float64)
    ts = C.c_double()
    n = L.sdo_speculate_unit(trie._h, _p(x, C.c_int32), x.shape[0], p, alpha, min_score, den_mode,
                             linear, _p(tok, C.c_int32), _p(par, C.c_int32), _p(sc, C.c_double),
                             C.byref(ts))
    if n < 0:
        return None
    return tok[:n].copy(), par[:n].copy(), sc[:n].copy(), ts.value


def generate(tg: Optional[Trie], tr: Optional[Trie], x, P: int, alpha: float, min_score: float,
             den_mode: int = 0, linear: int = 0):
    """GenerateCandidateTree.  Returns dict(tokens, parents, scores, tree_score, match_len,
    source, n_nodes)."""
    L = _load()
    x = _i32(x)
    K = max(1, int(np.floor(alpha * P)))
    tok = np.zeros(K, np.int32)
    par = np.zeros(K, np.int32)
    sc = np.zeros(K, np.float64)
    ts = C.c_double()
    ml, src = C.c_int32(), C.c_int32()
    n = L.sdo_generate(tg._h if tg is not None else None, tr._h if tr is not None else None,
                       _p(x, C.c_int32), x.shape[0], P, alpha, min_score, den_mode, linear,
                       _p(tok, C.c_int32), _p(par, C.c_int32), _p(sc, C.c_double), C.byref(ts),
                       C.byref(ml), C.byref(src))
    return dict(tokens=tok[:n].copy(), parents=par[:n].copy(), scores=sc[:n].copy(),
                tree_score=ts.value, match_len=ml.value, source=src.value, n_nodes=n)


def accept(tokens, parents, target):
    """Greedy verification walk.  Returns (accept_len, path, bonus)."""
    L = _load()
    tokens, parents, target = _i32(tokens), _i32(parents), _i32(target)
    n = tokens.shape[0]
    path = np.zeros(max(n, 1), np.int32)
    bonus = C.c_int32()
    k = L.sdo_accept(n, _p(tokens, C.c_int32), _p(parents, C.c_int32), _p(target, C.c_int32),
                     _p(path, C.c_int32), C.byref(bonus))
    return k, path[:k].copy(), bonus.value
