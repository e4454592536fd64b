"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad configurations before touching a device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    src = open(os.path.join(ROOT, "include", "sd.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(sd_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    from paper_2411_04975_amd import binding
    if not os.path.exists(binding.lib_path()):
        pytest.skip("libsd.so not built in this checkout")
    lib = C.CDLL(binding.lib_path())
    names = _declared_symbols()
    assert {"sd_create", "sd_destroy", "sd_index_build", "sd_index_append", "sd_index_insert", "sd_index_entropy", "sd_accept_append", "sd_accept_append_speculate",
            "sd_speculate", "sd_accept", "sd_get_stats", "sd_last_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_create_rejects_bad_configs_on_the_host():
    from paper_2411_04975_amd import binding
    if not os.path.exists(binding.lib_path()):
        pytest.skip("libsd.so not built in this checkout")
    sd = binding
    good = dict(vocab=100, D=8, P=4, alpha=1.0, min_score=0.1, max_batch_slots=4,
                max_ctx_tokens=64, max_global_tokens=1000)
    for bad in (dict(P=8), dict(P=0), dict(D=256), dict(alpha=0.0), dict(min_score=1.5),
                dict(min_score=-0.1), dict(vocab=0), dict(alpha=100.0), dict(max_batch_slots=0),
                dict(max_global_tokens=2 ** 31), dict(P=65, D=80)):
        cfg = dict(good)
        cfg.update(bad)
        with pytest.raises(sd.SdError) as e:
            sd.sd_create(**cfg)
        assert e.value.code == 1, bad


def test_binding_has_no_fallback():
    """The product package must not import the oracle."""
    import paper_2411_04975_amd
    pkg = os.path.dirname(paper_2411_04975_amd.__file__)
    for root, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                txt = open(os.path.join(root, f)).read()
                assert "import oracle" not in txt and "from oracle" not in txt, f
                assert "suffix_trie" not in txt, f


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N above 1 exits with a message before anything touches a GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and "--gpus 2" in r.stderr
    assert r.stdout.strip() == ""


def test_workload_generators_are_seeded_and_shaped():
    """The synthetic inputs are functions of (configuration, seed) alone, with the shapes the
    configuration names."""
    import numpy as np
    from workloads import CONFIGS, make_workload, scaled
    a = make_workload("tiny", seed=3)
    b = make_workload("tiny", seed=3)
    c = make_workload("tiny", seed=4)
    for f in ("corpus", "doc_offsets", "contexts", "future"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f
    assert not np.array_equal(a.corpus, c.corpus)
    cfg = CONFIGS["tiny"]
    assert a.contexts.shape == (cfg["batch"], cfg["ctx"]) and a.batch == cfg["batch"]
    assert a.corpus.dtype == np.int32 and a.contexts.dtype == np.int32
    assert a.corpus.min() >= 0 and a.corpus.max() < cfg["vocab"]
    assert a.doc_offsets[0] == 0 and a.doc_offsets[-1] == len(a.corpus)
    assert np.all(np.diff(a.doc_offsets) > 0)
    assert a.max_nodes == int(np.floor(cfg["alpha"] * cfg["P"]))
    z = make_workload(scaled("lowrep", n_docs=20, doc_len=(300, 300), batch=4, ctx=64), seed=1)
    assert z.contexts.shape == (4, 64) and len(z.corpus) == 20 * 300
    # the low-repetition stream is skewed: its most frequent token is far above the uniform share
    top = np.bincount(z.corpus).max() / len(z.corpus)
    assert top > 20.0 / z.vocab
    # further contexts: seeded, shaped, copied from the same templates as the corpus (their
    # 8-token windows occur in it far more often than chance allows), yet other contexts
    from workloads.synth import extra_contexts
    e = extra_contexts("tiny", 3, 5)
    assert e.shape == (5, cfg["ctx"]) and e.dtype == np.int32
    assert np.array_equal(e, extra_contexts("tiny", 3, 5))
    assert not np.array_equal(e[:5], a.contexts[:5])
    win = set(map(bytes, np.lib.stride_tricks.sliding_window_view(a.corpus, 8)))
    hits = sum(bytes(x) in win for x in np.lib.stride_tricks.sliding_window_view(e[0], 8))
    assert hits > 100
    other = extra_contexts("tiny", 4, 5)       # another seed: other templates
    assert sum(bytes(x) in win for x in np.lib.stride_tricks.sliding_window_view(other[0], 8)) == 0
    ez = extra_contexts(scaled("lowrep", ctx=64), 1, 3)
    assert ez.shape == (3, 64) and ez.max() < z.vocab
