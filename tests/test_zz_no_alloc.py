"""sd_speculate_static (the drafting call that uses the library's static device array as its
working memory) against sd_speculate on the same contexts: two calls in a row, the second with
a smaller batch and shorter contexts, so that what the first call left in the array lies under
and behind what the second one uses."""
import numpy as np
import pytest

from tests import parity
from workloads import make_workload, scaled

pytestmark = pytest.mark.gpu


def _trees_as_dict(tr):
    return dict(n_nodes=tr.n_nodes.cpu().numpy(), tokens=tr.tokens.cpu().numpy(),
                parents=tr.parents.cpu().numpy(), scores=tr.scores.cpu().numpy(),
                tree_score=tr.tree_score.cpu().numpy(), match_len=tr.match_len.cpu().numpy(),
                source=tr.source.cpu().numpy(), use_draft=tr.use_draft.cpu().numpy())


def test_static_scratch_entry_point_matches_sd_speculate():
    import torch
    import paper_2411_04975_amd as sd
    # low-repetition contexts: hundreds of occurrences of the last token, lists of more than 64
    # suffixes, i.e. both kinds of working memory are in use
    w = make_workload(scaled("lowrep", n_docs=100, batch=48, ctx=4096), seed=3, name="lowrep-s")
    docs = w.docs()
    B = w.batch
    g = parity.GpuPath(w.vocab, w.D, w.P, w.alpha, w.min_score, B, w.ctx_len + 8,
                       len(w.corpus) + len(docs))
    try:
        g.build_global(docs)
        first = [w.contexts[b] for b in range(B)]
        second = [w.contexts[b][1500:] for b in range(0, B, 3)]       # fewer and shorter
        for contexts in (first, second):
            n = len(contexts)
            g.build_requests(range(n), contexts)
            want = g.speculate(range(n))
            assert g.stats()["spec_request_wide"] > 0
            tr = sd.Trees(n, g.max_nodes, g.dev)
            for t in (tr.tokens, tr.parents, tr.n_nodes, tr.match_len, tr.source, tr.use_draft):
                t.fill_(-7)
            tr.scores.fill_(-7.0)
            tr.tree_score.fill_(-7.0)
            sd.sd_speculate_static(g.ctx, torch.arange(n, dtype=torch.int32, device=g.dev), tr)
            torch.cuda.synchronize()
            got = _trees_as_dict(tr)
            for k in want:
                assert np.array_equal(got[k], want[k]), k
        assert (want["n_nodes"] > 0).any()
    finally:
        g.close()


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    import paper_2411_04975_amd as sd
    # 96 requests x 32768 tokens x 8 bytes = 24 MiB > 16 MiB; 64 requests fit exactly
    g = parity.GpuPath(100, 8, 4, 1.0, 0.1, 96, 32768, 1000)
    try:
        tr = sd.Trees(96, g.max_nodes, g.dev)
        slots = torch.arange(96, dtype=torch.int32, device=g.dev)
        with pytest.raises(sd.SdError) as e:
            sd.sd_speculate_static(g.ctx, slots, tr)
        assert e.value.code == 4 and "SD_STATIC_SCRATCH_BYTES" in str(e.value)
        sd.sd_speculate_static(g.ctx, slots[:64].contiguous(), tr)      # empty contexts: no trees
        torch.cuda.synchronize()
        assert int(tr.n_nodes[:64].abs().sum().item()) == 0
    finally:
        g.close()
