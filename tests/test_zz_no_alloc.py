"""pqt_query_batch_noalloc (the entry point for callers that cannot allocate device memory) against
pqt_query_batch: same ids and distance bits, on two calls in a row, the second with a smaller input."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
from oracle import pqt_index_io as IO  # noqa: E402

pytestmark = pytest.mark.gpu


def test_noalloc_entry_point_matches_query_batch(tiny, tmp_path):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: no silent fallback")
    import paper_1702_05911_amd.binding as pqt
    from workloads import tiny_mixture
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    Yall = torch.from_numpy(tiny_mixture(2000, d=cfg.D, seed=77)).cuda()
    gix = pqt.pqt_index_load(path, 0)
    try:
        assert pqt.pqt_noalloc_workspace_bytes() == 32 << 20
        # (queries, k, w): a full batch, then a smaller one with longer lists, then a handful
        # (the small-batch launch shape), all through the same static workspace
        for lo, hi, k, w in ((0, 2000, cfg.k, cfg.w), (1000, 1700, 20, cfg.k1), (5, 42, 3, 1)):
            print(f"no-alloc call: queries {lo}..{hi} k={k} w={w}", flush=True)
            yq = Yall[lo:hi].contiguous()
            want_ids, want_d = pqt.pqt_query_batch(gix, yq, k, w)
            torch.cuda.synchronize()
            ids = torch.full((hi - lo, k), -7, dtype=torch.int64, device="cuda")
            d = torch.full((hi - lo, k), -7.0, dtype=torch.float32, device="cuda")
            pqt.pqt_query_batch_noalloc(gix, yq, k, w, ids, d)
            torch.cuda.synchronize()
            assert torch.equal(ids, want_ids), "ids differ from pqt_query_batch"
            assert torch.equal(d.view(torch.int32), want_d.view(torch.int32)), "distance bits differ"
        # a batch whose workspace exceeds the static array is refused, and nothing is written
        pqt.pqt_set_budget(gix, 8192, cfg.C)
        big = Yall.repeat(3, 1).contiguous()                     # 6000 queries x 8 T bytes of runs alone > 32 MiB
        ids = torch.full((big.shape[0], cfg.k), -7, dtype=torch.int64, device="cuda")
        d = torch.zeros((big.shape[0], cfg.k), dtype=torch.float32, device="cuda")
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_query_batch_noalloc(gix, big, cfg.k, cfg.w, ids, d)
        assert e.value.code == pqt.PQT_EINVAL
        torch.cuda.synchronize()
        assert bool((ids == -7).all())
        # the fixed bin order: refused until a pqt_query_batch call has built its tables, then identical
        pqt.pqt_set_budget(gix, cfg.T, cfg.C)
        pqt.pqt_set_bin_order(gix, pqt.PQT_ORDER_STATIC_SLOPES)
        yq = Yall[:300].contiguous()
        ids = torch.empty((300, cfg.k), dtype=torch.int64, device="cuda")
        d = torch.empty((300, cfg.k), dtype=torch.float32, device="cuda")
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_query_batch_noalloc(gix, yq, cfg.k, cfg.w, ids, d)
        assert e.value.code == pqt.PQT_EUNSUPPORTED
        want_ids, want_d = pqt.pqt_query_batch(gix, yq, cfg.k, cfg.w)
        pqt.pqt_query_batch_noalloc(gix, yq, cfg.k, cfg.w, ids, d)
        torch.cuda.synchronize()
        assert torch.equal(ids, want_ids) and torch.equal(d.view(torch.int32), want_d.view(torch.int32))
    finally:
        pqt.pqt_index_free(gix)
