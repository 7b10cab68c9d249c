"""The entry point that allocates nothing (plaid_search_static) against plaid_search, through the C ABI: bit-identical
ids and scores on two calls in a row, the second with a smaller input, and a clear error when one query does not fit."""
import numpy as np
import pytest
import torch

from synth import get_config, make_workload, tiny_config

import parity_util as pu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(pl, gidx, Q, params):
    nprobe, t_cs, ndocs, k = params
    want_ids, want_sc = pl.plaid_search(gidx, Q, nprobe, t_cs, ndocs, k)
    ids = torch.full((Q.shape[0], k), -7, dtype=torch.int32, device=DEV)
    sc = torch.full((Q.shape[0], k), float("nan"), dtype=torch.float32, device=DEV)
    pl.plaid_search_static(gidx, Q, nprobe, t_cs, ndocs, k, ids, sc)
    torch.cuda.synchronize()
    assert torch.equal(ids, want_ids), params
    assert torch.equal(sc.view(torch.int32), want_sc.view(torch.int32)), params   # bit for bit


def test_static_workspace_search_equals_plaid_search():
    import paper_2205_09707_amd as pl
    pl.load_library()
    w = make_workload(get_config("cfg1"), noise="calibrated")
    gidx = pl.plaid_index_from_view(pu.device_arrays(w), w.cfg.nbits, device=0, copy=True)
    try:
        Q = w.queries.to(DEV)
        _both(pl, gidx, Q, (2, 0.45, 1024, 100))                 # all 16 queries
        _both(pl, gidx, Q[:3].contiguous(), (1, 0.5, 256, 10))   # right after it, a smaller call: stale contents must not matter
        _both(pl, gidx, Q[5:6].contiguous(), (12, 0.5, 128, 10)) # the general top-nprobe path
        _both(pl, gidx, Q, (2, np.inf, 64, 5))
    finally:
        pl.plaid_index_free(gidx)


def test_static_workspace_rejects_what_does_not_fit():
    import paper_2205_09707_amd as pl
    pl.load_library()
    need, _ = pl.plaid_workspace_bytes(16, 5_000_000, 1, 1, 16, 4)
    assert need > (64 << 20)
    w = make_workload(tiny_config(C=16, P=5_000_000, lo=1, hi=1, nbits=2, nq=1, seed=81), noise="calibrated")
    gidx = pl.plaid_index_from_view(pu.device_arrays(w), 2, device=0, copy=True)
    try:
        ids = torch.empty((1, 4), dtype=torch.int32, device=DEV)
        sc = torch.empty((1, 4), dtype=torch.float32, device=DEV)
        with pytest.raises(pl.PlaidError):
            pl.plaid_search_static(gidx, w.queries.to(DEV), 1, 0.5, 16, 4, ids, sc)
        pl.plaid_search(gidx, w.queries.to(DEV), 1, 0.5, 16, 4)   # the allocating entry point still serves it
        torch.cuda.synchronize()
    finally:
        pl.plaid_index_free(gidx)
