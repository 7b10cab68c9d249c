"""Queries that hold NaN or infinities: results for them are unspecified, but the call must return normally, every
returned id must lie in [-1, P), and the well-formed queries of the same batch must get exactly the results they get
in a batch without the malformed ones (no kernel indexes memory with a value derived from a score except through ids
that are valid by construction or clamped: the probe kernel fills a slot it could not rank with a valid centroid id,
bins are clamped, selections work on integer keys)."""
import numpy as np
import pytest
import torch

from synth import make_workload, tiny_config

import parity_util as pu
from test_gpu_parity import _kernel_forms

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("form,stage2", [("split16", "inverted"), ("split16", "stream"), ("matrix", "inverted"),
                                         ("vector", "stream")])
def test_nonfinite_query_tokens(form, stage2):
    import paper_2205_09707_amd as pl
    pl.load_library()
    cfg = tiny_config(C=700, P=3000, lo=2, hi=40, nbits=2, nq=40, seed=61)
    w = make_workload(cfg, noise="calibrated")
    Q = w.queries.clone()
    bad = [1, 5, 9, 17, 33, 38]
    Q[1, 3, :] = float("nan")                     # one token of NaN
    Q[5, :, :] = float("nan")                     # a whole query of NaN
    Q[9, 0, 7] = float("inf")                     # one +inf element: its column holds +-inf and NaN
    Q[17, 30, :] = float("-inf")
    Q[33, 2, 5] = float("nan")
    Q[33, 8, 100] = float("inf")
    Q[38, :, 0] = float("inf")
    Q[38, 4, 1] = float("-inf")
    good = [q for q in range(cfg.nq) if q not in bad]
    with _kernel_forms(form, stage2):
        gidx = pl.plaid_index_from_view(pu.device_arrays(w), cfg.nbits, device=0, copy=True)
    try:
        Qd = Q.to(DEV)
        Qclean = w.queries[good].contiguous().to(DEV)
        for params in [(1, 0.5, 64, 8), (2, 0.45, 256, 20), (4, -np.inf, 128, 16), (2, np.inf, 64, 8), (12, 0.3, 100, 10)]:
            print(f"[nonfinite] form={form} stage2={stage2} params={params}", flush=True)
            ids, sc = pl.plaid_search(gidx, Qd, *params)
            want_ids, want_sc = pl.plaid_search(gidx, Qclean, *params)
            torch.cuda.synchronize()
            ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
            assert ids.min() >= -1 and ids.max() < cfg.P, params
            np.testing.assert_array_equal(ids[good], want_ids.cpu().numpy(), err_msg=str(params))
            np.testing.assert_array_equal(pu.bits(sc[good]), pu.bits(want_sc.cpu().numpy()), err_msg=str(params))
            for q in bad:   # no id twice among a malformed query's results either
                got = ids[q][ids[q] >= 0]
                assert len(set(got.tolist())) == len(got), (params, q)
        # one malformed query alone (the single-query launch shapes)
        for q in bad:
            i1, _ = pl.plaid_search(gidx, Qd[q:q + 1], 2, 0.45, 256, 20)
            torch.cuda.synchronize()
            i1 = i1.cpu().numpy()
            assert i1.min() >= -1 and i1.max() < cfg.P, q
    finally:
        pl.plaid_index_free(gidx)
