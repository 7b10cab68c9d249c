"""plaid_search_static under HIP graph capture: the entry point that allocates nothing is the one a caller can record
into a graph (a serving loop replays the graph instead of enqueueing a dozen kernels per query).

The search is captured once on a side stream with fixed query / output buffers, then replayed several times with new
queries copied into the query buffer, with eager searches and synchronisations of the program between the replays;
every replay must give exactly what the eager search gives for the same queries (the library clears its workspace with
a kernel, not with a memset node, so replays after the first see clean counters)."""
import pytest
import torch

from synth import get_config, make_workload

import parity_util as pu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("nq,noise", [(1, "calibrated"), (5, "literal")])
def test_replays_match_eager_searches(nq, noise):
    import paper_2205_09707_amd as pl
    pl.load_library()
    cfg = get_config("cfg1")
    w = make_workload(cfg, device="cpu", noise=noise)
    gidx = pl.plaid_index_from_view(pu.device_arrays(w), cfg.nbits, device=0, copy=True)
    try:
        Q = w.queries.to(DEV)
        params = (cfg.nprobe, cfg.t_cs, cfg.ndocs, cfg.k)
        Qb = Q[:nq].clone()
        ids = torch.empty((nq, cfg.k), dtype=torch.int32, device=DEV)
        sc = torch.empty((nq, cfg.k), dtype=torch.float32, device=DEV)
        # first call outside the capture: the library looks up its static workspace once per device
        pl.plaid_search_static(gidx, Qb, *params, ids, sc)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            pl.plaid_search_static(gidx, Qb, *params, ids, sc)
        torch.cuda.synchronize()
        n_groups = Q.shape[0] // nq
        for rep in range(6):
            g0 = (rep * 3) % n_groups
            Qb.copy_(Q[g0 * nq:(g0 + 1) * nq])
            graph.replay()
            torch.cuda.synchronize()
            got_ids, got_sc = ids.clone(), sc.clone()
            # the program's own eager work between replays: the same queries, and another batch on the shared workspace
            e_ids, e_sc = pl.plaid_search(gidx, Q[g0 * nq:(g0 + 1) * nq], *params)
            pl.plaid_search(gidx, Q, *params)
            torch.cuda.synchronize()
            assert torch.equal(got_ids, e_ids), f"replay {rep}: ids differ from the eager search"
            assert torch.equal(got_sc, e_sc), f"replay {rep}: scores differ from the eager search"
    finally:
        pl.plaid_index_free(gidx)
