"""Does the synthetic workload behave like the paper's?  Two of its analyses, rerun on the calibrated generator.

Section 3.3 / Figure 3: retrieval with the centroids alone (every passage ranked by its unpruned centroid-interaction
score, Eq. 3-4, no residuals) finds the passages exhaustive MaxSim ranks first: the share of the exhaustive top-k that
lies within the centroid-only top-k', k' >= k; the paper reports 99+ % at k' = 10 k.

Section 3.4 / Figure 5 and Table 2: the pipeline's hyperparameters.  Recall of the exhaustive top-k by the full
pipeline over a grid of t_cs and ndocs: insensitive to t_cs as long as the threshold sits between the small tail of
high centroid scores and the bulk (the calibrated generator's centroid scores are bimodal: a query token's own
centroid scores about 0.9, every other one below 0.4), collapsing once the threshold cuts into the tail, and growing
with ndocs.

The CPU test computes both from the oracle alone on a few queries of cfg1; the GPU tests compute them with the library
on all of cfg1 and on a sample of cfg2, where the exhaustive ranking is the library's own pipeline with every filter
switched off (nprobe = C, t_cs = -inf, ndocs = 4 P: equal to exhaustive MaxSim, which the parity tests check against
the oracle at small sizes).  Thresholds are stated next to each assertion.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from synth import get_config, make_workload

K_DEPTHS = (1, 2, 5, 10)


def _recall(found, truth):
    truth = set(int(i) for i in truth if i >= 0)
    return len(truth & set(int(i) for i in found if i >= 0)) / max(1, len(truth))


# ------------------------------------------------------------------ oracle only (CPU)
def test_oracle_recall_on_cfg1(cfg1_calibrated):
    w = cfg1_calibrated
    cfg = w.cfg
    ix = orc.Index(w.numpy(), cfg.nbits)
    allp = np.arange(cfg.P, dtype=np.int32)
    k = cfg.k
    depth = {m: [] for m in K_DEPTHS}
    grid = {}
    for q in range(4):
        Q = w.queries[q].numpy()
        truth, _ = orc.exhaustive(ix, Q, k)
        ci = orc.centroid_interaction(orc.scq(ix.centroids, Q), allp, ix, None)
        order = np.lexsort((allp, -ci.astype(np.float64)))
        for m in K_DEPTHS:
            depth[m].append(_recall(order[:m * k], truth))
        for t_cs in (-np.inf, cfg.t_cs, 0.97):
            for ndocs in (4 * k, 64, 256):
                ids, _ = orc.search(ix, Q, cfg.nprobe, t_cs, ndocs, k)
                grid.setdefault((t_cs, ndocs), []).append(_recall(ids, truth))
    depth = {m: float(np.mean(v)) for m, v in depth.items()}
    grid = {key: float(np.mean(v)) for key, v in grid.items()}
    print("centroid-only recall of the exhaustive top-%d within depth m*k:" % k, depth)
    print("pipeline recall over (t_cs, ndocs):", grid)
    assert depth[10] >= 0.99, "Section 3.3: 10 k passages found with centroids alone hold 99+ % of the exhaustive top k"
    assert depth[1] <= depth[2] <= depth[5] <= depth[10]
    assert grid[(cfg.t_cs, cfg.ndocs)] >= 0.95, "Table 2's setting for this k loses (almost) nothing"
    for t_cs in (-np.inf, cfg.t_cs):   # more candidates kept by stage 2 never hurt at these thresholds
        assert grid[(t_cs, 4 * k)] <= grid[(t_cs, 64)] + 1e-9 <= grid[(t_cs, 256)] + 2e-9
    assert grid[(0.97, 256)] < grid[(cfg.t_cs, 256)], "a threshold inside the tail of high centroid scores prunes what matters"


# ------------------------------------------------------------------ the library (GPU)
def _library_recall(cfg_name, queries, t_grid, ndocs_grid):
    import paper_2205_09707_amd as pl
    pl.load_library()
    cfg = get_config(cfg_name)
    dev = torch.device("cuda:0")
    w = make_workload(cfg, device=dev, noise="calibrated")
    names = ("centroids", "doc_offsets", "codes", "residuals", "bucket_weights", "ivf_offsets", "ivf_pids")
    gidx = pl.plaid_index_from_view({n: getattr(w, n) for n in names}, cfg.nbits, device=0, copy=False)
    try:
        Q = w.queries[queries].contiguous()
        k, P, C = cfg.k, cfg.P, cfg.C
        # every filter off: the exhaustive MaxSim ranking
        truth, _ = pl.plaid_search(gidx, Q, C, -np.inf, 4 * P, k)
        # centroids alone: with t_cs = -inf stage 2 and stage 3 rank by the same unpruned centroid interaction, so the
        # passages stage 3 keeps out of ndocs = 4 k' are the centroid-only top k'
        depth = {}
        for m in K_DEPTHS:
            _, _, b = pl.plaid_search_debug(gidx, Q, C, -np.inf, 4 * m * k, k, want=("sel3_ids", "n3"))
            torch.cuda.synchronize()
            sel3, n3 = b["sel3_ids"].cpu().numpy(), b["n3"].cpu().numpy()
            depth[m] = float(np.mean([_recall(sel3[j, :n3[j]], truth[j].cpu().numpy()) for j in range(len(queries))]))
        grid = {}
        for t_cs in t_grid:
            for ndocs in ndocs_grid:
                ids, _ = pl.plaid_search(gidx, Q, cfg.nprobe, t_cs, ndocs, k)
                torch.cuda.synchronize()
                grid[(t_cs, ndocs)] = float(np.mean([_recall(ids[j].cpu().numpy(), truth[j].cpu().numpy())
                                                     for j in range(len(queries))]))
        return cfg, w, truth.cpu().numpy(), depth, grid
    finally:
        pl.plaid_index_free(gidx)


@pytest.mark.gpu
def test_library_recall_on_cfg1():
    qs = list(range(16))
    t_grid = (-np.inf, 0.3, 0.5, 0.7, 0.97)
    cfg, w, truth, depth, grid = _library_recall("cfg1", qs, t_grid, (40, 64, 256, 1024))
    print("cfg1 centroid-only recall within depth m*k:", depth)
    for t in t_grid:
        print(f"cfg1 pipeline recall, t_cs={t}:", {n: round(grid[(t, n)], 3) for n in (40, 64, 256, 1024)})
    assert depth[10] >= 0.99 and depth[1] <= depth[2] <= depth[5] <= depth[10]
    assert grid[(cfg.t_cs, cfg.ndocs)] >= 0.95
    for t in (-np.inf, 0.3, 0.5, 0.7):
        assert grid[(t, 40)] <= grid[(t, 64)] + 1e-9 <= grid[(t, 256)] + 2e-9 <= grid[(t, 1024)] + 3e-9
        assert abs(grid[(t, 256)] - grid[(0.5, 256)]) <= 0.02, "flat between the tail and the bulk of the centroid scores"
    assert grid[(0.97, 256)] < grid[(0.5, 256)]
    # the exhaustive ranking the recalls refer to is the oracle's (4 queries; ids may swap only inside score ties)
    ix = orc.Index(w.numpy(), cfg.nbits)
    Qh = w.queries.cpu().numpy()
    for q in range(4):
        o_ids, _ = orc.exhaustive(ix, Qh[q], cfg.k)
        assert _recall(truth[q], o_ids) >= 1.0 - 1.0 / cfg.k


@pytest.mark.gpu
def test_library_recall_on_cfg2():
    rng = np.random.default_rng(7)
    qs = sorted(rng.choice(256, size=24, replace=False).tolist())
    t_grid = (-np.inf, 0.5, 0.97)
    cfg, w, truth, depth, grid = _library_recall("cfg2", qs, t_grid, (40, 256, 1024))
    print("cfg2 centroid-only recall within depth m*k:", depth)
    for t in t_grid:
        print(f"cfg2 pipeline recall, t_cs={t}:", {n: round(grid[(t, n)], 3) for n in (40, 256, 1024)})
    assert depth[10] >= 0.99 and depth[1] <= depth[2] <= depth[5] <= depth[10]
    assert grid[(cfg.t_cs, cfg.ndocs)] >= 0.95
    for t in (-np.inf, 0.5):
        assert grid[(t, 40)] <= grid[(t, 256)] + 1e-9 <= grid[(t, 1024)] + 2e-9
    assert grid[(0.97, 256)] < grid[(0.5, 256)]
