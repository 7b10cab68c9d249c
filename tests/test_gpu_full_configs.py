"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py times.

The index is generated on the GPU (seeded), handed to the library without a copy, and searched (a) with the
whole query batch in one call and (b) one query per call; a sample of queries is then recomputed by the CPU
oracle from host copies of the same buffers and compared stage by stage.  cfg4 / cfg5 (0.6 and 1.4 billion
embeddings, 22 and 28 GB of index) run like the others; they are skipped only when the device or the host lacks the
memory to hold the index (stated in the skip reason).
"""
import os

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from synth import get_config, make_workload

import parity_util as pu

pytestmark = pytest.mark.gpu


def _memory_shortfall(cfg):
    """None when the configuration fits, else the reason it does not: the index (codes, residuals, inverted lists) must
    fit the free device memory three times over (generation temporaries, the library's workspace of up to 24 GiB) and
    the host's available memory twice (the oracle works on host copies of the same arrays)."""
    import psutil
    mean_len = {"cfg4": 68, "cfg5": 70}.get(cfg.name, 70)
    index_bytes = cfg.P * mean_len * (4 + 16 * cfg.nbits + 4)
    free_dev, _ = torch.cuda.mem_get_info(0)
    if free_dev < 3 * index_bytes:
        return f"{cfg.name}: {free_dev / 2**30:.0f} GiB of free device memory, {3 * index_bytes / 2**30:.0f} GiB wanted"
    avail = psutil.virtual_memory().available
    if avail < 2 * index_bytes:
        return f"{cfg.name}: {avail / 2**30:.0f} GiB of host memory available, {2 * index_bytes / 2**30:.0f} GiB wanted"
    return None


def _run(cfg_name, noise, n_sample, n_dump, stage2=None, form=None):
    """stage2: None = the library's choice of the stage-2 form, "stream" / "inverted" = forced (PLAID_STAGE2_FORM);
    form: None = the library's choice of the score kernel (split-fp16), "matrix" = the double-precision one."""
    import paper_2205_09707_amd as pl
    pl.load_library()
    cfg = get_config(cfg_name)
    dev = torch.device("cuda:0")
    print(f"[full] generating {cfg_name}/{noise}", flush=True)
    w = make_workload(cfg, device=dev, noise=noise)
    names = ("centroids", "doc_offsets", "codes", "residuals", "bucket_weights", "ivf_offsets", "ivf_pids")
    from test_gpu_parity import _kernel_forms
    with _kernel_forms(form, stage2):
        gidx = pl.plaid_index_from_view({n: getattr(w, n) for n in names}, cfg.nbits, device=0, copy=False)
    if form is not None:
        assert pl.plaid_get_score_kernel(gidx) == {"vector": 0, "matrix": 1, "split16": 2}[form]
    if stage2 is not None:
        assert bool(pl.plaid_get_stage2_kernel(gidx)) == stage2.startswith("inverted")
    print(f"[full] {cfg_name}/{noise}: stage-2 form {('stream', 'inverted, 2048 passages per workgroup', 'inverted, 8192 passages per workgroup')[pl.plaid_get_stage2_kernel(gidx)]}",
          flush=True)
    params = (cfg.nprobe, cfg.t_cs, cfg.ndocs, cfg.k)
    Q = w.queries
    nq = Q.shape[0]
    try:
        print(f"[full] {cfg_name}/{noise}: N={w.N}, batch search of {nq} queries", flush=True)
        ids, sc = pl.plaid_search(gidx, Q, *params)
        torch.cuda.synchronize()
        rng = np.random.default_rng(cfg.query_seed)
        sample = sorted(rng.choice(nq, size=min(n_sample, nq), replace=False).tolist())
        # (b) one query per call must give the same bits as the batch
        for q in sample:
            i1, s1 = pl.plaid_search(gidx, Q[q:q + 1], *params)
            assert torch.equal(i1[0], ids[q]) and torch.equal(s1[0], sc[q]), f"batch-1 differs from batch at q{q}"
        ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
        ix = orc.Index(w.numpy(), cfg.nbits)
        Qh = Q.cpu().numpy()
        identical = 0
        for n, q in enumerate(sample):
            g = dict(ids=ids[q], scores=sc[q])
            if n < n_dump:   # stage-by-stage dumps for a few queries (S_cq alone is 128*C bytes per query)
                out = pu.run_gpu_debug(pl, gidx, Q[q:q + 1], params)
                g = pu.slice_query(out, 0)
                assert np.array_equal(g["ids"], ids[q]) and np.array_equal(pu.bits(g["scores"]), pu.bits(sc[q]))
            print(f"[full] {cfg_name}/{noise} q{q} vs oracle", flush=True)
            identical += bool(pu.compare_query(ix, Qh[q], params, g, ctx=f"{cfg_name}/{noise} q{q}",
                                               approx=pu.is_approx(pl, gidx, params)))
        # informational: with k = 1000 a few adjacent ranks whose oracle scores differ by less than the fp32
        # accumulation error (about 1e-6) are expected to swap; compare_query has already checked that every
        # difference lies inside such a near-tie and that every score is within TOL
        print(f"[full] {cfg_name}/{noise}: {identical}/{len(sample)} sampled queries with id lists identical to the oracle's; "
              f"largest deviations so far (split-fp16 score kernel): {pu.MEASURED}", flush=True)
    finally:
        pl.plaid_index_free(gidx)
        del w
        torch.cuda.empty_cache()


@pytest.mark.parametrize("cfg_name,noise,stage2,form", [("cfg2", "literal", None, None), ("cfg2", "calibrated", None, None),
                                                        ("cfg3", "literal", None, None), ("cfg3", "calibrated", None, None),
                                                        ("cfg3", "literal", "stream", None),
                                                        ("cfg3", "calibrated", "stream", None),
                                                        ("cfg3", "calibrated", None, "matrix")])
def test_mid_configs(cfg_name, noise, stage2, form):
    _run(cfg_name, noise, n_sample=12, n_dump=3, stage2=stage2, form=form)


@pytest.mark.parametrize("cfg_name,noise", [("cfg4", "literal"), ("cfg4", "calibrated"), ("cfg5", "literal"),
                                            ("cfg5", "calibrated")])
def test_big_configs(cfg_name, noise):
    short = _memory_shortfall(get_config(cfg_name))
    if short:
        pytest.skip(short)
    _run(cfg_name, noise, n_sample=4, n_dump=1)


@pytest.mark.parametrize("cfg_name", ["cfg2", "cfg3"])
def test_index_construction_at_full_size(cfg_name):
    """The index-construction calls at the configuration's real sizes, as bench.py times them: the inverted lists of all
    tokens against the oracle's, the residual encoding of the first 2^20 tokens against the oracle's, nearest centroids
    of 2048 sampled token vectors against the oracle's S_cq + top-1."""
    import paper_2205_09707_amd as pl
    pl.load_library()
    cfg = get_config(cfg_name)
    dev = torch.device("cuda:0")
    print(f"[build] generating {cfg_name}", flush=True)
    w = make_workload(cfg, device=dev, noise="literal", keep_embeddings=1 << 20)
    x = w.sample_embeddings
    n = x.shape[0]
    print(f"[build] {cfg_name}: inverted lists of N={w.N} tokens", flush=True)
    off, pids = pl.plaid_build_ivf(w.codes, w.doc_offsets, cfg.C)
    torch.cuda.synchronize()
    o_off, o_pids = orc.build_ivf(w.codes.cpu().numpy(), w.doc_offsets.cpu().numpy(), cfg.C)
    np.testing.assert_array_equal(off.cpu().numpy(), o_off)
    np.testing.assert_array_equal(pids.cpu().numpy(), o_pids)
    print(f"[build] {cfg_name}: residual encoding of {n} tokens", flush=True)
    res = pl.plaid_encode_residuals(w.centroids, x, w.codes[:n].contiguous(), w.bucket_cutoffs.to(dev), cfg.nbits)
    torch.cuda.synchronize()
    want = orc.encode(x.cpu().numpy(), w.codes[:n].cpu().numpy(), w.centroids.cpu().numpy(), w.bucket_cutoffs.cpu().numpy(),
                      cfg.nbits)
    np.testing.assert_array_equal(res.cpu().numpy(), want)
    print(f"[build] {cfg_name}: nearest centroids of {n} tokens, 2048 of them checked", flush=True)
    codes = pl.plaid_assign_centroids(w.centroids, x)
    torch.cuda.synchronize()
    rng = np.random.default_rng(cfg.index_seed)
    groups = sorted(rng.choice(n // 32, size=64, replace=False).tolist())
    cen = w.centroids.cpu().numpy()
    xh = x.cpu().numpy()
    got = codes.cpu().numpy()
    for g in groups:
        S = orc.scq(cen, xh[32 * g:32 * g + 32])
        np.testing.assert_array_equal(got[32 * g:32 * g + 32], orc.top_nprobe(S, 1)[:, 0], err_msg=f"group {g}")
