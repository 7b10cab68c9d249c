"""GPU parity of plaid_search_vanilla (vanilla ColBERTv2 retrieval, the paper's baseline) against the oracle's routine.

Bit-exact: the candidate passages (embedding lists of the probed centroids -> passages).  Within tolerance: the pruning
scores (fp16-split matrix arithmetic on decompressed residuals plus the S_cq rows) and therefore the set kept by the
ncandidates cap, which may differ from the oracle's only among candidates whose oracle scores lie within TOL of the
cut; the final ranking is checked on the set the library kept.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from synth import get_config, make_workload, tiny_config

import parity_util as pu
from test_gpu_parity import _kernel_forms

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _check(pl, w, cases, queries=None, form=None, max_chunk=None):
    ix = pu.oracle_index(w)
    eoff, eids = orc.build_ivf_embeddings(ix.codes, ix.C)
    with _kernel_forms(form, None):
        gidx = pl.plaid_index_from_view(pu.device_arrays(w), w.cfg.nbits, device=0, copy=True)
    if max_chunk is not None:
        pl.plaid_set_max_chunk(gidx, max_chunk)
    Qd = w.queries.to(DEV)
    Qh = w.queries.numpy()
    try:
        for nprobe, ncand, k in cases:
            print(f"[vanilla] {w.cfg.name} nprobe={nprobe} ncandidates={ncand} k={k}", flush=True)
            ids, sc, b = pl.plaid_search_vanilla(gidx, Qd, nprobe, ncand, k, debug=True)
            torch.cuda.synchronize()
            ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
            b = {n: t.cpu().numpy() for n, t in b.items()}
            for q in (range(Qh.shape[0]) if queries is None else queries):
                ctx = f"{w.cfg.name} ({nprobe},{ncand},{k}) q{q}"
                o_ids, o_sc, d = orc.vanilla_search(ix, eoff, eids, Qh[q], nprobe, ncand, k, dumps=True)
                cand = b["cand"][q, :b["n_cand"][q]]
                assert np.array_equal(cand, d["cand"]), f"{ctx}: candidates differ"
                kept = b["kept_ids"][q, :b["n_kept"][q]]
                if not d["pruned"]:
                    assert np.array_equal(np.sort(kept), d["cand"]), f"{ctx}: nothing to prune, yet the kept set differs"
                else:
                    probed = orc.top_nprobe(orc.scq(ix.centroids, Qh[q]), nprobe)
                    ps = orc.vanilla_prune_scores(ix, Qh[q], probed, d["cand"])
                    pu.assert_selection_matches(kept, b["kept_scores"][q, :len(kept)], d["cand"], ps, ncand, pu.TOL, pu.TOL,
                                                ctx=f"{ctx}: kept")
                kept = np.sort(kept)
                s4 = orc.maxsim(ix, Qh[q], kept)
                same = pu.assert_final_matches(ids[q], sc[q], kept, s4, k, ctx=ctx)
                if same and np.array_equal(kept, d["kept"]):
                    assert np.array_equal(ids[q], o_ids), f"{ctx}: ids"
    finally:
        pl.plaid_index_free(gidx)


@pytest.fixture(scope="module")
def pl():
    import paper_2205_09707_amd as pl_
    pl_.load_library()
    return pl_


@pytest.mark.parametrize("noise", ["calibrated", "literal"])
def test_cfg1(pl, noise):
    w = make_workload(get_config("cfg1"), device="cpu", noise=noise)
    # no cap reached / the cap at work / a cap of a handful / more probes (the last beyond the fast probe kernel);
    # the oracle decompresses every embedding of the probed lists on the CPU: it checks every third query and the last
    nq = w.queries.shape[0]
    _check(pl, w, [(1, 1 << 16, 10), (2, 2048, 100), (4, 64, 10), (1, 7, 10), (12, 512, 20)],
           queries=sorted(set(range(0, nq, 3)) | {nq - 1}))


def test_nothing_filtered_is_exhaustive(pl):
    w = make_workload(tiny_config(C=48, P=150, lo=1, hi=70, nbits=2, nq=5, seed=11), noise="calibrated")
    ix = pu.oracle_index(w)
    gidx = pl.plaid_index_from_view(pu.device_arrays(w), 2, device=0, copy=True)
    try:
        k = 20
        ids, sc = pl.plaid_search_vanilla(gidx, w.queries.to(DEV), 48, 150, k)
        ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
        allp = np.arange(150, dtype=np.int32)
        for q in range(5):
            Q = w.queries[q].numpy()
            same = pu.assert_final_matches(ids[q], sc[q], allp, orc.maxsim(ix, Q, allp), k, ctx=f"exhaustive q{q}")
            if same:
                assert np.array_equal(ids[q], orc.exhaustive(ix, Q, k)[0])
    finally:
        pl.plaid_index_free(gidx)


SMALL = [
    # C, P, lo, hi, nbits, seed, nq, score kernel, queries per chunk
    (16, 50, 1, 9, 2, 1, 4, None, None),
    (70, 321, 0, 40, 1, 5, 4, "vector", None),      # empty passages, 1-bit residuals
    (33, 200, 1, 130, 2, 4, 4, "matrix", None),     # passages longer than several 64-token chunks
    (50, 6, 2300, 2400, 1, 32, 2, None, None),      # very long passages: the ring wraps many times
    (40, 5000, 1, 6, 2, 9, 7, None, 3),             # chunks of 3, 3 and 1 queries
    (1, 9, 1, 5, 2, 6, 3, None, None),              # a single centroid
]


@pytest.mark.parametrize("C,P,lo,hi,nbits,seed,nq,form,max_chunk", SMALL)
def test_small_indexes(pl, C, P, lo, hi, nbits, seed, nq, form, max_chunk):
    w = make_workload(tiny_config(C=C, P=P, lo=lo, hi=hi, nbits=nbits, nq=nq, seed=seed), noise="calibrated")
    cases = [(1, P + 5, 3), (min(2, C), max(1, P // 3), 5), (min(3, C), 1, 1), (C, 4, 9)]
    _check(pl, w, cases, form=form, max_chunk=max_chunk)


def test_cfg2_sample(pl):
    """Full size: the cap at work on 200 000 passages (the oracle decompresses the embeddings of the probed lists one by
    one, so only two queries are compared)."""
    cfg = get_config("cfg2")
    w = make_workload(cfg, device=torch.device(DEV), noise="calibrated")
    names = ("centroids", "doc_offsets", "codes", "residuals", "bucket_weights", "ivf_offsets", "ivf_pids")
    gidx = pl.plaid_index_from_view({n: getattr(w, n) for n in names}, cfg.nbits, device=0, copy=False)
    try:
        nprobe, ncand, k = 1, 4096, 10
        ids, sc, b = pl.plaid_search_vanilla(gidx, w.queries, nprobe, ncand, k, debug=True)
        torch.cuda.synchronize()
        ix = orc.Index(w.numpy(), cfg.nbits)
        eoff, eids = orc.build_ivf_embeddings(ix.codes, ix.C)
        Qh = w.queries.cpu().numpy()
        for q in (3, 200):
            print(f"[vanilla] cfg2 q{q} vs oracle", flush=True)
            o_ids, o_sc, d = orc.vanilla_search(ix, eoff, eids, Qh[q], nprobe, ncand, k, dumps=True)
            n_c = int(b["n_cand"][q])
            assert np.array_equal(b["cand"][q, :n_c].cpu().numpy(), d["cand"])
            kept = np.sort(b["kept_ids"][q, :int(b["n_kept"][q])].cpu().numpy())
            s4 = orc.maxsim(ix, Qh[q], kept)
            same = pu.assert_final_matches(ids[q].cpu().numpy(), sc[q].cpu().numpy(), kept, s4, k, ctx=f"cfg2 q{q}")
            # the kept sets agree except, at most, for candidates tied at the cut
            assert len(set(kept.tolist()) ^ set(d["kept"].tolist())) <= 4
            if same and np.array_equal(kept, d["kept"]):
                assert np.array_equal(ids[q].cpu().numpy(), o_ids)
    finally:
        pl.plaid_index_free(gidx)


def test_argument_errors(pl):
    w = make_workload(tiny_config(C=8, P=10, lo=1, hi=4, nbits=2, nq=2, seed=9), noise="literal")
    gidx = pl.plaid_index_from_view(pu.device_arrays(w), 2, device=0, copy=True)
    try:
        for bad in ((0, 4, 2), (9, 4, 2), (1, 0, 2), (1, 4, 0)):
            with pytest.raises(pl.PlaidError) as e:
                pl.plaid_search_vanilla(gidx, w.queries.to(DEV), *bad)
            assert e.value.status == pl.plaid.PLAID_EINVAL
    finally:
        pl.plaid_index_free(gidx)
