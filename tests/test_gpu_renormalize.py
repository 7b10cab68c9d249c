"""GPU parity of the storage variant "reconstructed vectors scaled back to unit length" (plaid_index_set_renormalize)
against the oracle's routine for it.

Bit-exact: the reconstructed vectors plaid_decompress_passages returns (one fp32 factor per token from a
double-precision sum of squares, one rounding per component).  Stages 1-3 use centroids only, so the passages that
reach stage 4 are those of the plain reading; the final scores are checked against the oracle's Eq. 1 on the scaled
vectors for exactly those passages, within the score tolerance, and the ids under the tie rule."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from synth import get_config, make_workload, tiny_config

import parity_util as pu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pl():
    import paper_2205_09707_amd as pl_
    pl_.load_library()
    return pl_


def _check(pl, w, cases, decompress_pids):
    ix = pu.oracle_index(w)
    ixr = ix.renormalized()
    gidx = pl.plaid_index_from_view(pu.device_arrays(w), w.cfg.nbits, device=0, copy=True)
    Qd = w.queries.to(DEV)
    Qh = w.queries.numpy()
    try:
        plain = {c: pl.plaid_search(gidx, Qd, *c) for c in cases}
        torch.cuda.synchronize()
        pl.plaid_index_set_renormalize(gidx, True)
        # reconstructed vectors, bit for bit
        pids = torch.tensor(decompress_pids, dtype=torch.int32, device=DEV)
        cap = int(sum(ix.doc_offsets[p + 1] - ix.doc_offsets[p] for p in decompress_pids))
        offs, vec, _ = pl.plaid_decompress_passages(gidx, pids, max(cap, 1), indices=False)
        vec, offs = vec.cpu().numpy(), offs.cpu().numpy()
        for a, p in enumerate(decompress_pids):
            t0, t1 = int(ix.doc_offsets[p]), int(ix.doc_offsets[p + 1])
            D, _ = orc.decompress(ixr, t0, t1)
            np.testing.assert_array_equal(vec[offs[a]:offs[a + 1]], D, err_msg=f"passage {p}")
        for case in cases:
            nprobe, t_cs, ndocs, k = case
            print(f"[renormalize] {w.cfg.name} {case}", flush=True)
            ids, sc, b = pl.plaid_search_debug(gidx, Qd, nprobe, t_cs, ndocs, k, want=("sel3_ids", "n3"))
            torch.cuda.synchronize()
            ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
            sel3, n3 = b["sel3_ids"].cpu().numpy(), b["n3"].cpu().numpy()
            for q in range(Qh.shape[0]):
                kept = np.sort(sel3[q, :n3[q]])
                s4 = orc.maxsim(ixr, Qh[q], kept)
                same = pu.assert_final_matches(ids[q], sc[q], kept, s4, k, ctx=f"{w.cfg.name} {case} q{q}")
                if same:  # the whole pipeline under the variant, when the oracle's stage 3 kept the same passages
                    o_ids, _, d = orc.search(ixr, Qh[q], nprobe, t_cs, ndocs, k, dumps=True)
                    if np.array_equal(np.sort(d["sel3_ids"]), kept):
                        np.testing.assert_array_equal(ids[q], o_ids)
        # switched off again: the plain reading's results, bit for bit
        pl.plaid_index_set_renormalize(gidx, False)
        for c in cases:
            ids, sc = pl.plaid_search(gidx, Qd, *c)
            assert torch.equal(ids, plain[c][0]) and torch.equal(sc, plain[c][1])
        # the baseline is not offered under the variant
        pl.plaid_index_set_renormalize(gidx, True)
        with pytest.raises(pl.PlaidError) as e:
            pl.plaid_search_vanilla(gidx, Qd, 1, 100, 5)
        assert e.value.status == pl.plaid.PLAID_EINVAL
    finally:
        pl.plaid_index_free(gidx)


@pytest.mark.parametrize("noise", ["calibrated", "literal"])
def test_cfg1(pl, noise):
    cfg = get_config("cfg1")
    w = make_workload(cfg, device="cpu", noise=noise)
    _check(pl, w, [(cfg.nprobe, cfg.t_cs, cfg.ndocs, cfg.k), (4, 0.3, 64, 10), (1, -np.inf, 4 * cfg.P, 20)], [0, 7, cfg.P - 1])


@pytest.mark.parametrize("C,P,lo,hi,nbits,seed,nq", [
    (16, 50, 1, 9, 2, 1, 4),
    (70, 321, 0, 40, 1, 5, 4),        # empty passages, 1-bit residuals
    (33, 200, 1, 130, 2, 4, 3),       # passages of several steps
    (50, 6, 2300, 2400, 1, 32, 2),    # very long passages
    (1, 9, 1, 5, 2, 6, 3),            # a single centroid
])
def test_small_indexes(pl, C, P, lo, hi, nbits, seed, nq):
    w = make_workload(tiny_config(C=C, P=P, lo=lo, hi=hi, nbits=nbits, nq=nq, seed=seed), noise="calibrated")
    _check(pl, w, [(min(2, C), 0.2, 8, 3), (C, -np.inf, 4 * P, 5), (1, 0.5, 1, 1)], [0, P // 2, P - 1])


def test_zero_vectors_stay_zero(pl):
    """A token whose reconstruction is the zero vector has no direction: factor 0, dot products 0."""
    dim, P = 128, 4
    cen = np.zeros((2, dim), np.float32)
    cen[1, 3] = 2.0
    arrays = dict(centroids=cen, doc_offsets=np.array([0, 1, 2, 4, 4], np.int64), codes=np.array([0, 1, 0, 1], np.int32),
                  residuals=np.zeros((4, dim // 4), np.uint8), bucket_weights=np.zeros(4, np.float32),
                  ivf_offsets=np.array([0, 2, 4], np.int64), ivf_pids=np.array([0, 2, 1, 2], np.int32))
    ixr = orc.Index(arrays, 2, renormalize=True)
    view = {n: torch.from_numpy(a).to(DEV) for n, a in arrays.items()}
    gidx = pl.plaid_index_from_view(view, 2, device=0, copy=True)
    try:
        pl.plaid_index_set_renormalize(gidx, True)
        Q = np.zeros((1, 32, dim), np.float32)
        Q[:, :, 3] = 1.0
        ids, sc = pl.plaid_search(gidx, torch.from_numpy(Q).to(DEV), 2, -np.inf, 16, 4)
        o_ids, o_sc = orc.search(ixr, Q[0], 2, -np.inf, 16, 4)
        np.testing.assert_array_equal(ids[0].cpu().numpy(), o_ids)
        np.testing.assert_allclose(sc[0].cpu().numpy(), o_sc, atol=pu.TOL)
    finally:
        pl.plaid_index_free(gidx)
