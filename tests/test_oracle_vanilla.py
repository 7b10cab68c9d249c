"""Pins of the oracle's vanilla ColBERTv2 retrieval (the paper's baseline: Sections 3.1-3.2, 4.1).

* embedding-level lists against numpy's stable argsort of the codes;
* the candidate passages against the passage-level candidates of the same probes (a passage owns an embedding of a
  probed centroid's list exactly when it is in that centroid's passage list);
* nothing filtered (nprobe = C, ncandidates >= P)  ==>  vanilla == exhaustive MaxSim;
* the pruning scores against numpy on the decompressed embeddings of E, never above exact MaxSim, equal to it for a
  passage all of whose tokens are in E; the kept set against a full sort;
* the hand example of test_oracle_hand_example.py, continued by hand:
    embedding lists: c0 -> {t0, t1}, c1 -> {t2}, c2 -> {t3, t4}.
    nprobe = 2: every centroid is probed, E = all five tokens, candidates {0, 1, 2}; the pruning scores are then the
      exact ones (9/4 for p1, 5/4 for p0 and p2), so ncandidates = 2 keeps p1 and, of the tie, the smaller pid p0.
    nprobe = 1: q0 probes c0, q1 probes c1, E = {t0, t1, t2}, candidates {0, 1}.  Pruning scores: p0 from t0, t1:
      max(1, 3/4) + max(0, 1/4) = 5/4;  p1 from t2 = (0, 3/2, 0, 0) alone: 0 + 3/2 = 3/2.  ncandidates = 1 keeps p1,
      whose exact score over both its tokens is 9/4.
"""
import json
import os

import numpy as np
import pytest

from oracle import oracle as orc
from synth import make_workload, tiny_config

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_example.json")


def _tiny(seed, C=24, P=120, lo=1, hi=14, nq=4, nbits=2):
    w = make_workload(tiny_config(C=C, P=P, lo=lo, hi=hi, nbits=nbits, nq=nq, seed=seed), noise="calibrated")
    return w, orc.Index(w.numpy(), nbits)


def test_embedding_lists_are_a_stable_sort_of_the_codes():
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 17, size=5000).astype(np.int32)
    codes[codes == 5] = 6                      # an empty list in the middle
    off, eids = orc.build_ivf_embeddings(codes, 17)
    np.testing.assert_array_equal(eids, np.argsort(codes, kind="stable"))
    np.testing.assert_array_equal(off, np.concatenate([[0], np.cumsum(np.bincount(codes, minlength=17))]))


@pytest.mark.parametrize("seed,nprobe", [(1, 1), (2, 3), (3, 24)])
def test_candidates_equal_the_passage_level_candidates(seed, nprobe):
    w, ix = _tiny(seed)
    eoff, eids = orc.build_ivf_embeddings(ix.codes, ix.C)
    for q in range(w.queries.shape[0]):
        Q = w.queries[q].numpy()
        _, _, d = orc.vanilla_search(ix, eoff, eids, Q, nprobe, 10 ** 6, 5, dumps=True)
        probed = orc.top_nprobe(orc.scq(ix.centroids, Q), nprobe)
        np.testing.assert_array_equal(d["cand"], orc.candidates(probed, ix))
        assert d["n_embeddings"] == int(np.isin(ix.codes, np.unique(probed)).sum())
        assert not d["pruned"]
        np.testing.assert_array_equal(d["kept"], d["cand"])


def test_nothing_filtered_is_exhaustive_search():
    w, ix = _tiny(4, C=16, P=90, lo=0, hi=20)
    eoff, eids = orc.build_ivf_embeddings(ix.codes, ix.C)
    for q in range(w.queries.shape[0]):
        Q = w.queries[q].numpy()
        ids, sc = orc.vanilla_search(ix, eoff, eids, Q, ix.C, ix.P, 12)
        e_ids, e_sc = orc.exhaustive(ix, Q, 12)
        # (passages without tokens never become candidates; exhaustive ranks them last at -inf: none among the best 12)
        np.testing.assert_array_equal(ids, e_ids)
        np.testing.assert_array_equal(sc, e_sc)


@pytest.mark.parametrize("seed,nprobe,ncand", [(5, 2, 7), (6, 1, 3), (7, 4, 20)])
def test_pruning_scores_and_kept_set(seed, nprobe, ncand):
    w, ix = _tiny(seed, C=40, P=150, lo=1, hi=18)
    eoff, eids = orc.build_ivf_embeddings(ix.codes, ix.C)
    do = ix.doc_offsets
    for q in range(w.queries.shape[0]):
        Q = w.queries[q].numpy()
        ids, sc, d = orc.vanilla_search(ix, eoff, eids, Q, nprobe, ncand, 5, dumps=True)
        if len(d["cand"]) <= ncand:
            assert not d["pruned"]
            continue
        assert d["pruned"] and len(d["kept"]) == ncand
        probed = np.unique(orc.top_nprobe(orc.scq(ix.centroids, Q), nprobe))
        Q64 = Q.astype(np.float64)
        want = {}
        for p in d["cand"]:
            D, _ = orc.decompress(ix, int(do[p]), int(do[p + 1]))
            inE = np.isin(ix.codes[do[p]:do[p + 1]], probed)
            assert inE.any()
            dots = (Q64 @ D[inE].astype(np.float64).T).astype(np.float32)     # [32, |E in p|]
            want[int(p)] = np.float32(dots.max(axis=1).astype(np.float64).sum())
            exact = orc.maxsim(ix, Q, np.array([p], np.int32))[0]
            assert want[int(p)] <= exact + 1e-6
            if inE.all():
                assert abs(want[int(p)] - exact) <= 1e-6
        order = sorted(want, key=lambda p: (-float(want[p]), p))
        cut = float(want[order[ncand - 1]])
        kept = set(d["kept"].tolist())
        for p in order:   # the kept set is the full sort's head, up to ties in the last few bits of the scores
            if float(want[p]) > cut + 1e-6:
                assert p in kept
            if float(want[p]) < cut - 1e-6:
                assert p not in kept
        for p, s in zip(d["kept"], d["kept_scores"]):
            assert abs(float(s) - float(want[int(p)])) <= 1e-6
        assert np.all(np.diff(d["kept"]) > 0)
        # the final ranking is exact MaxSim over the kept passages
        s4 = orc.maxsim(ix, Q, d["kept"])
        top = np.lexsort((d["kept"], -s4.astype(np.float64)))[:5]
        np.testing.assert_array_equal(ids[:len(top)], d["kept"][top])
        np.testing.assert_array_equal(sc[:len(top)], s4[top])


def test_hand_example():
    g = json.load(open(GOLD))
    ivf_off = np.cumsum([0] + [len(l) for l in g["ivf"]]).astype(np.int64)
    arrays = dict(centroids=np.array(g["centroids"], np.float32), doc_offsets=np.array(g["doc_offsets"], np.int64),
                  codes=np.array(g["codes"], np.int32), residuals=np.array(g["packed_bytes"], np.uint8).reshape(-1, 1),
                  bucket_weights=np.array(g["bucket_weights"], np.float32), ivf_offsets=ivf_off,
                  ivf_pids=np.array([p for l in g["ivf"] for p in l], np.int32))
    ix = orc.Index(arrays, g["nbits"])
    Q = np.array(g["Q"], np.float32)
    eoff, eids = orc.build_ivf_embeddings(ix.codes, 3)
    np.testing.assert_array_equal(eoff, [0, 2, 3, 5])
    np.testing.assert_array_equal(eids, [0, 1, 2, 3, 4])
    ninf = -np.inf
    # nprobe = 2, no pruning needed
    ids, sc, d = orc.vanilla_search(ix, eoff, eids, Q, 2, 3, 2, dumps=True)
    np.testing.assert_array_equal(d["cand"], [0, 1, 2])
    assert d["n_embeddings"] == 5 and not d["pruned"]
    np.testing.assert_array_equal(ids, [1, 0])
    np.testing.assert_array_equal(sc, np.array([2.25, 1.25], np.float32))
    # nprobe = 2, ncandidates = 2: the tie at 5/4 keeps the smaller pid
    ids, sc, d = orc.vanilla_search(ix, eoff, eids, Q, 2, 2, 3, dumps=True)
    assert d["pruned"]
    np.testing.assert_array_equal(d["kept"], [0, 1])
    np.testing.assert_array_equal(d["kept_scores"], np.array([1.25, 2.25], np.float32))
    np.testing.assert_array_equal(ids, [1, 0, -1])
    np.testing.assert_array_equal(sc, np.array([2.25, 1.25, ninf], np.float32))
    # nprobe = 1, ncandidates = 1: pruned on the embeddings of the probed lists only
    ids, sc, d = orc.vanilla_search(ix, eoff, eids, Q, 1, 1, 2, dumps=True)
    np.testing.assert_array_equal(d["cand"], [0, 1])
    assert d["n_embeddings"] == 3 and d["pruned"]
    np.testing.assert_array_equal(d["kept"], [1])
    np.testing.assert_array_equal(d["kept_scores"], np.array([1.5], np.float32))
    np.testing.assert_array_equal(ids, [1, -1])
    np.testing.assert_array_equal(sc, np.array([2.25, ninf], np.float32))


def test_argument_errors():
    w, ix = _tiny(8)
    eoff, eids = orc.build_ivf_embeddings(ix.codes, ix.C)
    Q = w.queries[0].numpy()
    for bad in ((0, 5, 3), (ix.C + 1, 5, 3), (1, 0, 3), (1, 5, 0)):
        with pytest.raises(ValueError):
            orc.vanilla_search(ix, eoff, eids, Q, *bad)
