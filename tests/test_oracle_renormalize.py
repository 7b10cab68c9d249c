"""Pins of the oracle's storage variant "reconstructed vectors scaled back to unit length" (the other reading of
Section 4.5's reconstruction; Section 3.1 stores unit vectors and scores by cosine similarity).

* numpy: the plain reconstruction (pinned elsewhere) divided by its float64 norm, against the oracle's scaled vectors;
  unit length to fp32 rounding;
* scale invariance: centroids and bucket weights multiplied by a power of two (exact in fp32) give bit-identical
  scaled vectors and MaxSim scores, while the plain reading's scores scale with the factor;
* Cauchy-Schwarz: with unit-length query tokens every dot product is at most 1, so MaxSim <= 32;
* a vector built by hand: centroid (3, 4, 0, ...), zero weights: scaled to (0.6, 0.8, 0, ...); a zero vector stays zero;
* MaxSim and the vanilla pruning scores are built on the scaled vectors (numpy on the scaled vectors)."""
import numpy as np
import pytest

from oracle import oracle as orc
from synth import make_workload, tiny_config


def _tiny(seed, nbits=2, C=24, P=80, lo=1, hi=14, nq=4):
    w = make_workload(tiny_config(C=C, P=P, lo=lo, hi=hi, nbits=nbits, nq=nq, seed=seed), noise="calibrated")
    return w, orc.Index(w.numpy(), nbits)


@pytest.mark.parametrize("seed,nbits", [(1, 2), (2, 1), (3, 2)])
def test_scaled_vectors_against_numpy(seed, nbits):
    w, ix = _tiny(seed, nbits)
    D, idx = orc.decompress(ix, 0, ix.N)
    Dr, idx_r = orc.decompress(ix.renormalized(), 0, ix.N)
    np.testing.assert_array_equal(idx, idx_r)
    n = np.sqrt((D.astype(np.float64) ** 2).sum(axis=1, keepdims=True))
    want = D.astype(np.float64) / n
    assert np.abs(Dr - want).max() <= 2.0 ** -23          # two fp32 roundings: of 1/n, of the product
    assert np.abs(np.sqrt((Dr.astype(np.float64) ** 2).sum(axis=1)) - 1.0).max() <= 4e-7
    # the factor is one fp32 number per token: every component is the plain component times it, rounded once
    inv = (1.0 / n).astype(np.float32)
    np.testing.assert_array_equal(Dr, D * inv)


@pytest.mark.parametrize("k", [-3, 2, 5])
def test_scale_invariance(k):
    w, ix = _tiny(4)
    a = ix._arrays()
    a["centroids"] = (a["centroids"] * np.float32(2.0 ** k)).astype(np.float32)
    a["bucket_weights"] = (a["bucket_weights"] * np.float32(2.0 ** k)).astype(np.float32)
    ixs = orc.Index(a, ix.nbits)
    pids = np.arange(ix.P, dtype=np.int32)
    Q = w.queries[0].numpy()
    D0, _ = orc.decompress(ix.renormalized(), 0, ix.N)
    D1, _ = orc.decompress(ixs.renormalized(), 0, ix.N)
    np.testing.assert_array_equal(D0, D1)
    np.testing.assert_array_equal(orc.maxsim(ix.renormalized(), Q, pids), orc.maxsim(ixs.renormalized(), Q, pids))
    # the plain reading is not invariant: its scores scale with the vectors
    np.testing.assert_allclose(orc.maxsim(ixs, Q, pids), orc.maxsim(ix, Q, pids) * 2.0 ** k, rtol=1e-6)


def test_maxsim_is_bounded_and_built_on_the_scaled_vectors():
    w, ix = _tiny(5, nbits=1, P=60)
    ixr = ix.renormalized()
    do = ix.doc_offsets
    for q in range(w.queries.shape[0]):
        Q = w.queries[q].numpy()
        pids = np.arange(ix.P, dtype=np.int32)
        got = orc.maxsim(ixr, Q, pids)
        assert got.max() <= 32.0 * (1 + 1e-6)
        for p in range(0, ix.P, 7):
            Dr, _ = orc.decompress(ixr, int(do[p]), int(do[p + 1]))
            dots = (Q.astype(np.float64) @ Dr.astype(np.float64).T).astype(np.float32)
            want = np.float32(dots.max(axis=1).astype(np.float64).sum())
            assert abs(float(got[p]) - float(want)) <= 1e-6
        # exhaustive search and the pipeline with every filter off rank by the same scores
        e_ids, e_sc = orc.exhaustive(ixr, Q, 8)
        order = np.lexsort((pids, -got.astype(np.float64)))[:8]
        np.testing.assert_array_equal(e_ids, pids[order])
        s_ids, s_sc = orc.search(ixr, Q, ix.C, -np.inf, 4 * ix.P, 8)
        np.testing.assert_array_equal(s_ids, e_ids)
        np.testing.assert_array_equal(s_sc, e_sc)


def test_hand_built_vectors():
    dim = 128
    cen = np.zeros((2, dim), np.float32)
    cen[0, 0], cen[0, 1] = 3.0, 4.0          # length 5 -> (0.6, 0.8)
    arrays = dict(centroids=cen, doc_offsets=np.array([0, 1, 2], np.int64), codes=np.array([0, 1], np.int32),
                  residuals=np.zeros((2, dim // 4), np.uint8), bucket_weights=np.zeros(4, np.float32),
                  ivf_offsets=np.array([0, 1, 2], np.int64), ivf_pids=np.array([0, 1], np.int32))
    ix = orc.Index(arrays, 2, renormalize=True)
    D, _ = orc.decompress(ix, 0, 2)
    want = np.zeros(dim, np.float32)
    want[0], want[1] = np.float32(3.0) * np.float32(0.2), np.float32(4.0) * np.float32(0.2)
    np.testing.assert_array_equal(D[0], want)
    np.testing.assert_array_equal(D[1], np.zeros(dim, np.float32))     # a zero vector has no direction: it stays zero
    Q = np.zeros((32, dim), np.float32)
    Q[:, 0] = 1.0
    sc = orc.maxsim(ix, Q, np.array([0, 1], np.int32))
    assert abs(float(sc[0]) - 32 * 0.6) <= 1e-5 and float(sc[1]) == 0.0


def test_vanilla_pruning_scores_use_the_scaled_vectors():
    w, ix = _tiny(6, C=30, P=90, hi=16)
    ixr = ix.renormalized()
    Q = w.queries[1].numpy()
    probed = np.unique(orc.top_nprobe(orc.scq(ix.centroids, Q), 2))
    cand = orc.candidates(orc.top_nprobe(orc.scq(ix.centroids, Q), 2), ix)
    got = orc.vanilla_prune_scores(ixr, Q, orc.top_nprobe(orc.scq(ix.centroids, Q), 2), cand)
    do = ix.doc_offsets
    for p, s in zip(cand[:20], got[:20]):
        Dr, _ = orc.decompress(ixr, int(do[p]), int(do[p + 1]))
        inE = np.isin(ix.codes[do[p]:do[p + 1]], probed)
        dots = (Q.astype(np.float64) @ Dr[inE].astype(np.float64).T).astype(np.float32)
        assert abs(float(s) - float(np.float32(dots.max(axis=1).astype(np.float64).sum()))) <= 1e-6
