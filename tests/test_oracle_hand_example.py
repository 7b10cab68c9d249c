"""Oracle vs a hand-computed micro index (tests/golden/hand_example.json).

Derivation (dim 4, |Q| = 2, weights w = (-1/4, 0, 1/4, 1/2), q0 = e0, q1 = e1):

* Eq. 2:  S[c] = (c . q0, c . q1):  c0 -> (1, 0);  c1 -> (0, 1);  c2 -> (1/2, 3/4).
* Section 4.5, MSB-first packing: token bucket indices (1,1,1,1) -> 0b01010101 = 85, (0,2,1,1) -> 37,
  (1,3,1,1) -> 117, (2,0,1,1) -> 133, (1,1,2,0) -> 88.  Reconstruction centroid + w[index]:
  t0 = c0 + (0,0,0,0) = (1,0,0,0);  t1 = c0 + (-1/4,1/4,0,0) = (3/4,1/4,0,0);  t2 = c1 + (0,1/2,0,0) = (0,3/2,0,0);
  t3 = c2 + (1/4,-1/4,0,0) = (3/4,1/2,0,0);  t4 = c2 + (0,0,1/4,-1/4) = (1/2,3/4,1/4,-1/4).
* Passages: p0 = {t0,t1} (codes 0,0);  p1 = {t2,t3} (codes 1,2);  p2 = {t4} (code 2).
  Inverted lists (Section 4.1): c0 -> {0}, c1 -> {1}, c2 -> {1,2}.
* Eq. 1 on the reconstructions: p0: max(1,3/4) + max(0,1/4) = 5/4;  p1: max(0,3/4) + max(3/2,1/2) = 9/4;
  p2: 1/2 + 3/4 = 5/4.  Exhaustive ranking: p1, then p0 and p2 tied at 5/4 in pid order.
* nprobe = 1: q0 probes c0, q1 probes c1 -> candidates {0,1}.  nprobe = 2: the second best of q0 is
  c2 (1/2 > 0), of q1 is c2 (3/4 > 0) -> candidates {0,1,2}.
* Eq. 5 at t_cs = 0.8: row maxima 1, 1, 3/4 -> c2 is pruned; at t_cs = 0.75 it is kept (inclusive >=).
* Stage 2 at 0.8 (Eq. 3-4 over surviving tokens): p0 -> (1,0) -> 1;  p1 -> only the c1 token -> (0,1) -> 1;
  p2 -> nothing survives -> -inf.  Ties order by pid.
* Stage 3 (no pruning): p0 -> 1;  p1 -> columnwise max of (0,1),(1/2,3/4) = (1/2,1) -> 3/2;  p2 -> 5/4.
  Keeps max(1, ndocs/4) passages.
"""
import json
import os

import numpy as np
import pytest

from oracle import oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_example.json")


def _f(v):
    return np.array([-np.inf if x == "-inf" else x for x in v], np.float32)


@pytest.fixture(scope="module")
def hand():
    g = json.load(open(GOLD))
    ivf_off = np.cumsum([0] + [len(l) for l in g["ivf"]]).astype(np.int64)
    ivf_pids = np.array([p for l in g["ivf"] for p in l], np.int32)
    arrays = dict(centroids=np.array(g["centroids"], np.float32), doc_offsets=np.array(g["doc_offsets"], np.int64),
                  codes=np.array(g["codes"], np.int32),
                  residuals=np.array(g["packed_bytes"], np.uint8).reshape(-1, 1),
                  bucket_weights=np.array(g["bucket_weights"], np.float32), ivf_offsets=ivf_off, ivf_pids=ivf_pids)
    return g, orc.Index(arrays, g["nbits"])


def test_scq(hand):
    g, ix = hand
    S = orc.scq(ix.centroids, np.array(g["Q"], np.float32))
    assert S.shape == (3, 2)
    np.testing.assert_array_equal(S, np.array(g["S"], np.float32))


def test_codec(hand):
    g, ix = hand
    D, idx = orc.decompress(ix, 0, 5)
    np.testing.assert_array_equal(idx, np.array(g["bucket_indices"], np.uint8))
    np.testing.assert_array_equal(D, np.array(g["decompressed"], np.float32))
    # encoding the reconstructions against cut-offs halfway between the weights gives the bytes back
    cut = np.array([-0.125, 0.125, 0.375], np.float32)
    packed = orc.encode(D, ix.codes, ix.centroids, cut, 2)
    np.testing.assert_array_equal(packed.reshape(-1), np.array(g["packed_bytes"], np.uint8))


def test_ivf(hand):
    g, ix = hand
    off, pids = orc.build_ivf(ix.codes, ix.doc_offsets, 3)
    np.testing.assert_array_equal(off, ix.ivf_offsets)
    np.testing.assert_array_equal(pids, ix.ivf_pids)


def test_exhaustive(hand):
    g, ix = hand
    ids, sc = orc.exhaustive(ix, np.array(g["Q"], np.float32), 3)
    np.testing.assert_array_equal(ids, g["exhaustive"]["ids"])
    np.testing.assert_array_equal(sc, _f(g["exhaustive"]["scores"]))


@pytest.mark.parametrize("case", range(4))
def test_pipeline(hand, case):
    g, ix = hand
    c = g["cases"][case]
    Q = np.array(g["Q"], np.float32)
    ids, sc, d = orc.search(ix, Q, c["nprobe"], c["t_cs"], c["ndocs"], c["k"], dumps=True)
    np.testing.assert_array_equal(d["probed"], np.array(c["probed"], np.int32))
    np.testing.assert_array_equal(d["cand"], c["cand"])
    np.testing.assert_array_equal(d["sel2_ids"], c["sel2_ids"])
    np.testing.assert_array_equal(d["sel2_scores"], _f(c["sel2_scores"]))
    np.testing.assert_array_equal(d["sel3_ids"], c["sel3_ids"])
    np.testing.assert_array_equal(d["sel3_scores"], _f(c["sel3_scores"]))
    np.testing.assert_array_equal(ids, c["ids"])
    np.testing.assert_array_equal(sc, _f(c["scores"]))
    # the composition from stage functions agrees with the C pipeline
    ids2, sc2, _ = orc.search_from_S(ix, Q, d["S"], c["nprobe"], c["t_cs"], c["ndocs"], c["k"])
    np.testing.assert_array_equal(ids2, ids)
    np.testing.assert_array_equal(sc2, sc)
