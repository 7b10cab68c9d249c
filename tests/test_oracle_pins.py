"""Pins of the CPU oracle against things other than itself: library routines, brute force on small
inputs, closed forms, invariants and values the paper prints (tests/golden/)."""
import itertools
import os

import numpy as np
import pytest

from oracle import oracle as orc
from synth import index_nbytes, make_workload, tiny_config

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _ix(w):
    return orc.Index(w.numpy(), w.cfg.nbits)


@pytest.fixture(scope="module")
def tiny2():
    return make_workload(tiny_config(C=96, P=60, lo=1, hi=12, nbits=2, nq=6, seed=3), noise="calibrated",
                         keep_embeddings=10_000)


@pytest.fixture(scope="module")
def tiny1():
    return make_workload(tiny_config(C=64, P=40, lo=1, hi=9, nbits=1, nq=5, seed=5), noise="literal",
                         keep_embeddings=10_000)


# ----------------------------------------------------------------------------- Eq. 2
def test_scq_equals_fp64_matmul():
    rng = np.random.default_rng(0)
    C = rng.standard_normal((517, 128)).astype(np.float32)
    Q = rng.standard_normal((32, 128)).astype(np.float32)
    S = orc.scq(C, Q)
    ref = (C.astype(np.float64) @ Q.astype(np.float64).T)
    assert S.shape == (517, 32)
    # rounding a double-accumulated dot product once: at most one fp32 ulp from the fp64 BLAS result
    assert np.max(np.abs(S - ref) / np.maximum(np.abs(ref), 1e-3)) < 1.5e-7
    # orientation: rows are centroids, columns query tokens (a transposed operand fails here)
    assert abs(S[5, 7] - float(C[5].astype(np.float64) @ Q[7].astype(np.float64))) < 1e-6


# ----------------------------------------------------------------------------- every top-n
def test_select_equals_full_sort():
    rng = np.random.default_rng(1)
    for n, m in [(0, 3), (1, 1), (50, 7), (50, 50), (50, 80), (1000, 256)]:
        scores = np.round(rng.standard_normal(n), 1).astype(np.float32)   # many exact ties
        if n > 10:
            scores[rng.integers(0, n, n // 5)] = -np.inf
        ids = rng.permutation(n * 3)[:n].astype(np.int32)
        oi, os_ = orc.select(ids, scores, m)
        order = sorted(range(n), key=lambda j: (-scores[j], ids[j]))[:m]
        np.testing.assert_array_equal(oi, ids[order])
        np.testing.assert_array_equal(os_, scores[order])


def test_top_nprobe_equals_lexsort():
    rng = np.random.default_rng(2)
    S = np.round(rng.standard_normal((97, 32)), 1).astype(np.float32)
    for nprobe in (1, 2, 5, 97):
        got = orc.top_nprobe(S, nprobe)
        for i in range(32):
            order = np.lexsort((np.arange(97), -S[:, i]))[:nprobe]
            np.testing.assert_array_equal(got[i], order)


# ----------------------------------------------------------------------------- inverted lists, candidates
def _brute_ivf(codes, doc_offsets, C):
    lists = [set() for _ in range(C)]
    for p in range(len(doc_offsets) - 1):
        for j in range(doc_offsets[p], doc_offsets[p + 1]):
            lists[codes[j]].add(p)
    return [sorted(s) for s in lists]


@pytest.mark.parametrize("fx", ["tiny1", "tiny2"])
def test_ivf_brute_force(fx, request):
    w = request.getfixturevalue(fx)
    a = w.numpy()
    off, pids = orc.build_ivf(a["codes"], a["doc_offsets"], w.cfg.C)
    lists = _brute_ivf(a["codes"], a["doc_offsets"], w.cfg.C)
    assert off[-1] == sum(len(l) for l in lists) == len({(c, p) for p in range(w.cfg.P)
                                                         for c in a["codes"][a["doc_offsets"][p]:a["doc_offsets"][p + 1]]})
    for c in range(w.cfg.C):
        assert list(pids[off[c]:off[c + 1]]) == lists[c]
    # the generator's lists are the same lists
    np.testing.assert_array_equal(off, a["ivf_offsets"])
    np.testing.assert_array_equal(pids, a["ivf_pids"])
    assert any(len(l) == 0 for l in lists), "the case should include empty lists"


def test_generator_ivf_matches_on_cfg1(cfg1_literal):
    a = cfg1_literal.numpy()
    off, pids = orc.build_ivf(a["codes"], a["doc_offsets"], cfg1_literal.cfg.C)
    np.testing.assert_array_equal(off, a["ivf_offsets"])
    np.testing.assert_array_equal(pids, a["ivf_pids"])


@pytest.mark.parametrize("fx", ["tiny1", "tiny2"])
def test_candidates_brute_force(fx, request):
    w = request.getfixturevalue(fx)
    a = w.numpy()
    ix = _ix(w)
    rng = np.random.default_rng(3)
    for nprobed in (1, 3, 10):
        T = rng.integers(0, w.cfg.C, nprobed).astype(np.int32)
        cand = orc.candidates(T, ix)
        want = [p for p in range(w.cfg.P)
                if set(a["codes"][a["doc_offsets"][p]:a["doc_offsets"][p + 1]]) & set(T.tolist())]
        assert list(cand) == want


# ----------------------------------------------------------------------------- Eq. 3-5
def _brute_ci(S, a, pids, keep=None):
    out = []
    for p in pids:
        codes = a["codes"][a["doc_offsets"][p]:a["doc_offsets"][p + 1]]
        if keep is not None:
            codes = codes[keep[codes] != 0]
        if len(codes) == 0:
            out.append(-np.inf)
            continue
        Dt = S[codes]                      # Eq. 3: one row of S_cq per token
        out.append(np.float32(Dt.max(axis=0).astype(np.float64).sum()))   # Eq. 4
    return np.array(out, np.float32)


@pytest.mark.parametrize("fx", ["tiny1", "tiny2"])
def test_centroid_interaction_brute_force(fx, request):
    w = request.getfixturevalue(fx)
    a = w.numpy()
    ix = _ix(w)
    pids = np.arange(w.cfg.P, dtype=np.int32)
    for q in range(w.cfg.nq):
        S = orc.scq(a["centroids"], a["queries"][q])
        np.testing.assert_array_equal(orc.centroid_interaction(S, pids, ix), _brute_ci(S, a, pids))
        for t in (-np.inf, float(np.quantile(S.max(1), 0.5)), float(np.quantile(S.max(1), 0.9)), np.inf):
            keep = orc.keep_mask(S, t)
            np.testing.assert_array_equal(keep, (S.max(axis=1) >= np.float32(t)).astype(np.uint8))
            np.testing.assert_array_equal(orc.centroid_interaction(S, pids, ix, keep), _brute_ci(S, a, pids, keep))


def test_keep_threshold_is_inclusive():
    S = np.array([[0.5, 0.1], [0.2, 0.49999997], [0.7, -1.0]], np.float32)
    np.testing.assert_array_equal(orc.keep_mask(S, 0.5), [1, 0, 1])


@pytest.mark.parametrize("fx", ["tiny1", "tiny2", "cfg1_calibrated"])
def test_centroid_interaction_is_maxsim_over_centroid_only_reconstructions(fx, request):
    """Unpruned centroid interaction == Eq. 1 on an index whose bucket weights are all zero (D_j = centroid)."""
    w = request.getfixturevalue(fx)
    a = w.numpy()
    ix = _ix(w)
    ix0 = ix.with_weights(np.zeros(1 << w.cfg.nbits, np.float32))
    pids = np.arange(min(w.cfg.P, 300), dtype=np.int32)
    for q in range(min(w.cfg.nq, 3)):
        S = orc.scq(a["centroids"], a["queries"][q])
        np.testing.assert_array_equal(orc.centroid_interaction(S, pids, ix), orc.maxsim(ix0, a["queries"][q], pids))


@pytest.mark.parametrize("fx", ["tiny2", "cfg1_calibrated"])
def test_stage2_invariants(fx, request):
    w = request.getfixturevalue(fx)
    a = w.numpy()
    ix = _ix(w)
    cfg = w.cfg
    for q in range(min(cfg.nq, 3)):
        S = orc.scq(a["centroids"], a["queries"][q])
        cand = orc.candidates(orc.top_nprobe(S, 2), ix)
        s3 = orc.centroid_interaction(S, cand, ix)
        prev = None
        for t in (-np.inf, 0.2, 0.5, 0.9, np.inf):
            s2 = orc.centroid_interaction(S, cand, ix, orc.keep_mask(S, t))
            assert np.all(s2 <= s3)                       # max over a subset of the rows
            if t == -np.inf:
                np.testing.assert_array_equal(s2, s3)
            if prev is not None:
                assert np.all(s2 <= prev)                 # non-increasing in t_cs
            prev = s2
        assert np.all(np.isneginf(prev))                  # t_cs = +inf prunes everything
        ids, sc = orc.select(cand, prev, 7)
        np.testing.assert_array_equal(ids, cand[:7])      # ... and selection falls back to pid order


# ----------------------------------------------------------------------------- Section 4.5 codec
@pytest.mark.parametrize("nbits", [1, 2, 4])
def test_byte_table_equals_unpackbits(nbits):
    t = orc.byte_table(nbits)
    bits = np.unpackbits(np.arange(256, dtype=np.uint8)[:, None], axis=1)          # MSB first
    want = bits.reshape(256, 8 // nbits, nbits) @ (1 << np.arange(nbits - 1, -1, -1))
    np.testing.assert_array_equal(t, want.astype(np.uint8))


@pytest.mark.parametrize("fx", ["tiny1", "tiny2", "cfg1_literal", "cfg1_calibrated"])
def test_codec_invariants(fx, request):
    w = request.getfixturevalue(fx)
    a = w.numpy()
    ix = _ix(w)
    nb = w.cfg.nbits
    n = min(w.N, 4096)
    x = w.sample_embeddings[:n].numpy()
    cut, wts = a["bucket_cutoffs"], a["bucket_weights"]
    assert a["residuals"].shape == (w.N, 16 * nb)                      # Section 3.1: 16 or 32 bytes per token
    assert a["codes"].nbytes + a["residuals"].nbytes == index_nbytes(w.N, nb)
    assert np.all(np.diff(cut) > 0) and np.all(np.diff(wts) > 0)
    assert np.all(wts[:-1] < cut) and np.all(cut < wts[1:])             # weight b lies inside bucket b
    # the generator's packed bytes are what the oracle's encoder produces from the uncompressed vectors
    packed = orc.encode(x, a["codes"][:n], a["centroids"], cut, nb)
    np.testing.assert_array_equal(packed, a["residuals"][:n])
    D, idx = orc.decompress(ix, 0, n)
    # independent unpack with numpy
    bits = np.unpackbits(a["residuals"][:n], axis=1).reshape(n, 128, nb)
    want_idx = (bits @ (1 << np.arange(nb - 1, -1, -1))).astype(np.uint8)
    np.testing.assert_array_equal(idx, want_idx)
    np.testing.assert_array_equal(D, a["centroids"][a["codes"][:n]] + wts[want_idx])
    # decode . encode . decode = decode
    np.testing.assert_array_equal(orc.encode(D, a["codes"][:n], a["centroids"], cut, nb), packed)
    # reconstruction error within bucket resolution
    r = x - a["centroids"][a["codes"][:n]]
    lo = np.concatenate([[r.min()], cut])[want_idx]
    hi = np.concatenate([cut, [r.max()]])[want_idx]
    assert np.all(lo <= r + 1e-7) and np.all(r <= hi + 1e-7)
    bound = np.maximum(hi - wts[want_idx], wts[want_idx] - lo)
    assert np.all(np.abs(D - x) <= bound + 1e-6)
    if n >= 4096:
        hist = np.bincount(want_idx.reshape(-1), minlength=1 << nb) / want_idx.size
        assert np.all(np.abs(hist - 1.0 / (1 << nb)) < 0.02)            # buckets are quantiles of the residuals


def test_bucket_of_each_weight_is_itself():
    cut = np.array([-0.1, 0.0, 0.1], np.float32)
    wts = np.array([-0.2, -0.05, 0.05, 0.2], np.float32)
    x = np.tile(wts, 32)[None, :]                                       # residual = weight (centroid is zero)
    packed = orc.encode(x, np.zeros(1, np.int32), np.zeros((1, 128), np.float32), cut, 2)
    assert np.all(packed == 0b00011011)
    # a value equal to a cut-off goes to the lower bucket
    x = np.tile(np.array([-0.1, 0.0, 0.1, 0.3], np.float32), 32)[None, :]
    packed = orc.encode(x, np.zeros(1, np.int32), np.zeros((1, 128), np.float32), cut, 2)
    assert np.all(packed == 0b00011011)


# ----------------------------------------------------------------------------- Eq. 1
@pytest.mark.parametrize("fx", ["tiny1", "tiny2"])
def test_maxsim_equals_numpy_brute_force(fx, request):
    w = request.getfixturevalue(fx)
    a = w.numpy()
    ix = _ix(w)
    nb = w.cfg.nbits
    bits = np.unpackbits(a["residuals"], axis=1).reshape(w.N, 128, nb)
    idx = bits @ (1 << np.arange(nb - 1, -1, -1))
    D = (a["centroids"][a["codes"]] + a["bucket_weights"][idx]).astype(np.float32)
    pids = np.arange(w.cfg.P, dtype=np.int32)
    for q in range(w.cfg.nq):
        Q = a["queries"][q]
        want = []
        for p in pids:
            Dp = D[a["doc_offsets"][p]:a["doc_offsets"][p + 1]].astype(np.float64)
            sim = (Q.astype(np.float64) @ Dp.T).astype(np.float32)      # [|Q|, |D|]
            want.append(np.float32(sim.max(axis=1).astype(np.float64).sum()))
        got = orc.maxsim(ix, Q, pids)
        np.testing.assert_allclose(got, np.array(want, np.float32), rtol=0, atol=2e-6)
        ids, sc = orc.exhaustive(ix, Q, 5)
        order = np.lexsort((pids, -got))[:5]
        np.testing.assert_array_equal(ids, pids[order])
        np.testing.assert_array_equal(sc, got[order])


# ----------------------------------------------------------------------------- whole pipeline
@pytest.mark.parametrize("fx", ["tiny1", "tiny2"])
def test_pipeline_equals_exhaustive_when_nothing_is_filtered(fx, request):
    """nprobe = C, t_cs = -inf and ndocs >= 4P (so that ndocs/4 >= P) disable every filter."""
    w = request.getfixturevalue(fx)
    a = w.numpy()
    ix = _ix(w)
    cfg = w.cfg
    lens = np.diff(a["doc_offsets"])
    assert lens.min() == 1
    for q in range(cfg.nq):
        for k in (1, 7, cfg.P, cfg.P + 3):
            ids, sc = orc.search(ix, a["queries"][q], cfg.C, -np.inf, 4 * cfg.P, k)
            eids, esc = orc.exhaustive(ix, a["queries"][q], k)
            np.testing.assert_array_equal(ids, eids)
            np.testing.assert_array_equal(sc, esc)
            if k > cfg.P:
                assert np.all(ids[cfg.P:] == -1) and np.all(np.isneginf(sc[cfg.P:]))


def test_pipeline_equals_exhaustive_on_cfg1(cfg1_calibrated):
    w = cfg1_calibrated
    a = w.numpy()
    ix = _ix(w)
    ids, sc = orc.search(ix, a["queries"][1], w.cfg.C, -np.inf, 4 * w.cfg.P, 10)
    eids, esc = orc.exhaustive(ix, a["queries"][1], 10)
    np.testing.assert_array_equal(ids, eids)
    np.testing.assert_array_equal(sc, esc)


@pytest.mark.parametrize("fx", ["tiny1", "tiny2"])
def test_pipeline_is_the_composition_of_its_stages(fx, request):
    w = request.getfixturevalue(fx)
    a = w.numpy()
    ix = _ix(w)
    cfg = w.cfg
    Svals = orc.scq(a["centroids"], a["queries"][0]).max(1)
    grid = itertools.product((1, 2, cfg.C), (-np.inf, float(np.median(Svals)), np.inf), (1, 4, 16, 4 * cfg.P),
                             (1, 4, cfg.P + 1))
    for nprobe, t, ndocs, k in grid:
        for q in range(2):
            ids, sc, d = orc.search(ix, a["queries"][q], nprobe, t, ndocs, k, dumps=True)
            ids2, sc2, d2 = orc.search_from_S(ix, a["queries"][q], d["S"], nprobe, t, ndocs, k)
            np.testing.assert_array_equal(ids, ids2)
            np.testing.assert_array_equal(sc, sc2)
            for key in ("probed", "cand", "sel2_ids", "sel2_scores", "sel3_ids", "sel3_scores"):
                np.testing.assert_array_equal(d[key], d2[key])
            assert len(d["sel2_ids"]) == min(ndocs, len(d["cand"]))
            assert len(d["sel3_ids"]) == min(max(1, ndocs // 4), len(d["sel2_ids"]))
            assert set(d["sel3_ids"]) <= set(d["sel2_ids"]) <= set(d["cand"])
            n_out = min(k, len(d["sel3_ids"]))
            assert np.all(ids[:n_out] >= 0) and np.all(ids[n_out:] == -1) and np.all(np.isneginf(sc[n_out:]))


def test_batch_equals_single(cfg1_calibrated):
    w = cfg1_calibrated
    a = w.numpy()
    ix = _ix(w)
    c = w.cfg
    ids, sc, used = orc.search_batch(ix, a["queries"][:4], c.nprobe, c.t_cs, c.ndocs, c.k, nthreads=2)
    assert used == 2
    for q in range(4):
        i1, s1 = orc.search(ix, a["queries"][q], c.nprobe, c.t_cs, c.ndocs, c.k)
        np.testing.assert_array_equal(ids[q], i1)
        np.testing.assert_array_equal(sc[q], s1)


def test_recall_of_pipeline_on_calibrated_cfg1(cfg1_calibrated):
    """With the paper's k=10 operating point the pipeline recovers the exhaustive top-10 on the calibrated workload
    (Section 3.3's premise: centroids alone identify strong candidates).  A sanity check, not a quality claim."""
    w = cfg1_calibrated
    a = w.numpy()
    ix = _ix(w)
    c = w.cfg
    hits = 0
    for q in range(3):
        ids, _ = orc.search(ix, a["queries"][q], c.nprobe, c.t_cs, c.ndocs, c.k)
        eids, _ = orc.exhaustive(ix, a["queries"][q], c.k)
        hits += len(set(ids.tolist()) & set(eids.tolist()))
    assert hits >= 27


# ----------------------------------------------------------------------------- values the paper prints
def test_storage_closed_form_against_table1():
    """Section 3.1: 4 bytes of centroid id + 16*b bytes of residual per token; Section 4.1: the inverted list
    holds at most one int32 per token.  Table 1's PLAID index sizes must fall between the two closed forms."""
    rows = [l.split() for l in open(os.path.join(GOLD, "table1_index_sizes.txt")) if l.strip() and l[0] != "#"]
    ivf_gb = None
    for r in rows:
        if r[0] == "msmarco_v2_ivf_GB":
            ivf_gb = float(r[1])
    for r in rows:
        if len(r) != 4:
            continue
        name, tokens, nbits, gib = r[0], float(r[1]), int(r[2]), float(r[3])
        lo = index_nbytes(int(tokens), nbits) / 2 ** 30
        hi = (index_nbytes(int(tokens), nbits) + 4 * tokens) / 2 ** 30
        slack = 0.02 * gib                                              # token counts are printed to 2-4 digits
        assert lo - slack <= gib <= hi + slack, (name, lo, gib, hi)
        if name == "msmarco_v2":
            assert abs(lo + ivf_gb * 1e9 / 2 ** 30 - gib) < 0.02 * gib


def test_table2_triples_are_the_configs():
    from synth import CONFIGS
    rows = [l.split() for l in open(os.path.join(GOLD, "table2_hyperparameters.txt")) if l.strip() and l[0] != "#"]
    table = {int(k): (int(n), float(t), int(d)) for k, n, t, d in rows}
    for name, k in (("cfg1", 10), ("cfg2", 10), ("cfg3", 100), ("cfg4", 1000)):
        c = CONFIGS[name]
        assert (c.nprobe, c.t_cs, c.ndocs) == table[k] and c.k == k
    c = CONFIGS["cfg5"]                                                  # 1-bit share of the largest corpus: k=1000 triple, k=100
    assert (c.nprobe, c.t_cs, c.ndocs) == table[1000]
