"""Helpers of the GPU parity tests: run the CPU oracle and the HIP library on the same seeded
workload and compare stage by stage.

The oracle never sees anything the GPU produced: both sides start from the generated index and
queries, and the comparison is done here on their separate outputs.

Matching rules.  Always bit-exact: probed centroids, candidate sets, the pruning map, bucket
indices and decompressed vectors.  With a double-precision score kernel also S_cq (each dot
product accumulated in double in index order, as the definition reads) and the stage-2 and
stage-3 selections with their scores (sums of 32 fp32 maxima in double, in index order).  With
the split-fp16 score kernel S_cq is within TOL_S, and a selection may differ from the oracle's
only among items whose oracle scores lie within TOL_CI of the cut; each later stage is then
checked on the set the library actually kept (compare_query).  Final MaxSim scores:
|gpu - oracle| <= TOL; final ids identical except where oracle scores tie inside TOL at the cut.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import oracle as orc

TOL = 1e-4   # fp32 scores of unit-norm 128-d vectors (the tolerance the benchmark spec fixes)


def oracle_index(w):
    return orc.Index(w.numpy(), w.cfg.nbits)


def device_arrays(w, device="cuda:0"):
    return {n: getattr(w, n).to(device).contiguous() for n in
            ("centroids", "doc_offsets", "codes", "residuals", "bucket_weights", "ivf_offsets", "ivf_pids")}


def sort_pairs(ids: np.ndarray, scores: np.ndarray):
    """(score desc, id asc) order of a list the library returns in unspecified order."""
    order = np.lexsort((ids, -scores.astype(np.float64)))
    return ids[order], scores[order]


def bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def assert_final_matches(gpu_ids, gpu_scores, cand_ids, cand_scores, k, tol=TOL, ctx=""):
    """gpu_ids/gpu_scores: the k slots returned for one query.  cand_ids/cand_scores: the oracle's exact MaxSim
    score of every passage that entered stage 4.  Returns True when the id lists are identical to the oracle's."""
    n = min(k, len(cand_ids))
    order = np.lexsort((cand_ids, -cand_scores.astype(np.float64)))
    o_ids, o_sc = cand_ids[order], cand_scores[order]
    assert np.all(gpu_ids[n:] == -1), f"{ctx}: unused id slots must be -1"
    assert np.all(np.isneginf(gpu_scores[n:])), f"{ctx}: unused score slots must be -inf"
    g_ids, g_sc = gpu_ids[:n], gpu_scores[:n]
    if n == 0:
        return True
    assert len(set(g_ids.tolist())) == n, f"{ctx}: duplicate ids"
    lut = {int(i): float(s) for i, s in zip(cand_ids, cand_scores)}
    for i, s in zip(g_ids, g_sc):
        assert int(i) in lut, f"{ctx}: id {i} never reached stage 4"
        assert abs(float(s) - lut[int(i)]) <= tol or (np.isneginf(s) and np.isneginf(lut[int(i)])), \
            f"{ctx}: score of {i}: gpu {s} oracle {lut[int(i)]}"
    # order: by the library's own scores, ties by id
    for a in range(n - 1):
        assert g_sc[a] > g_sc[a + 1] or (g_sc[a] == g_sc[a + 1] and g_ids[a] < g_ids[a + 1]), f"{ctx}: order at rank {a}"
    # membership: everything clearly above the cut is in, nothing clearly below it is
    cut = float(o_sc[n - 1])
    got = set(int(i) for i in g_ids)
    for i, s in zip(o_ids, o_sc):
        if float(s) > cut + tol:
            assert int(i) in got, f"{ctx}: passage {i} (oracle {s}, cut {cut}) missing"
    for i in g_ids:
        assert lut[int(i)] >= cut - tol, f"{ctx}: passage {i} (oracle {lut[int(i)]}) below the cut {cut}"
    # rank by rank: a differing id is only allowed inside a near-tie of oracle scores
    same = True
    for a in range(n):
        if int(g_ids[a]) != int(o_ids[a]):
            same = False
            assert abs(lut[int(g_ids[a])] - float(o_sc[a])) <= tol, \
                f"{ctx}: rank {a}: gpu id {g_ids[a]} ({lut[int(g_ids[a])]}) vs oracle id {o_ids[a]} ({o_sc[a]})"
    return same


EPS_S = 2.0 ** -15    # the split-fp16 score kernel's documented bound on |S_cq - exact| (include/plaid.h)
TOL_S = 2e-6          # what its entries are held to here (observed: a few 1e-7)
TOL_CI = 2e-5         # centroid-interaction scores built from such entries: sums of 32 of them
MEASURED = {"S": 0.0, "s3": 0.0, "s4": 0.0}   # largest deviations seen in this process (printed by the tests)


def unpack_keep(words: np.ndarray, C: int) -> np.ndarray:
    """[ceil(C/32)] 32-bit words -> [C] 0/1 (bit c % 32 of word c / 32)."""
    w = np.ascontiguousarray(words).view(np.uint32)
    return ((w[:, None] >> np.arange(32, dtype=np.uint32)[None, :]) & 1).astype(np.uint8).reshape(-1)[:C]


def assert_selection_matches(g_ids, g_scores, pool_ids, pool_scores, m, tol_sel, tol_score, ctx=""):
    """A stage's selection taken on scores that carry an error: g_ids / g_scores = what the library kept (any order),
    pool_ids / pool_scores = the oracle's score of every item the stage chose from.  The kept set must be the oracle's
    except for items whose oracle score lies within tol_sel of the oracle's cut-off score, and every kept item's score
    must be within tol_score of the oracle's.  Returns True when the kept set is exactly the oracle's."""
    n = min(m, len(pool_ids))
    assert len(g_ids) == n, f"{ctx}: kept {len(g_ids)} items, expected {n}"
    if n == 0:
        return True
    assert len(set(g_ids.tolist())) == n, f"{ctx}: duplicate ids"
    lut = {int(i): float(s) for i, s in zip(pool_ids, pool_scores)}
    for i, s in zip(g_ids, g_scores):
        assert int(i) in lut, f"{ctx}: id {i} was not among the stage's inputs"
        o = lut[int(i)]
        assert (np.isneginf(s) and np.isneginf(o)) or abs(float(s) - o) <= tol_score, f"{ctx}: score of {i}: gpu {s} oracle {o}"
    order = np.lexsort((pool_ids, -pool_scores.astype(np.float64)))
    o_ids, o_sc = pool_ids[order], pool_scores[order]
    cut = float(o_sc[n - 1])
    got = set(int(i) for i in g_ids)
    if np.isneginf(cut):
        # the cut falls among the empty bags, which rank by passage id: everything non-empty is in, and the empty ones
        # kept are exactly the smallest ids
        assert got == set(int(i) for i in o_ids[:n]), f"{ctx}: selection differs where the cut lies among empty bags"
        return True
    for i, sc in zip(o_ids, o_sc):
        if float(sc) > cut + tol_sel:
            assert int(i) in got, f"{ctx}: item {i} (oracle {sc}, cut {cut}) missing"
    for i in g_ids:
        assert lut[int(i)] >= cut - tol_sel, f"{ctx}: item {i} (oracle {lut[int(i)]}) below the cut {cut}"
    return got == set(int(i) for i in o_ids[:n])


def compare_query(ix, Q, params, gpu, ctx="", approx=False):
    """One query: oracle pipeline with dumps vs the library's debug outputs (numpy, already sliced to this query).
    gpu keys: ids, scores and optionally S_cq, probed, cand, keep, sel2_ids, sel2_scores, sel3_ids, sel3_scores.

    approx = False (double-precision score kernels): everything up to stage 3 bit for bit.
    approx = True (split-fp16 score kernel): S_cq within TOL_S; probes, candidates and the pruning map identical; the
    stage-2 selection and its scores identical when at most 63 centroids survive (their rows are re-evaluated in
    double), else within tolerance; stage 3 is checked on the set the library's stage 2 kept and stage 4 on the set its
    stage 3 kept, each against the oracle's scores of those same sets: a selection may differ from the oracle's only
    among items within TOL_CI of the cut."""
    nprobe, t_cs, ndocs, k = params
    o_ids, o_sc, d = orc.search(ix, Q, nprobe, t_cs, ndocs, k, dumps=True)
    if "S_cq" in gpu:
        if approx:
            with np.errstate(invalid="ignore"):
                err = float(np.max(np.abs(gpu["S_cq"].astype(np.float64) - d["S"].astype(np.float64))))
            MEASURED["S"] = max(MEASURED["S"], err)
            assert err <= TOL_S, f"{ctx}: S_cq off by {err}"
        else:
            assert np.array_equal(bits(gpu["S_cq"]), bits(d["S"])), f"{ctx}: S_cq differs in " \
                f"{int((bits(gpu['S_cq']) != bits(d['S'])).sum())} entries"
    if "probed" in gpu:
        assert np.array_equal(gpu["probed"], d["probed"]), f"{ctx}: probed centroids differ"
    if "cand" in gpu:
        assert np.array_equal(gpu["cand"], d["cand"]), f"{ctx}: candidate set differs " \
            f"(gpu {len(gpu['cand'])}, oracle {len(d['cand'])})"
    keep = orc.keep_mask(d["S"], t_cs)
    if "keep" in gpu:
        assert np.array_equal(unpack_keep(gpu["keep"], ix.C), keep), f"{ctx}: pruning map differs"
    if not approx:
        for st in ("sel2", "sel3"):
            if st + "_ids" in gpu:
                gi, gs = sort_pairs(gpu[st + "_ids"], gpu[st + "_scores"])
                assert np.array_equal(gi, d[st + "_ids"]), f"{ctx}: {st} ids differ"
                assert np.array_equal(bits(gs), bits(d[st + "_scores"])), f"{ctx}: {st} scores differ"
        sel3 = d["sel3_ids"]
    else:
        sel2, sel3 = d["sel2_ids"], d["sel3_ids"]
        if "sel2_ids" in gpu:
            gi, gs = sort_pairs(gpu["sel2_ids"], gpu["sel2_scores"])
            if int(keep.sum()) <= 63:
                assert np.array_equal(gi, d["sel2_ids"]), f"{ctx}: sel2 ids differ"
                assert np.array_equal(bits(gs), bits(d["sel2_scores"])), f"{ctx}: sel2 scores differ"
            else:
                s2 = orc.centroid_interaction(d["S"], d["cand"], ix, keep)
                assert_selection_matches(gi, gs, d["cand"], s2, ndocs, TOL_CI, TOL_CI, ctx=f"{ctx}: sel2")
            sel2 = np.sort(gi)
        if "sel3_ids" in gpu:
            gi, gs = sort_pairs(gpu["sel3_ids"], gpu["sel3_scores"])
            s3 = orc.centroid_interaction(d["S"], sel2, ix, None)
            assert_selection_matches(gi, gs, sel2, s3, max(1, ndocs // 4), TOL_CI, TOL_CI, ctx=f"{ctx}: sel3")
            lut = dict(zip(sel2.tolist(), s3.tolist()))
            fin = [abs(float(s) - lut[int(i)]) for i, s in zip(gi, gs) if np.isfinite(s)]
            if fin:
                MEASURED["s3"] = max(MEASURED["s3"], max(fin))
            sel3 = np.sort(gi)
    s4 = orc.maxsim(ix, Q, sel3)
    same = assert_final_matches(gpu["ids"], gpu["scores"], sel3, s4, k, ctx=ctx)
    if same and np.array_equal(sel3, np.sort(d["sel3_ids"])):
        assert np.array_equal(gpu["ids"], o_ids), f"{ctx}: ids"
    return same and np.array_equal(gpu["ids"], o_ids)


def run_gpu_debug(pl, gidx, Qdev, params, want=None):
    nprobe, t_cs, ndocs, k = params
    ids, sc, bufs = pl.plaid_search_debug(gidx, Qdev, nprobe, t_cs, ndocs, k, want=want)
    torch.cuda.synchronize()
    out = dict(ids=ids.cpu().numpy(), scores=sc.cpu().numpy())
    for n, t in bufs.items():
        out[n] = t.cpu().numpy()
    return out


def slice_query(out, q):
    g = dict(ids=out["ids"][q], scores=out["scores"][q])
    if "S_cq" in out:
        g["S_cq"] = out["S_cq"][q]
    if "probed" in out:
        g["probed"] = out["probed"][q]
    if "cand" in out:
        g["cand"] = out["cand"][q][: int(out["n_cand"][q])]
    if "sel2_ids" in out:
        n2 = int(out["n2"][q])
        g["sel2_ids"], g["sel2_scores"] = out["sel2_ids"][q][:n2], out["sel2_scores"][q][:n2]
    if "sel3_ids" in out:
        n3 = int(out["n3"][q])
        g["sel3_ids"], g["sel3_scores"] = out["sel3_ids"][q][:n3], out["sel3_scores"][q][:n3]
    if "keep" in out:
        g["keep"] = out["keep"][q]
    return g


def is_approx(pl, gidx, params) -> bool:
    """Whether a search with these parameters runs the split-fp16 score kernel (it serves nprobe <= 8)."""
    return pl.plaid_get_score_kernel(gidx) == 2 and params[0] <= 8
