"""Helpers of the GPU parity tests: run the CPU oracle and the HIP library on the same seeded
workload and compare stage by stage.

The oracle never sees anything the GPU produced: both sides start from the generated index and
queries, and the comparison is done here on their separate outputs.

Matching rules.  Bit-exact: S_cq (the library accumulates each dot product in double in index
order, as the definition reads, so there is no rounding-order freedom), probed centroids,
candidate sets, the stage-2 and stage-3 selections with their scores (fixed-shape fp64 sums of
fp32 maxima are exact unless a partial sum needs more than 53 bits), bucket indices and
decompressed vectors.  Final MaxSim scores: |gpu - oracle| <= TOL (the library contracts in fp32
on the matrix cores); final ids identical except where oracle scores tie inside TOL at the cut.
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


def compare_query(ix, Q, params, gpu, ctx=""):
    """One query: oracle pipeline with dumps vs the library's debug outputs (numpy, already sliced to this query).
    gpu keys: ids, scores and optionally S_cq, probed, cand, sel2_ids, sel2_scores, sel3_ids, sel3_scores."""
    nprobe, t_cs, ndocs, k = params
    o_ids, o_sc, d = orc.search(ix, Q, nprobe, t_cs, ndocs, k, dumps=True)
    if "S_cq" in gpu:
        assert np.array_equal(bits(gpu["S_cq"]), bits(d["S"])), f"{ctx}: S_cq differs in " \
            f"{int((bits(gpu['S_cq']) != bits(d['S'])).sum())} entries"
    if "probed" in gpu:
        assert np.array_equal(gpu["probed"], d["probed"]), f"{ctx}: probed centroids differ"
    if "cand" in gpu:
        assert np.array_equal(gpu["cand"], d["cand"]), f"{ctx}: candidate set differs " \
            f"(gpu {len(gpu['cand'])}, oracle {len(d['cand'])})"
    for st in ("sel2", "sel3"):
        if st + "_ids" in gpu:
            gi, gs = sort_pairs(gpu[st + "_ids"], gpu[st + "_scores"])
            assert np.array_equal(gi, d[st + "_ids"]), f"{ctx}: {st} ids differ"
            assert np.array_equal(bits(gs), bits(d[st + "_scores"])), f"{ctx}: {st} scores differ"
    s4 = orc.maxsim(ix, Q, d["sel3_ids"])
    same = assert_final_matches(gpu["ids"], gpu["scores"], d["sel3_ids"], s4, k, ctx=ctx)
    if same:
        assert np.array_equal(gpu["ids"], o_ids), f"{ctx}: ids"
    return same


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
    return g
