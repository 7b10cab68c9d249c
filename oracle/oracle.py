"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE, not the product).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this.  It compiles
``plaid_oracle.c`` with gcc into ``liboracle.so`` beside the source and exposes each function of
the C file on numpy arrays.  Nothing here touches the HIP library.
"""
from __future__ import annotations

import ctypes as ct
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "plaid_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc -O2, OpenMP across queries only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Index(ct.Structure):
    _fields_ = [("dim", ct.c_int32), ("nbits", ct.c_int32), ("C", ct.c_int64), ("P", ct.c_int64), ("N", ct.c_int64),
                ("centroids", ct.c_void_p), ("doc_offsets", ct.c_void_p), ("codes", ct.c_void_p),
                ("residuals", ct.c_void_p), ("bucket_weights", ct.c_void_p), ("ivf_offsets", ct.c_void_p),
                ("ivf_pids", ct.c_void_p), ("renormalize", ct.c_int32)]


class _Dumps(ct.Structure):
    _fields_ = [(n, ct.c_void_p) for n in ("S", "probed", "cand", "n_cand", "sel2_ids", "sel2_scores", "n2",
                                            "sel3_ids", "sel3_scores", "n3")]


def _load():
    global _lib
    if _lib is None:
        # PLAID_ORACLE_LIB names another build of plaid_oracle.c: the planted-mistake test loads deliberately broken
        # copies through it to show that the pins notice
        other = os.environ.get("PLAID_ORACLE_LIB")
        if other:
            _lib = ct.CDLL(other)
        else:
            build()
            _lib = ct.CDLL(_LIB)
        _lib.orc_select.restype = ct.c_int64
        _lib.orc_candidates.restype = ct.c_int64
        _lib.orc_build_ivf.restype = ct.c_int64
        _lib.orc_search.restype = ct.c_int32
        _lib.orc_vanilla_search.restype = ct.c_int32
        _lib.orc_build_ivf_embeddings.restype = ct.c_int64
        _lib.orc_search_batch.restype = ct.c_int32
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else ct.c_void_p(a.ctypes.data)


def _chk(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


class Index:
    """Borrowed view of host index buffers (keeps the numpy arrays alive)."""

    def __init__(self, arrays: Dict[str, np.ndarray], nbits: int, renormalize: bool = False):
        """renormalize: the storage variant in which reconstructed vectors are scaled back to unit length
        (orc_decompress); off by default."""
        self.renormalize = bool(renormalize)
        self.centroids = _chk(arrays["centroids"], np.float32)
        self.doc_offsets = _chk(arrays["doc_offsets"], np.int64)
        self.codes = _chk(arrays["codes"], np.int32)
        self.residuals = _chk(arrays["residuals"], np.uint8)
        self.bucket_weights = _chk(arrays["bucket_weights"], np.float32)
        self.ivf_offsets = _chk(arrays["ivf_offsets"], np.int64)
        self.ivf_pids = _chk(arrays["ivf_pids"], np.int32)
        self.C, self.dim = self.centroids.shape
        self.P = self.doc_offsets.shape[0] - 1
        self.N = self.codes.shape[0]
        self.nbits = nbits
        assert self.bucket_weights.shape[0] == (1 << nbits)
        assert self.residuals.size == self.N * self.dim * nbits // 8
        self.c = _Index(self.dim, nbits, self.C, self.P, self.N, self.centroids.ctypes.data,
                        self.doc_offsets.ctypes.data, self.codes.ctypes.data, self.residuals.ctypes.data,
                        self.bucket_weights.ctypes.data, self.ivf_offsets.ctypes.data, self.ivf_pids.ctypes.data,
                        1 if self.renormalize else 0)

    def _arrays(self) -> Dict[str, np.ndarray]:
        return dict(centroids=self.centroids, doc_offsets=self.doc_offsets, codes=self.codes, residuals=self.residuals,
                    bucket_weights=self.bucket_weights, ivf_offsets=self.ivf_offsets, ivf_pids=self.ivf_pids)

    def with_weights(self, weights: np.ndarray) -> "Index":
        d = self._arrays()
        d["bucket_weights"] = np.asarray(weights, np.float32)
        return Index(d, self.nbits, self.renormalize)

    def renormalized(self, on: bool = True) -> "Index":
        """The same arrays under the other reading of the reconstruction's length."""
        return Index(self._arrays(), self.nbits, on)


# ---- stage functions -----------------------------------------------------------------------

def scq(centroids: np.ndarray, Q: np.ndarray) -> np.ndarray:
    """Eq. 2: S[c][i] = centroid c . query token i, [C, qlen] fp32."""
    centroids = _chk(centroids, np.float32)
    Q = _chk(Q, np.float32)
    C, dim = centroids.shape
    qlen = Q.shape[0]
    S = np.empty((C, qlen), np.float32)
    _load().orc_scq(_p(centroids), ct.c_int64(C), _p(Q), ct.c_int32(qlen), ct.c_int32(dim), _p(S))
    return S


def select(ids: np.ndarray, scores: np.ndarray, m: int):
    """First min(m, n) items by (score desc, id asc)."""
    ids = _chk(ids, np.int32)
    scores = _chk(scores, np.float32)
    n = ids.shape[0]
    cap = max(0, min(m, n))
    oi = np.empty(cap, np.int32)
    os_ = np.empty(cap, np.float32)
    r = _load().orc_select(_p(ids), _p(scores), ct.c_int64(n), ct.c_int64(m), _p(oi), _p(os_))
    assert r == cap
    return oi, os_


def top_nprobe(S: np.ndarray, nprobe: int) -> np.ndarray:
    S = _chk(S, np.float32)
    C, qlen = S.shape
    out = np.empty((qlen, nprobe), np.int32)
    _load().orc_top_nprobe(_p(S), ct.c_int64(C), ct.c_int32(qlen), ct.c_int32(nprobe), _p(out))
    return out


def candidates(probed: np.ndarray, ix: Index) -> np.ndarray:
    probed = _chk(probed, np.int32).reshape(-1)
    cand = np.empty(max(ix.P, 1), np.int32)
    n = _load().orc_candidates(_p(probed), ct.c_int64(probed.shape[0]), _p(ix.ivf_offsets), _p(ix.ivf_pids),
                               ct.c_int64(ix.P), _p(cand))
    return cand[:n].copy()


def keep_mask(S: np.ndarray, t_cs: float) -> np.ndarray:
    S = _chk(S, np.float32)
    C, qlen = S.shape
    keep = np.empty(C, np.uint8)
    _load().orc_keep(_p(S), ct.c_int64(C), ct.c_int32(qlen), ct.c_float(t_cs), _p(keep))
    return keep


def centroid_interaction(S: np.ndarray, pids: np.ndarray, ix: Index, keep: Optional[np.ndarray] = None) -> np.ndarray:
    S = _chk(S, np.float32)
    pids = _chk(pids, np.int32)
    if keep is not None:
        keep = _chk(keep, np.uint8)
    out = np.empty(pids.shape[0], np.float32)
    _load().orc_centroid_interaction(_p(S), ct.c_int32(S.shape[1]), _p(pids), ct.c_int64(pids.shape[0]),
                                     _p(ix.doc_offsets), _p(ix.codes), _p(keep), _p(out))
    return out


def byte_table(nbits: int) -> np.ndarray:
    t = np.empty((256, 8 // nbits), np.uint8)
    _load().orc_build_byte_table(ct.c_int32(nbits), _p(t))
    return t


def decompress(ix: Index, t0: int, t1: int):
    """Reconstructed fp32 vectors and unpacked bucket indices of tokens [t0, t1)."""
    D = np.empty((t1 - t0, ix.dim), np.float32)
    idx = np.empty((t1 - t0, ix.dim), np.uint8)
    _load().orc_decompress(ct.byref(ix.c), ct.c_int64(t0), ct.c_int64(t1), _p(D), _p(idx))
    return D, idx


def encode(x: np.ndarray, codes: np.ndarray, centroids: np.ndarray, cutoffs: np.ndarray, nbits: int) -> np.ndarray:
    x = _chk(x, np.float32)
    codes = _chk(codes, np.int32)
    centroids = _chk(centroids, np.float32)
    cutoffs = _chk(cutoffs, np.float32)
    n, dim = x.shape
    out = np.empty((n, dim * nbits // 8), np.uint8)
    _load().orc_encode(_p(x), _p(codes), ct.c_int64(n), _p(centroids), ct.c_int32(dim), ct.c_int32(nbits), _p(cutoffs),
                       _p(out))
    return out


def build_ivf(codes: np.ndarray, doc_offsets: np.ndarray, C: int):
    codes = _chk(codes, np.int32)
    doc_offsets = _chk(doc_offsets, np.int64)
    P = doc_offsets.shape[0] - 1
    off = np.empty(C + 1, np.int64)
    total = _load().orc_build_ivf(_p(codes), _p(doc_offsets), ct.c_int64(P), ct.c_int64(C), _p(off), None)
    pids = np.empty(total, np.int32)
    _load().orc_build_ivf(_p(codes), _p(doc_offsets), ct.c_int64(P), ct.c_int64(C), _p(off), _p(pids))
    return off, pids


def maxsim(ix: Index, Q: np.ndarray, pids: np.ndarray) -> np.ndarray:
    Q = _chk(Q, np.float32)
    pids = _chk(pids, np.int32)
    out = np.empty(pids.shape[0], np.float32)
    _load().orc_maxsim(ct.byref(ix.c), _p(Q), ct.c_int32(Q.shape[0]), _p(pids), ct.c_int64(pids.shape[0]), _p(out))
    return out


def exhaustive(ix: Index, Q: np.ndarray, k: int):
    Q = _chk(Q, np.float32)
    ids = np.empty(k, np.int32)
    sc = np.empty(k, np.float32)
    _load().orc_exhaustive(ct.byref(ix.c), _p(Q), ct.c_int32(Q.shape[0]), ct.c_int32(k), _p(ids), _p(sc))
    return ids, sc


# ---- whole pipeline ------------------------------------------------------------------------

def search(ix: Index, Q: np.ndarray, nprobe: int, t_cs: float, ndocs: int, k: int, dumps: bool = False):
    """One query through the four stages.  Returns (ids[k], scores[k]) or, with dumps, also a dict of intermediates."""
    Q = _chk(Q, np.float32)
    qlen = Q.shape[0]
    ids = np.empty(k, np.int32)
    sc = np.empty(k, np.float32)
    d = None
    keepalive = {}
    if dumps:
        m3 = max(1, ndocs // 4)
        keepalive = dict(S=np.empty((ix.C, qlen), np.float32), probed=np.empty((qlen, nprobe), np.int32),
                         cand=np.empty(max(ix.P, 1), np.int32), n_cand=np.zeros(1, np.int64),
                         sel2_ids=np.empty(ndocs, np.int32), sel2_scores=np.empty(ndocs, np.float32),
                         n2=np.zeros(1, np.int64), sel3_ids=np.empty(m3, np.int32),
                         sel3_scores=np.empty(m3, np.float32), n3=np.zeros(1, np.int64))
        d = _Dumps(*[keepalive[n].ctypes.data for n, _ in _Dumps._fields_])
    rc = _load().orc_search(ct.byref(ix.c), _p(Q), ct.c_int32(qlen), ct.c_int32(nprobe), ct.c_float(t_cs),
                            ct.c_int32(ndocs), ct.c_int32(k), _p(ids), _p(sc), ct.byref(d) if d is not None else None)
    if rc != 0:
        raise ValueError("orc_search: invalid arguments")
    if not dumps:
        return ids, sc
    nc, n2, n3 = int(keepalive["n_cand"][0]), int(keepalive["n2"][0]), int(keepalive["n3"][0])
    out = dict(S=keepalive["S"], probed=keepalive["probed"], cand=keepalive["cand"][:nc].copy(),
               sel2_ids=keepalive["sel2_ids"][:n2].copy(), sel2_scores=keepalive["sel2_scores"][:n2].copy(),
               sel3_ids=keepalive["sel3_ids"][:n3].copy(), sel3_scores=keepalive["sel3_scores"][:n3].copy())
    return ids, sc, out


def search_batch(ix: Index, Q: np.ndarray, nprobe: int, t_cs: float, ndocs: int, k: int, nthreads: int = 0):
    """nq independent queries, parallel across queries only.  Returns (ids[nq,k], scores[nq,k], threads used)."""
    Q = _chk(Q, np.float32)
    nq, qlen, _ = Q.shape
    ids = np.empty((nq, k), np.int32)
    sc = np.empty((nq, k), np.float32)
    used = _load().orc_search_batch(ct.byref(ix.c), _p(Q), ct.c_int32(nq), ct.c_int32(qlen), ct.c_int32(nprobe),
                                    ct.c_float(t_cs), ct.c_int32(ndocs), ct.c_int32(k), _p(ids), _p(sc),
                                    ct.c_int32(nthreads))
    return ids, sc, used


# ---- vanilla ColBERTv2 retrieval (the paper's baseline) ---------------------------------------

class _VanillaDumps(ct.Structure):
    _fields_ = [(n, ct.c_void_p) for n in ("cand", "n_cand", "n_embeddings", "kept", "kept_scores", "n_kept", "pruned")]


def build_ivf_embeddings(codes: np.ndarray, C: int):
    """Embedding-level inverted lists: (offsets [C+1] int64, eids [N] int64), list c = ascending token indices coded c."""
    codes = _chk(codes, np.int32)
    off = np.empty(C + 1, np.int64)
    eids = np.empty(codes.shape[0], np.int64)
    _load().orc_build_ivf_embeddings(_p(codes), ct.c_int64(codes.shape[0]), ct.c_int64(C), _p(off), _p(eids))
    return off, eids


def vanilla_prune_scores(ix: Index, Q: np.ndarray, probed: np.ndarray, pids: np.ndarray) -> np.ndarray:
    """Pruning score of each listed passage from the embeddings of the probed centroids' lists alone."""
    Q = _chk(Q, np.float32)
    pids = _chk(pids, np.int32)
    in_e = np.ascontiguousarray(np.isin(ix.codes, np.unique(np.asarray(probed).reshape(-1))).astype(np.uint8))
    out = np.empty(pids.shape[0], np.float32)
    _load().orc_vanilla_prune_scores(ct.byref(ix.c), _p(Q), ct.c_int32(Q.shape[0]), _p(in_e), _p(pids), ct.c_int64(pids.shape[0]),
                                     _p(out))
    return out


def vanilla_search(ix: Index, eoff: np.ndarray, eids: np.ndarray, Q: np.ndarray, nprobe: int, ncandidates: int, k: int,
                   dumps: bool = False):
    """One query through vanilla retrieval.  Returns (ids[k], scores[k]) or, with dumps, also a dict with the candidate
    passages, |E|, the candidates kept by the ncandidates cap (ascending) with their pruning scores, and whether pruning ran."""
    Q = _chk(Q, np.float32)
    eoff = _chk(eoff, np.int64)
    eids = _chk(eids, np.int64)
    ids = np.empty(k, np.int32)
    sc = np.empty(k, np.float32)
    d = None
    keep = {}
    if dumps:
        cap = max(1, min(int(ncandidates), ix.P))
        keep = dict(cand=np.empty(max(ix.P, 1), np.int32), n_cand=np.zeros(1, np.int64), n_embeddings=np.zeros(1, np.int64),
                    kept=np.empty(max(ix.P, 1), np.int32), kept_scores=np.full(cap, np.nan, np.float32),
                    n_kept=np.zeros(1, np.int64), pruned=np.zeros(1, np.int32))
        d = _VanillaDumps(*[keep[n].ctypes.data for n, _ in _VanillaDumps._fields_])
    rc = _load().orc_vanilla_search(ct.byref(ix.c), _p(eoff), _p(eids), _p(Q), ct.c_int32(Q.shape[0]), ct.c_int32(nprobe),
                                    ct.c_int64(ncandidates), ct.c_int32(k), _p(ids), _p(sc),
                                    ct.byref(d) if d is not None else None)
    if rc != 0:
        raise ValueError("orc_vanilla_search: invalid arguments")
    if not dumps:
        return ids, sc
    nc, nk = int(keep["n_cand"][0]), int(keep["n_kept"][0])
    return ids, sc, dict(cand=keep["cand"][:nc].copy(), n_embeddings=int(keep["n_embeddings"][0]),
                         kept=keep["kept"][:nk].copy(), kept_scores=keep["kept_scores"][:nk].copy(),
                         pruned=bool(keep["pruned"][0]))


def search_from_S(ix: Index, Q: np.ndarray, S: np.ndarray, nprobe: int, t_cs: float, ndocs: int, k: int):
    """Stages after Eq. 2, composed from the stage functions, starting from a given S_cq.

    Tests use it to continue the pipeline from another implementation's S_cq, so that every
    later discrete decision is taken on identical fp32 inputs."""
    probed = top_nprobe(S, nprobe)
    cand = candidates(probed, ix)
    keep = keep_mask(S, t_cs)
    s2 = centroid_interaction(S, cand, ix, keep)
    sel2, sel2s = select(cand, s2, ndocs)
    s3 = centroid_interaction(S, sel2, ix, None)
    sel3, sel3s = select(sel2, s3, max(1, ndocs // 4))
    s4 = maxsim(ix, Q, sel3)
    top, tops = select(sel3, s4, k)
    ids = np.full(k, -1, np.int32)
    sc = np.full(k, -np.inf, np.float32)
    ids[:top.shape[0]] = top
    sc[:top.shape[0]] = tops
    return ids, sc, dict(S=S, probed=probed, cand=cand, keep=keep, sel2_ids=sel2, sel2_scores=sel2s, sel3_ids=sel3,
                         sel3_scores=sel3s, s4=s4)
