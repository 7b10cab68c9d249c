"""ctypes binding of libplaid.so -- same names as include/plaid.h, argument marshalling only.

Every step of the search path runs inside the HIP library; this module only turns torch tensors
into device pointers, allocates the output tensors and hands over torch's current stream.  There is
no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as ct
import os
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libplaid.so")

PLAID_QLEN = 32
PLAID_DIM = 128
PLAID_NUM_STAGES = 10
STAGE_NAMES = ("prep", "scq", "probes", "ivf_union", "stage2_ci", "select_ndocs", "stage3_ci", "select_ndocs4",
               "stage4_maxsim", "topk")

PLAID_OK, PLAID_EINVAL, PLAID_ENOMEM, PLAID_EHIP, PLAID_EIO, PLAID_EFORMAT = 0, -1, -2, -3, -4, -5
_STATUS = {0: "PLAID_OK", -1: "PLAID_EINVAL", -2: "PLAID_ENOMEM", -3: "PLAID_EHIP", -4: "PLAID_EIO", -5: "PLAID_EFORMAT"}


class PlaidError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


class plaid_index_view(ct.Structure):
    _fields_ = [("dim", ct.c_int32), ("nbits", ct.c_int32), ("num_centroids", ct.c_int64), ("num_passages", ct.c_int64),
                ("num_embeddings", ct.c_int64), ("centroids", ct.c_void_p), ("doc_offsets", ct.c_void_p),
                ("codes", ct.c_void_p), ("residuals", ct.c_void_p), ("bucket_weights", ct.c_void_p),
                ("ivf_offsets", ct.c_void_p), ("ivf_pids", ct.c_void_p), ("on_device", ct.c_int32)]


class plaid_debug_buffers(ct.Structure):
    _fields_ = [(n, ct.c_void_p) for n in ("S_cq", "probed", "cand", "n_cand", "sel2_ids", "sel2_scores", "n2",
                                            "sel3_ids", "sel3_scores", "n3", "keep")]


class plaid_vanilla_debug(ct.Structure):
    _fields_ = [(n, ct.c_void_p) for n in ("cand", "n_cand", "kept_ids", "kept_scores", "n_kept")]


EXPORTS = ("plaid_index_load", "plaid_index_from_view", "plaid_index_free", "plaid_search", "plaid_search_debug",
           "plaid_search_static", "plaid_search_vanilla", "plaid_decompress_passages", "plaid_index_info", "plaid_set_stage_timing", "plaid_get_stage_ms",
           "plaid_get_score_kernel_clocks",
           "plaid_set_max_chunk", "plaid_get_score_kernel", "plaid_get_stage2_kernel", "plaid_assign_centroids",
           "plaid_encode_residuals", "plaid_build_ivf", "plaid_workspace_bytes", "plaid_index_set_renormalize",
           "plaid_last_error")

_lib = None


def load_library() -> ct.CDLL:
    """Load libplaid.so (built in-tree by build.py).  Raises if it is absent: there is no other path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not found: run `python -m paper_2205_09707_amd.build` first")
        lib = ct.CDLL(LIB_PATH)
        lib.plaid_last_error.restype = ct.c_char_p
        lib.plaid_index_free.restype = None
        for n in EXPORTS:
            if n not in ("plaid_last_error", "plaid_index_free"):
                getattr(lib, n).restype = ct.c_int
        lib.plaid_index_load.argtypes = [ct.c_char_p, ct.c_int, ct.POINTER(ct.c_void_p)]
        lib.plaid_index_from_view.argtypes = [ct.POINTER(plaid_index_view), ct.c_int, ct.c_int, ct.POINTER(ct.c_void_p)]
        lib.plaid_index_free.argtypes = [ct.c_void_p]
        lib.plaid_search.argtypes = [ct.c_void_p, ct.c_void_p, ct.c_int32, ct.c_int32, ct.c_float, ct.c_int32, ct.c_int32,
                                     ct.c_void_p, ct.c_void_p, ct.c_void_p]
        lib.plaid_search_debug.argtypes = lib.plaid_search.argtypes + [ct.POINTER(plaid_debug_buffers)]
        lib.plaid_search_static.argtypes = lib.plaid_search.argtypes
        lib.plaid_search_vanilla.argtypes = [ct.c_void_p, ct.c_void_p, ct.c_int32, ct.c_int32, ct.c_int32, ct.c_int32, ct.c_void_p,
                                             ct.c_void_p, ct.c_void_p, ct.POINTER(plaid_vanilla_debug)]
        lib.plaid_decompress_passages.argtypes = [ct.c_void_p, ct.c_void_p, ct.c_int32, ct.c_void_p, ct.c_void_p,
                                                  ct.c_void_p, ct.c_int64, ct.c_void_p]
        lib.plaid_index_info.argtypes = [ct.c_void_p] + [ct.c_void_p] * 5
        lib.plaid_set_stage_timing.argtypes = [ct.c_void_p, ct.c_int32]
        lib.plaid_get_stage_ms.argtypes = [ct.c_void_p, ct.c_void_p]
        lib.plaid_get_score_kernel_clocks.argtypes = [ct.c_void_p, ct.c_void_p]
        lib.plaid_set_max_chunk.argtypes = [ct.c_void_p, ct.c_int32]
        lib.plaid_get_score_kernel.argtypes = [ct.c_void_p, ct.c_void_p]
        lib.plaid_get_stage2_kernel.argtypes = [ct.c_void_p, ct.c_void_p]
        lib.plaid_workspace_bytes.argtypes = [ct.c_int64, ct.c_int64, ct.c_int32, ct.c_int32, ct.c_int32, ct.c_int32, ct.c_int32,
                                              ct.POINTER(ct.c_int64), ct.POINTER(ct.c_int32)]
        lib.plaid_assign_centroids.argtypes = [ct.c_void_p, ct.c_int64, ct.c_void_p, ct.c_int64, ct.c_void_p, ct.c_int, ct.c_void_p]
        lib.plaid_encode_residuals.argtypes = [ct.c_void_p, ct.c_int64, ct.c_void_p, ct.c_void_p, ct.c_int64, ct.c_void_p,
                                               ct.c_int32, ct.c_void_p, ct.c_int, ct.c_void_p]
        lib.plaid_build_ivf.argtypes = [ct.c_void_p, ct.c_void_p, ct.c_int64, ct.c_int64, ct.c_int64, ct.c_void_p, ct.c_void_p,
                                        ct.c_int64, ct.POINTER(ct.c_int64), ct.c_int, ct.c_void_p]
        _lib = lib
    return _lib


def plaid_last_error() -> str:
    return load_library().plaid_last_error().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise PlaidError(rc, plaid_last_error())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ct.c_void_p(t.data_ptr())


def _stream(device: torch.device) -> ct.c_void_p:
    return ct.c_void_p(torch.cuda.current_stream(device).cuda_stream)


class Index:
    """Owner of a plaid_index handle (and of the tensors it borrows when copy = 0)."""

    def __init__(self, handle: int, device: torch.device, keepalive=None):
        self.handle = ct.c_void_p(handle)
        self.device = device
        self._keepalive = keepalive
        info = plaid_index_info(self)
        self.C, self.P, self.N, self.nbits, self.ivf_len = (info[k] for k in ("C", "P", "N", "nbits", "ivf_len"))

    def close(self) -> None:
        if self.handle is not None and self.handle.value:
            load_library().plaid_index_free(self.handle)
        self.handle = None
        self._keepalive = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def plaid_index_load(path: str, device: int = 0) -> Index:
    h = ct.c_void_p()
    _check(load_library().plaid_index_load(os.fsencode(path), int(device), ct.byref(h)))
    return Index(h.value, torch.device("cuda", int(device)))


_VIEW_DTYPES = dict(centroids=torch.float32, doc_offsets=torch.int64, codes=torch.int32, residuals=torch.uint8,
                    bucket_weights=torch.float32, ivf_offsets=torch.int64, ivf_pids=torch.int32)


def plaid_index_from_view(arrays: Dict[str, torch.Tensor], nbits: int, device: int = 0, copy: bool = False) -> Index:
    """arrays: centroids [C,128] f32, doc_offsets [P+1] i64, codes [N] i32, residuals [N,16*nbits] u8,
    bucket_weights [2^nbits] f32, ivf_offsets [C+1] i64, ivf_pids i32 -- all on the host or all on `device`."""
    ts = {}
    for name, dt in _VIEW_DTYPES.items():
        t = arrays[name]
        if not isinstance(t, torch.Tensor):
            t = torch.as_tensor(t)
        if t.dtype != dt:
            raise TypeError(f"{name}: expected {dt}, got {t.dtype}")
        ts[name] = t.contiguous()
    on_dev = {t.is_cuda for t in ts.values()}
    if len(on_dev) != 1:
        raise ValueError("index arrays must be all on the host or all on the device")
    on_device = on_dev.pop()
    v = plaid_index_view()
    v.dim = int(ts["centroids"].shape[1]) if ts["centroids"].dim() == 2 else -1
    v.nbits = int(nbits)
    v.num_centroids = int(ts["centroids"].shape[0])
    v.num_passages = int(ts["doc_offsets"].shape[0]) - 1
    v.num_embeddings = int(ts["codes"].shape[0])
    for name in _VIEW_DTYPES:
        setattr(v, name, ts[name].data_ptr())
    v.on_device = 1 if on_device else 0
    if ts["residuals"].numel() != v.num_embeddings * 16 * v.nbits:
        raise ValueError("residuals must hold 16*nbits bytes per token")
    if ts["bucket_weights"].numel() != (1 << v.nbits):
        raise ValueError("bucket_weights must hold 2^nbits values")
    if ts["ivf_offsets"].numel() != v.num_centroids + 1:
        raise ValueError("ivf_offsets must hold C+1 values")
    if on_device:
        ivf_len = int(ts["ivf_offsets"][-1].item())
        if ts["ivf_pids"].numel() < ivf_len:
            raise ValueError("ivf_pids shorter than ivf_offsets[C]")
    h = ct.c_void_p()
    _check(load_library().plaid_index_from_view(ct.byref(v), int(device), 1 if copy else 0, ct.byref(h)))
    return Index(h.value, torch.device("cuda", int(device)), keepalive=None if copy else ts)


def plaid_index_free(idx: Index) -> None:
    idx.close()


def plaid_index_info(idx: Index) -> Dict[str, int]:
    C, P, N, L = ct.c_int64(), ct.c_int64(), ct.c_int64(), ct.c_int64()
    nb = ct.c_int32()
    _check(load_library().plaid_index_info(idx.handle, ct.byref(C), ct.byref(P), ct.byref(N), ct.byref(nb), ct.byref(L)))
    return dict(C=C.value, P=P.value, N=N.value, nbits=nb.value, ivf_len=L.value)


def _check_Q(idx: Index, Q: torch.Tensor) -> torch.Tensor:
    if not Q.is_cuda or Q.dtype != torch.float32 or Q.dim() != 3 or Q.shape[1] != PLAID_QLEN or Q.shape[2] != PLAID_DIM:
        raise ValueError("Q must be a CUDA float32 tensor of shape [nq, 32, 128]")
    if Q.device != idx.device:
        raise ValueError("Q is on another device than the index")
    return Q.contiguous()


def plaid_search(idx: Index, Q: torch.Tensor, nprobe: int, t_cs: float, ndocs: int, k: int, out_ids=None, out_scores=None):
    """Returns (ids [nq,k] int32, scores [nq,k] float32) on the device; asynchronous on torch's current stream."""
    Q = _check_Q(idx, Q)
    nq = Q.shape[0]
    kk = max(int(k), 0)
    if out_ids is None:
        out_ids = torch.empty((nq, kk), dtype=torch.int32, device=Q.device)
    if out_scores is None:
        out_scores = torch.empty((nq, kk), dtype=torch.float32, device=Q.device)
    _check(load_library().plaid_search(idx.handle, _ptr(Q), nq, int(nprobe), float(t_cs), int(ndocs), int(k),
                                       _ptr(out_ids), _ptr(out_scores), _stream(Q.device)))
    return out_ids, out_scores


def plaid_search_static(idx: Index, Q: torch.Tensor, nprobe: int, t_cs: float, ndocs: int, k: int, out_ids: torch.Tensor,
                        out_scores: torch.Tensor):
    """plaid_search on the library's static workspace: the library allocates nothing, and neither does this wrapper, so
    the caller brings the output tensors ([nq, k] int32 / float32 on the index's device)."""
    Q = _check_Q(idx, Q)
    nq = Q.shape[0]
    if out_ids.shape != (nq, int(k)) or out_scores.shape != (nq, int(k)) or out_ids.dtype != torch.int32 or \
            out_scores.dtype != torch.float32 or not out_ids.is_contiguous() or not out_scores.is_contiguous():
        raise ValueError("out_ids / out_scores must be contiguous [nq, k] int32 / float32 tensors")
    _check(load_library().plaid_search_static(idx.handle, _ptr(Q), nq, int(nprobe), float(t_cs), int(ndocs), int(k),
                                              _ptr(out_ids), _ptr(out_scores), _stream(Q.device)))
    return out_ids, out_scores


def plaid_search_vanilla(idx: Index, Q: torch.Tensor, nprobe: int, ncandidates: int, k: int, debug: bool = False):
    """Vanilla ColBERTv2 retrieval (the paper's baseline) on the same index.  Returns (ids, scores) [nq,k] or, with
    debug, also a dict of device tensors: cand [nq,P], n_cand, kept_ids / kept_scores [nq,ncandidates], n_kept."""
    Q = _check_Q(idx, Q)
    nq = Q.shape[0]
    dev = Q.device
    out_ids = torch.empty((nq, int(k)), dtype=torch.int32, device=dev)
    out_scores = torch.empty((nq, int(k)), dtype=torch.float32, device=dev)
    bufs = None
    dbg = None
    if debug:
        bufs = dict(cand=torch.zeros((nq, idx.P), dtype=torch.int32, device=dev), n_cand=torch.zeros(nq, dtype=torch.int32, device=dev),
                    kept_ids=torch.zeros((nq, int(ncandidates)), dtype=torch.int32, device=dev),
                    kept_scores=torch.zeros((nq, int(ncandidates)), dtype=torch.float32, device=dev),
                    n_kept=torch.zeros(nq, dtype=torch.int32, device=dev))
        dbg = ct.byref(plaid_vanilla_debug(**{n: t.data_ptr() for n, t in bufs.items()}))
    _check(load_library().plaid_search_vanilla(idx.handle, _ptr(Q), nq, int(nprobe), int(ncandidates), int(k), _ptr(out_ids),
                                               _ptr(out_scores), _stream(dev), dbg))
    return (out_ids, out_scores, bufs) if debug else (out_ids, out_scores)


def plaid_search_debug(idx: Index, Q: torch.Tensor, nprobe: int, t_cs: float, ndocs: int, k: int, want=None):
    """plaid_search plus the per-stage intermediates of include/plaid.h's plaid_debug_buffers (device tensors).
    `want` restricts which buffers are allocated (default: all)."""
    Q = _check_Q(idx, Q)
    nq = Q.shape[0]
    dev = Q.device
    m3 = max(1, int(ndocs) // 4)
    shapes = dict(S_cq=((nq, idx.C, PLAID_QLEN), torch.float32), probed=((nq, PLAID_QLEN, int(nprobe)), torch.int32),
                  cand=((nq, idx.P), torch.int32), n_cand=((nq,), torch.int32),
                  sel2_ids=((nq, int(ndocs)), torch.int32), sel2_scores=((nq, int(ndocs)), torch.float32),
                  n2=((nq,), torch.int32), sel3_ids=((nq, m3), torch.int32), sel3_scores=((nq, m3), torch.float32),
                  n3=((nq,), torch.int32), keep=((nq, (idx.C + 31) // 32), torch.int32))
    names = list(shapes) if want is None else list(want)
    bufs = {n: torch.zeros(shapes[n][0], dtype=shapes[n][1], device=dev) for n in names}
    dbg = plaid_debug_buffers(**{n: bufs[n].data_ptr() for n in names})
    out_ids = torch.empty((nq, int(k)), dtype=torch.int32, device=dev)
    out_scores = torch.empty((nq, int(k)), dtype=torch.float32, device=dev)
    _check(load_library().plaid_search_debug(idx.handle, _ptr(Q), nq, int(nprobe), float(t_cs), int(ndocs), int(k),
                                             _ptr(out_ids), _ptr(out_scores), _stream(dev), ct.byref(dbg)))
    return out_ids, out_scores, bufs


def plaid_decompress_passages(idx: Index, pids: torch.Tensor, capacity: int, vectors: bool = True, indices: bool = True):
    """Returns (offsets [n+1] int64, vectors [capacity,128] f32 or None, bucket indices [capacity,128] u8 or None)."""
    if not pids.is_cuda or pids.dtype != torch.int32 or pids.dim() != 1:
        raise ValueError("pids must be a 1-d CUDA int32 tensor")
    pids = pids.contiguous()
    n = pids.shape[0]
    dev = pids.device
    offs = torch.empty(n + 1, dtype=torch.int64, device=dev)
    vec = torch.empty((capacity, PLAID_DIM), dtype=torch.float32, device=dev) if vectors else None
    ind = torch.empty((capacity, PLAID_DIM), dtype=torch.uint8, device=dev) if indices else None
    _check(load_library().plaid_decompress_passages(idx.handle, _ptr(pids), n, _ptr(offs), _ptr(vec), _ptr(ind),
                                                    int(capacity), _stream(dev)))
    return offs, vec, ind


def plaid_set_stage_timing(idx: Index, on: bool) -> None:
    _check(load_library().plaid_set_stage_timing(idx.handle, 1 if on else 0))


def plaid_get_stage_ms(idx: Index) -> Dict[str, float]:
    arr = (ct.c_float * PLAID_NUM_STAGES)()
    _check(load_library().plaid_get_stage_ms(idx.handle, arr))
    return {STAGE_NAMES[i]: float(arr[i]) for i in range(PLAID_NUM_STAGES)}


def plaid_get_score_kernel_clocks(idx: Index):
    """(shader-clock ticks, 100 MHz timer ticks) summed over the workgroups of the S_cq kernel of the last timed search."""
    arr = (ct.c_uint64 * 2)()
    _check(load_library().plaid_get_score_kernel_clocks(idx.handle, arr))
    return int(arr[0]), int(arr[1])


def plaid_set_max_chunk(idx: Index, max_queries_per_chunk: int) -> None:
    _check(load_library().plaid_set_max_chunk(idx.handle, int(max_queries_per_chunk)))


def plaid_index_set_renormalize(idx: Index, on: bool) -> None:
    """Storage variant: score (stage 4) and return (plaid_decompress_passages) reconstructed vectors scaled back to unit
    length.  The first call that switches it on computes one factor per token on the device."""
    lib = load_library()
    lib.plaid_index_set_renormalize.argtypes = [ct.c_void_p, ct.c_int32]
    _check(lib.plaid_index_set_renormalize(idx.handle, 1 if on else 0))


def plaid_get_score_kernel(idx: Index) -> int:
    """The kernel that computes S_cq for this index: 2 = fp16 matrix instruction on two-term operand splits (decisions
    completed in double), 1 = double-precision matrix instruction, 0 = double-precision vector FMA chain."""
    form = ct.c_int32(-1)
    _check(load_library().plaid_get_score_kernel(idx.handle, ct.byref(form)))
    return int(form.value)


def plaid_get_stage2_kernel(idx: Index) -> int:
    """1 when candidates and pruned scores come from the inverted lists, 0 for list union + code stream."""
    form = ct.c_int32(-1)
    _check(load_library().plaid_get_stage2_kernel(idx.handle, ct.byref(form)))
    return int(form.value)


def plaid_workspace_bytes(C: int, P: int, nq: int, nprobe: int, ndocs: int, k: int, max_queries_per_chunk: int = 0):
    """(bytes of device workspace a search with these parameters needs, queries per internal chunk); no GPU involved."""
    b, qc = ct.c_int64(0), ct.c_int32(0)
    _check(load_library().plaid_workspace_bytes(int(C), int(P), int(nq), int(nprobe), int(ndocs), int(k),
                                                int(max_queries_per_chunk), ct.byref(b), ct.byref(qc)))
    return int(b.value), int(qc.value)


# ------------------------------------------------------------------ index construction
def _dev_tensor(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype:
        raise ValueError(f"{name} must be a CUDA tensor of dtype {dtype}")
    return t.contiguous()


def plaid_assign_centroids(centroids: torch.Tensor, x: torch.Tensor) -> torch.Tensor:
    """codes [n] int32: the nearest centroid (largest dot product, ties to the smaller id) of each row of x [n, 128]."""
    centroids = _dev_tensor(centroids, torch.float32, "centroids")
    x = _dev_tensor(x, torch.float32, "x")
    codes = torch.empty((x.shape[0],), dtype=torch.int32, device=x.device)
    _check(load_library().plaid_assign_centroids(_ptr(centroids), centroids.shape[0], _ptr(x), x.shape[0], _ptr(codes),
                                                 x.device.index or 0, _stream(x.device)))
    return codes


def plaid_encode_residuals(centroids: torch.Tensor, x: torch.Tensor, codes: torch.Tensor, cutoffs: torch.Tensor,
                           nbits: int) -> torch.Tensor:
    """residuals [n, 16 * nbits] uint8: packed bucket indices of x - centroids[codes]."""
    centroids = _dev_tensor(centroids, torch.float32, "centroids")
    x = _dev_tensor(x, torch.float32, "x")
    codes = _dev_tensor(codes, torch.int32, "codes")
    cutoffs = _dev_tensor(cutoffs, torch.float32, "cutoffs")
    if cutoffs.numel() != (1 << int(nbits)) - 1:
        raise ValueError("cutoffs must hold 2^nbits - 1 values")
    out = torch.empty((x.shape[0], 16 * int(nbits)), dtype=torch.uint8, device=x.device)
    _check(load_library().plaid_encode_residuals(_ptr(centroids), centroids.shape[0], _ptr(x), _ptr(codes), x.shape[0],
                                                 _ptr(cutoffs), int(nbits), _ptr(out), x.device.index or 0, _stream(x.device)))
    return out


def plaid_build_ivf(codes: torch.Tensor, doc_offsets: torch.Tensor, num_centroids: int):
    """(ivf_offsets [C+1] int64, ivf_pids int32): per centroid the ascending unique ids of the passages that contain it."""
    codes = _dev_tensor(codes, torch.int32, "codes")
    doc_offsets = _dev_tensor(doc_offsets, torch.int64, "doc_offsets")
    dev = codes.device
    P, N, C = doc_offsets.shape[0] - 1, codes.shape[0], int(num_centroids)
    off = torch.empty((C + 1,), dtype=torch.int64, device=dev)
    total = ct.c_int64(0)
    lib = load_library()
    # one call: the lists hold at most one entry per token, so a buffer of N entries always suffices
    pids = torch.empty((max(N, 1),), dtype=torch.int32, device=dev)
    _check(lib.plaid_build_ivf(_ptr(codes), _ptr(doc_offsets), P, N, C, _ptr(off), _ptr(pids), pids.shape[0], ct.byref(total),
                               dev.index or 0, _stream(dev)))
    return off, pids[:int(total.value)]
