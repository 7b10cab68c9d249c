"""CPU-side checks of libplaid.so: it loads, exports every function include/plaid.h declares, and its
host-side validation rejects malformed input before any device is touched.  No compute calls."""
import ctypes as ct
import os
import re
import struct

import numpy as np
import pytest

import paper_2205_09707_amd as pl
from paper_2205_09707_amd import plaid
from synth import make_workload, save_index_file, tiny_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "plaid.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(plaid.LIB_PATH):
        from paper_2205_09707_amd import build
        build.build()
    return pl.load_library()


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(plaid_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert "plaid_search" in names and "plaid_index_load" in names and len(names) >= 10
    for n in names:
        assert hasattr(lib, n), f"{n} declared in plaid.h but not exported by libplaid.so"
    assert sorted(plaid.EXPORTS) == names, "the Python binding must carry the same names as the header"


def _struct_fields(name):
    """(type, field) pairs of `typedef struct { ... } name;` in the header, in declaration order"""
    src = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    body = re.search(r"typedef struct\s*\{([^}]*)\}\s*" + name + r"\s*;", src, flags=re.S).group(1)
    out = []
    for decl in body.split(";"):
        decl = " ".join(decl.split())
        if decl:
            m = re.match(r"(.*?)(\*?)\s*([A-Za-z_0-9]+)$", decl)
            out.append(((m.group(1).strip() + m.group(2)).replace(" *", "*"), m.group(3)))
    return out


def test_binding_structs_mirror_the_header():
    """Field order and widths of the two structs that cross the boundary by pointer."""
    ctype_of = {"int32_t": ct.c_int32, "int64_t": ct.c_int64}
    for name, cls in (("plaid_index_view", plaid.plaid_index_view), ("plaid_debug_buffers", plaid.plaid_debug_buffers)):
        fields = _struct_fields(name)
        assert [f for _, f in fields] == [f for f, _ in cls._fields_], name
        for (ctype, field), (_, pytype) in zip(fields, cls._fields_):
            want = ct.c_void_p if ctype.endswith("*") else ctype_of[ctype]
            assert pytype is want, f"{name}.{field}: header says {ctype}"


def _view(w, **over):
    a = w.numpy()
    v = plaid.plaid_index_view()
    v.dim, v.nbits = 128, w.cfg.nbits
    v.num_centroids, v.num_passages, v.num_embeddings = a["centroids"].shape[0], a["doc_offsets"].shape[0] - 1, a["codes"].shape[0]
    for n in ("centroids", "doc_offsets", "codes", "residuals", "bucket_weights", "ivf_offsets", "ivf_pids"):
        setattr(v, n, a[n].ctypes.data)
    v.on_device = 0
    for k, val in over.items():
        setattr(v, k, val)
    return v, a


def test_from_view_rejects_malformed_host_views(lib):
    w = make_workload(tiny_config(C=8, P=10, lo=1, hi=4, nbits=2, nq=1, seed=1), noise="literal")
    h = ct.c_void_p()

    def call(v, copy=1):
        return lib.plaid_index_from_view(ct.byref(v), 0, copy, ct.byref(h))

    assert lib.plaid_index_from_view(None, 0, 1, ct.byref(h)) == plaid.PLAID_EINVAL
    v, keep = _view(w, dim=64)
    assert call(v) == plaid.PLAID_EINVAL and "dim" in pl.plaid_last_error()
    v, keep = _view(w, nbits=3)
    assert call(v) == plaid.PLAID_EINVAL
    v, keep = _view(w, centroids=None)
    assert call(v) == plaid.PLAID_EINVAL
    v, keep = _view(w)
    assert call(v, copy=0) == plaid.PLAID_EINVAL            # host arrays cannot be adopted
    v, keep = _view(w, num_embeddings=keep["codes"].shape[0] + 1)
    assert call(v) == plaid.PLAID_EINVAL                    # doc_offsets[P] != N
    v, keep = _view(w)
    keep["codes"][3] = 8                                    # centroid id out of range
    assert call(v) == plaid.PLAID_EINVAL and "codes[3]" in pl.plaid_last_error()
    v, keep = _view(w)
    keep["doc_offsets"][4] = keep["doc_offsets"][5] + 1     # offsets decrease
    assert call(v) == plaid.PLAID_EINVAL
    v, keep = _view(w)
    lst = [c for c in range(8) if keep["ivf_offsets"][c + 1] - keep["ivf_offsets"][c] >= 2][0]
    e = keep["ivf_offsets"][lst]
    keep["ivf_pids"][e + 1] = keep["ivf_pids"][e]           # list no longer strictly ascending
    assert call(v) == plaid.PLAID_EINVAL
    assert h.value is None


def test_index_load_errors(lib, tmp_path):
    h = ct.c_void_p()
    assert lib.plaid_index_load(None, 0, ct.byref(h)) == plaid.PLAID_EINVAL
    assert lib.plaid_index_load(os.fsencode(str(tmp_path / "missing")), 0, ct.byref(h)) == plaid.PLAID_EIO
    bad = tmp_path / "bad"
    bad.write_bytes(b"NOTANIDX" + b"\0" * 100)
    assert lib.plaid_index_load(os.fsencode(str(bad)), 0, ct.byref(h)) == plaid.PLAID_EFORMAT
    w = make_workload(tiny_config(C=8, P=10, lo=1, hi=4, nbits=2, nq=1, seed=1), noise="literal")
    good = tmp_path / "good"
    save_index_file(str(good), w.numpy(), 2)
    data = good.read_bytes()
    assert len(data) % 64 == 0 and data[:8] == b"PLAIDIX1"
    dim, nbits, C, P, N, L = struct.unpack("<iiqqqq", data[8:48])
    assert (dim, nbits, C, P, N) == (128, 2, 8, 10, w.N) and L == w.ivf_pids.numel()
    trunc = tmp_path / "trunc"
    trunc.write_bytes(data[: len(data) - 64])
    assert lib.plaid_index_load(os.fsencode(str(trunc)), 0, ct.byref(h)) == plaid.PLAID_EFORMAT
    hdr = bytearray(data)
    hdr[12:16] = struct.pack("<i", 5)                       # nbits = 5
    (tmp_path / "hdr").write_bytes(bytes(hdr))
    assert lib.plaid_index_load(os.fsencode(str(tmp_path / "hdr")), 0, ct.byref(h)) == plaid.PLAID_EFORMAT


def test_null_handles(lib):
    lib.plaid_index_free(None)                              # allowed
    buf = (ct.c_float * 8)()
    assert lib.plaid_get_stage_ms(None, buf) == plaid.PLAID_EINVAL
    assert lib.plaid_set_stage_timing(None, 1) == plaid.PLAID_EINVAL
    assert lib.plaid_set_max_chunk(None, 4) == plaid.PLAID_EINVAL
    assert lib.plaid_index_info(None, None, None, None, None, None) == plaid.PLAID_EINVAL
    assert lib.plaid_search(None, None, 1, 1, ct.c_float(0.5), 4, 2, None, None, None) == plaid.PLAID_EINVAL
    assert lib.plaid_decompress_passages(None, None, 0, None, None, None, 0, None) == plaid.PLAID_EINVAL


def test_index_construction_rejects_bad_arguments_before_touching_the_gpu(lib):
    """Sizes, null pointers and alignment are checked on the host first, so these calls fail with PLAID_EINVAL even on a
    machine without a GPU (the pointer values below are never dereferenced)."""
    ok16, odd = ct.c_void_p(4096), ct.c_void_p(4100)        # 16-byte aligned / only 4-byte aligned
    total = ct.c_int64(-1)
    E = plaid.PLAID_EINVAL
    assert lib.plaid_assign_centroids(None, 8, ok16, 4, ok16, 0, None) == E
    assert lib.plaid_assign_centroids(ok16, 0, ok16, 4, ok16, 0, None) == E               # no centroids
    assert lib.plaid_assign_centroids(ok16, 8, ok16, -1, ok16, 0, None) == E
    assert lib.plaid_assign_centroids(ok16, 8, odd, 4, ok16, 0, None) == E                # x not 16-byte aligned
    assert lib.plaid_assign_centroids(ok16, 8, None, 4, ok16, 0, None) == E
    assert lib.plaid_encode_residuals(ok16, 8, ok16, ok16, 4, ok16, 3, ok16, 0, None) == E   # nbits
    assert lib.plaid_encode_residuals(ok16, 8, ok16, ok16, 4, None, 2, ok16, 0, None) == E   # no cut-offs
    assert lib.plaid_encode_residuals(odd, 8, ok16, ok16, 4, ok16, 2, ok16, 0, None) == E    # centroids misaligned
    assert lib.plaid_encode_residuals(ok16, 8, ok16, ok16, 4, ok16, 2, ct.c_void_p(4098), 0, None) == E  # output misaligned
    assert lib.plaid_encode_residuals(ok16, 1 << 31, ok16, ok16, 4, ok16, 2, ok16, 0, None) == E
    assert lib.plaid_build_ivf(ok16, None, 4, 10, 8, ok16, None, 0, ct.byref(total), 0, None) == E   # no offsets
    assert lib.plaid_build_ivf(ok16, ok16, 0, 10, 8, ok16, None, 0, ct.byref(total), 0, None) == E   # no passages
    assert lib.plaid_build_ivf(ok16, ok16, 4, 10, 0, ok16, None, 0, ct.byref(total), 0, None) == E   # no centroids
    assert lib.plaid_build_ivf(ok16, ok16, 4, -1, 8, ok16, None, 0, ct.byref(total), 0, None) == E
    assert lib.plaid_build_ivf(ok16, ok16, 4, 10, 8, None, None, 0, ct.byref(total), 0, None) == E
    assert total.value == -1                                                                   # untouched on error
    assert b"" != lib.plaid_last_error()


def test_workspace_size_arithmetic():
    """plaid_workspace_bytes is host arithmetic: per query about 132 C + 16 P bytes plus the selection lists, the chunk is
    512 queries unless the caller's limit, the batch or the 24 GiB budget is smaller, and nothing depends on nq beyond it."""
    C, P = 65536, 400000                                     # the benchmark configuration
    one, qc1 = pl.plaid_workspace_bytes(C, P, 1, 2, 1024, 100)
    assert qc1 == 1 and 132 * C + 16 * P <= one <= 1.1 * (132 * C + 16 * P) + (1 << 20)
    b512, qc = pl.plaid_workspace_bytes(C, P, 512, 2, 1024, 100)
    assert qc == 512 and 0.9 * 512 * (132 * C + 16 * P) <= b512 <= 512 * one
    assert pl.plaid_workspace_bytes(C, P, 5000, 2, 1024, 100) == (b512, 512)          # more queries: more chunks, same memory
    b64, qc = pl.plaid_workspace_bytes(C, P, 512, 2, 1024, 100, max_queries_per_chunk=64)
    assert qc == 64 and b64 < b512 / 7
    big, qc = pl.plaid_workspace_bytes(262144, 20_000_000, 1000, 4, 4096, 100)           # 1-bit configuration: the budget binds
    assert 1 <= qc < 512 and big <= (24 << 30) + (1 << 28)
    sizes = [pl.plaid_workspace_bytes(C, P, 16, nprobe, 1024, 100)[0] for nprobe in (1, 2, 8, 9, 64)]
    assert sizes == sorted(sizes)
    with pytest.raises(pl.PlaidError):
        pl.plaid_workspace_bytes(C, P, 0, 2, 1024, 100)
    with pytest.raises(pl.PlaidError):
        pl.plaid_workspace_bytes(C, P, 1, C + 1, 1024, 100)


def test_binding_refuses_cpu_tensors():
    import torch
    class Fake:
        device = torch.device("cuda", 0)
        handle = ct.c_void_p(1)
    with pytest.raises(ValueError):
        pl.plaid_search(Fake(), torch.zeros(1, 32, 128), 1, 0.5, 4, 2)
