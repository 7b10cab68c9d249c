"""GPU parity of the index-construction calls (nearest-centroid assignment, residual encoding, inverted lists) against
the CPU oracle, bit for bit, and of a search over an index whose arrays were all built on the GPU.

Runs only on a machine with an MI355X (`-m gpu`).
"""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from synth import make_workload, tiny_config

import parity_util as pu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pl():
    import paper_2205_09707_amd as pl_
    pl_.load_library()   # fails loudly when libplaid.so has not been built
    assert torch.cuda.is_available(), "these tests need the GPU"
    return pl_


def _workload(nbits=2, C=64, P=300, lo=0, hi=50, seed=51):
    w = make_workload(tiny_config(C=C, P=P, lo=lo, hi=hi, nbits=nbits, nq=2, seed=seed), noise="calibrated",
                      keep_embeddings=1 << 30)
    assert w.sample_embeddings.shape[0] == w.codes.shape[0]   # the uncompressed vector of every token
    return w


def _oracle_nearest(centroids: np.ndarray, x: np.ndarray) -> np.ndarray:
    """argmax_c of the Eq. 2 scores (double accumulation, one rounding), ties to the smaller id: the oracle's S_cq routine
    on groups of up to 32 vectors followed by its top-1 routine."""
    out = np.empty(x.shape[0], np.int32)
    for a in range(0, x.shape[0], 32):
        S = orc.scq(centroids, x[a:a + 32])
        out[a:a + 32] = orc.top_nprobe(S, 1)[:, 0]
    return out


@pytest.mark.parametrize("nbits", [2, 1])
def test_encode_residuals_bit_exact(pl, nbits):
    w = _workload(nbits=nbits)
    a = w.numpy()
    x = w.sample_embeddings.numpy()
    cut = w.bucket_cutoffs.numpy()
    want = orc.encode(x, a["codes"], a["centroids"], cut, nbits)
    np.testing.assert_array_equal(want, a["residuals"])   # the generator's own encoder agrees with the oracle's
    got = pl.plaid_encode_residuals(w.centroids.to(DEV), w.sample_embeddings.to(DEV), w.codes.to(DEV), w.bucket_cutoffs.to(DEV),
                                    nbits)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy(), want)


def test_encode_residuals_at_the_cutoffs(pl):
    """A residual equal to a cut-off goes to the lower bucket; the first dimension lands in the top bits of its byte."""
    cut = np.array([-0.25, 0.0, 0.5], np.float32)
    cen = np.zeros((1, 128), np.float32)
    x = np.zeros((3, 128), np.float32)
    x[0, :8] = [-1.0, -0.25, -0.2, 0.0, 0.1, 0.5, 0.6, 9.0]
    x[1, :] = np.nextafter(np.float32(0.5), np.float32(1.0))
    x[2, 127] = 1.0
    codes = np.zeros(3, np.int32)
    want = orc.encode(x, codes, cen, cut, 2)
    got = pl.plaid_encode_residuals(torch.from_numpy(cen).to(DEV), torch.from_numpy(x).to(DEV), torch.from_numpy(codes).to(DEV),
                                    torch.from_numpy(cut).to(DEV), 2)
    np.testing.assert_array_equal(got.cpu().numpy(), want)
    assert want[0, 0] == (0 << 6 | 0 << 4 | 1 << 2 | 1) and want[0, 1] == (2 << 6 | 2 << 4 | 3 << 2 | 3)


@pytest.mark.parametrize("n_extra", [0, 5, 31])
def test_assign_centroids_equals_oracle(pl, n_extra):
    """Token vectors of a small index plus adversarial rows: copies of centroids, a pair of identical centroids (a tie:
    the smaller id wins), a zero vector (every centroid ties: id 0).  n_extra makes the count ragged against 32."""
    w = _workload(C=200, P=150, lo=1, hi=30, seed=52)
    cen = w.centroids.numpy().copy()
    cen[77] = cen[13]                                  # two identical centroids
    x = np.concatenate([cen[[13, 77, 199, 0]], np.zeros((1, 128), np.float32), w.sample_embeddings.numpy()])
    n = ((x.shape[0] - 32) // 32) * 32 + n_extra
    x = np.ascontiguousarray(x[:n])
    x[-1] = cen[77] * np.float32(0.5)                  # the tie also in the last (possibly incomplete) group
    want = _oracle_nearest(cen, x)
    got = pl.plaid_assign_centroids(torch.from_numpy(cen).to(DEV), torch.from_numpy(x).to(DEV))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy(), want)
    assert want[-1] == 13


def test_assign_centroids_in_several_chunks(pl):
    """More groups of 32 than one internal chunk holds (512), with a ragged tail."""
    g = torch.Generator().manual_seed(53)
    cen = torch.nn.functional.normalize(torch.randn(48, 128, generator=g), dim=1)
    x = torch.nn.functional.normalize(torch.randn(512 * 32 * 2 + 32 * 3 + 7, 128, generator=g), dim=1)
    want = _oracle_nearest(cen.numpy(), x.numpy())
    got = pl.plaid_assign_centroids(cen.to(DEV), x.to(DEV))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy(), want)


IVF_CASES = [
    dict(C=64, P=300, lo=0, hi=50, seed=54),        # empty passages among them
    dict(C=5, P=4000, lo=1, hi=6, seed=55),         # more passages than groups: several passages per group; long lists
    dict(C=1, P=9, lo=1, hi=5, seed=56),            # a single centroid
    dict(C=300, P=1, lo=40, hi=40, seed=57),        # a single passage
    dict(C=50, P=6, lo=2300, hi=2400, seed=58),     # passages far longer than a wave
]


@pytest.mark.parametrize("kw", IVF_CASES, ids=[f"C{k['C']}_P{k['P']}" for k in IVF_CASES])
def test_build_ivf_equals_oracle(pl, kw):
    w = make_workload(tiny_config(nbits=2, nq=1, **kw), noise="calibrated")
    a = w.numpy()
    off, pids = orc.build_ivf(a["codes"], a["doc_offsets"], w.cfg.C)
    np.testing.assert_array_equal(off, a["ivf_offsets"])
    np.testing.assert_array_equal(pids, a["ivf_pids"])
    goff, gpids = pl.plaid_build_ivf(w.codes.to(DEV), w.doc_offsets.to(DEV), w.cfg.C)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(goff.cpu().numpy(), off)
    np.testing.assert_array_equal(gpids.cpu().numpy(), pids)
    # twice: the lists are deterministic
    goff2, gpids2 = pl.plaid_build_ivf(w.codes.to(DEV), w.doc_offsets.to(DEV), w.cfg.C)
    assert torch.equal(goff, goff2) and torch.equal(gpids, gpids2)


def test_build_ivf_long_lists_over_several_id_ranges(pl):
    """More than 2^20 passages, two lists that hold a third of them each (sorted through the bitmap, one range of 2^20
    ids at a time), the rest short (sorted by a wave), some of them empty."""
    rng = np.random.default_rng(62)
    P, C = 1_300_000, 5000
    lengths = rng.integers(0, 3, size=P)
    doc_offsets = np.zeros(P + 1, dtype=np.int64)
    np.cumsum(lengths, out=doc_offsets[1:])
    N = int(doc_offsets[-1])
    codes = np.where(rng.random(N) < 0.5, rng.integers(0, 2, size=N), rng.integers(2, C - 100, size=N)).astype(np.int32)
    off, pids = orc.build_ivf(codes, doc_offsets, C)
    assert off[1] - off[0] > (1 << 18) and np.all(off[C - 100:] == off[C])
    goff, gpids = pl.plaid_build_ivf(torch.from_numpy(codes).to(DEV), torch.from_numpy(doc_offsets).to(DEV), C)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(goff.cpu().numpy(), off)
    np.testing.assert_array_equal(gpids.cpu().numpy(), pids)


def test_build_ivf_with_two_million_centroids(pl):
    """So many centroids that the counter tables get fewer stripes than the usual 64; one list is long."""
    rng = np.random.default_rng(63)
    P, C = 3000, (1 << 21) + 7
    lengths = rng.integers(1, 7, size=P)
    doc_offsets = np.zeros(P + 1, dtype=np.int64)
    np.cumsum(lengths, out=doc_offsets[1:])
    N = int(doc_offsets[-1])
    codes = rng.integers(0, C, size=N).astype(np.int32)
    codes[doc_offsets[:2500]] = 5                     # the first token of 2500 passages
    codes[doc_offsets[:2500:2] + lengths[:2500:2] - 1] = 5   # and, in every other one, the last token too (counted once)
    off, pids = orc.build_ivf(codes, doc_offsets, C)
    assert off[6] - off[5] == 2500
    goff, gpids = pl.plaid_build_ivf(torch.from_numpy(codes).to(DEV), torch.from_numpy(doc_offsets).to(DEV), C)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(goff.cpu().numpy(), off)
    np.testing.assert_array_equal(gpids.cpu().numpy(), pids)


def test_index_built_on_the_gpu_searches_like_the_oracle(pl):
    """Assignment, encoding and inverted lists on the GPU; the oracle searches an index made of those very arrays."""
    w = _workload(C=128, P=400, lo=1, hi=40, seed=59)
    cen, x = w.centroids.to(DEV), w.sample_embeddings.to(DEV)
    codes = pl.plaid_assign_centroids(cen, x)
    res = pl.plaid_encode_residuals(cen, x, codes, w.bucket_cutoffs.to(DEV), 2)
    off, pids = pl.plaid_build_ivf(codes, w.doc_offsets.to(DEV), w.cfg.C)
    torch.cuda.synchronize()
    arrays = dict(centroids=cen, doc_offsets=w.doc_offsets.to(DEV), codes=codes, residuals=res,
                  bucket_weights=w.bucket_weights.to(DEV), ivf_offsets=off, ivf_pids=pids.contiguous())
    ix = orc.Index({k: v.cpu().numpy() for k, v in arrays.items()}, 2)
    gidx = pl.plaid_index_from_view(arrays, 2, device=0, copy=True)
    try:
        Qdev = w.queries.to(DEV)
        for params in [(2, 0.45, 64, 10), (4, -np.inf, 1700, 30)]:
            out = pu.run_gpu_debug(pl, gidx, Qdev, params)
            for q in range(w.queries.shape[0]):
                pu.compare_query(ix, w.queries[q].numpy(), params, pu.slice_query(out, q), ctx=f"gpu-built {params} q{q}",
                                 approx=pu.is_approx(pl, gidx, params))
    finally:
        pl.plaid_index_free(gidx)


def test_index_build_argument_errors(pl):
    w = _workload(C=16, P=20, lo=1, hi=5, seed=60)
    cen, x, codes = w.centroids.to(DEV), w.sample_embeddings.to(DEV), w.codes.to(DEV)
    bad = codes.clone()
    bad[3] = 16                                         # one past the last centroid
    with pytest.raises(pl.PlaidError):
        pl.plaid_encode_residuals(cen, x, bad, w.bucket_cutoffs.to(DEV), 2)
    with pytest.raises(pl.PlaidError):
        pl.plaid_build_ivf(bad, w.doc_offsets.to(DEV), 16)
    with pytest.raises(pl.PlaidError):
        pl.plaid_build_ivf(codes, w.doc_offsets.to(DEV)[:-1].contiguous(), 16)     # offsets do not end at N
    back = w.doc_offsets.clone()
    back[5] = back[3]                                   # passage 4 would end before it starts, passage 5 overlaps 3 and 4
    if int(back[5]) < int(back[4]):
        with pytest.raises(pl.PlaidError):
            pl.plaid_build_ivf(codes, back.to(DEV), 16)
    with pytest.raises(pl.PlaidError):
        pl.plaid_encode_residuals(cen, x, codes, torch.zeros(7, device=DEV), 3)      # nbits must be 1 or 2
    with pytest.raises(ValueError):
        pl.plaid_encode_residuals(cen, x, codes, w.bucket_cutoffs.to(DEV)[:1], 2)
    with pytest.raises(pl.PlaidError):
        pl.plaid_assign_centroids(cen, x.flatten()[1:-127].view(-1, 128))        # not 16-byte aligned
    torch.cuda.synchronize()
    # the library still works afterwards
    np.testing.assert_array_equal(pl.plaid_build_ivf(codes, w.doc_offsets.to(DEV), 16)[0].cpu().numpy(), w.ivf_offsets.numpy())
