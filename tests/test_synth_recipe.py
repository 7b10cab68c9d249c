"""The synthetic workload honours its recipe (it stands in for the paper's collections, which are not available): seeded
and reproducible, unit-norm centroids / embeddings / queries, lengths inside their range, Zipf-distributed codes with
the stated head share, bucket populations near equal, the two readings of the noise scale with the cosines they imply,
inverted lists consistent with the codes, sizes equal to the storage formula of Section 3.1.  CPU only."""
import functools

import numpy as np
import torch

from synth import get_config, make_workload
from synth.workload import index_nbytes


@functools.lru_cache(maxsize=None)
def _w(noise):
    return make_workload(get_config("cfg1"), device="cpu", noise=noise, keep_embeddings=1 << 30)


def test_same_seed_same_workload_and_other_seed_another():
    cfg = get_config("cfg1")
    a, b = make_workload(cfg, noise="literal"), make_workload(cfg, noise="literal")
    for f in ("centroids", "doc_offsets", "codes", "residuals", "bucket_weights", "ivf_offsets", "ivf_pids", "queries"):
        assert torch.equal(getattr(a, f), getattr(b, f)), f
    c = make_workload(cfg.replace(index_seed=cfg.index_seed + 1), noise="literal")
    assert not torch.equal(a.codes[:1000], c.codes[:1000])


def test_shapes_norms_and_ranges():
    w = _w("calibrated")
    cfg = w.cfg
    C, P = cfg.C, cfg.P
    assert w.centroids.shape == (C, 128) and w.doc_offsets.shape == (P + 1,) and w.queries.shape == (cfg.nq, 32, 128)
    np.testing.assert_allclose(w.centroids.norm(dim=1).numpy(), 1.0, atol=1e-5)
    np.testing.assert_allclose(w.sample_embeddings.norm(dim=1).numpy(), 1.0, atol=1e-5)
    np.testing.assert_allclose(w.queries.norm(dim=2).numpy(), 1.0, atol=1e-5)
    lens = (w.doc_offsets[1:] - w.doc_offsets[:-1]).numpy()
    assert lens.min() >= 20 and lens.max() <= 60 and abs(lens.mean() - 40) < 1.0           # uniform on [20, 60]
    assert int(w.doc_offsets[0]) == 0 and int(w.doc_offsets[-1]) == w.N
    assert w.codes.min() >= 0 and w.codes.max() < C
    assert w.residuals.shape == (w.N, 16 * cfg.nbits) and w.residuals.dtype == torch.uint8
    assert w.residuals.numel() + 4 * w.N == index_nbytes(w.N, cfg.nbits)                   # 4 + 16 b bytes per token


def test_codes_follow_the_zipf_law():
    w = _w("literal")
    C = w.cfg.C
    counts = np.bincount(w.codes.numpy(), minlength=C).astype(np.float64)
    p = (np.arange(1, C + 1) ** -1.1)
    p /= p.sum()
    assert abs(counts[0] / counts.sum() - p[0]) < 0.01                                      # head share (about 18 % at C = 1024)
    top = slice(0, 16)
    np.testing.assert_allclose(counts[top] / counts.sum(), p[top], rtol=0.1)


def test_buckets_are_about_equally_populated():
    w = _w("calibrated")
    res = w.residuals.numpy()
    idx = np.stack([(res >> s) & 3 for s in (6, 4, 2, 0)], axis=-1).reshape(-1)             # 2-bit indices, first dimension on top
    share = np.bincount(idx, minlength=4) / idx.size
    np.testing.assert_allclose(share, 0.25, atol=0.01)
    cut, wts = w.bucket_cutoffs.numpy(), w.bucket_weights.numpy()
    assert np.all(np.diff(cut) > 0) and np.all(np.diff(wts) > 0)
    assert wts[0] < cut[0] < wts[1] < cut[1] < wts[2] < cut[2] < wts[3]


def test_the_two_noise_readings():
    """Per-coordinate sigma (the configuration text read literally) leaves cos(token, its centroid) near 0.5; a noise
    vector of norm sigma leaves it near 0.99: the small tail of high centroid scores the paper's Figure 5 shows."""
    lit, cal = _w("literal"), _w("calibrated")
    for w, lo, hi in ((lit, 0.45, 0.57), (cal, 0.98, 0.995)):
        x = w.sample_embeddings[:4096]
        c = w.centroids[w.codes[:4096].long()]
        cos = (x * c).sum(dim=1).mean().item()
        assert lo < cos < hi, (w.noise, cos)
    # a query token is a noisy copy of the token it was drawn from
    t = cal.query_src_tokens[0]
    cosq = (cal.queries[0] * cal.sample_embeddings[t]).sum(dim=1).mean().item()
    assert cosq > 0.95


def test_inverted_lists_match_the_codes():
    w = _w("literal")
    off, pids, codes, doc = w.ivf_offsets.numpy(), w.ivf_pids.numpy(), w.codes.numpy(), w.doc_offsets.numpy()
    tok_pid = np.repeat(np.arange(w.cfg.P), np.diff(doc))
    pairs = np.unique(np.stack([codes.astype(np.int64), tok_pid], axis=1), axis=0)          # sorted by (code, pid)
    assert pairs.shape[0] == off[-1]
    np.testing.assert_array_equal(pids, pairs[:, 1])
    np.testing.assert_array_equal(np.diff(off), np.bincount(pairs[:, 0], minlength=w.cfg.C))
