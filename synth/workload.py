"""Seeded generator for PLAID-shaped synthetic indexes and queries.

What it draws (everything is a stand-in for the paper's MS MARCO / Wikipedia /
LoTTE workloads, whose passages and ColBERTv2 embeddings are not available):

* centroids: C x 128 i.i.d. N(0,1) rows, L2-normalised, fp32;
* passage lengths: uniform integers or a rounded, clipped normal;
* per-token centroid id: Zipf(s) over ids 0..C-1, P(c) ~ (c+1)^-s;
* per-token embedding x = normalize(centroid + sigma_d * n), n ~ N(0, I_128);
* stored form of a token: int32 centroid id + the residual x - centroid
  quantised per dimension into 2^nbits buckets (cut-offs / weights are pooled
  quantiles of a fixed sample of residuals), bit-packed MSB-first, 16*nbits
  bytes per token (Section 3.1 of the paper: 4-byte id + 16 or 32 bytes);
* inverted lists: centroid id -> ascending unique passage ids (Section 4.1);
* queries: 32 tokens, each normalize(x_t + sigma_q * n) for a random token t.

``noise="literal"`` scales every coordinate of n by sigma (the wording of the
configuration text); ``noise="calibrated"`` scales the whole noise *vector* to
expected norm sigma (per-coordinate sigma / sqrt(128)), which gives the
token-to-centroid cosines (~0.99) and the small tail of high centroid scores
that Section 3.4 / Figure 5 of the paper describe.

The generator runs on any torch device; the random streams are per
(seed, chunk) so every chunk can be regenerated independently.  CPU and GPU
streams differ, so a workload is identified by (config, noise, device type).
"""
from __future__ import annotations

import dataclasses
import math
import struct
from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np
import torch

DIM = 128
QLEN = 32
CHUNK_TOKENS = 1 << 18          # tokens generated per RNG stream
QUANTILE_SAMPLE_TOKENS = 1 << 20  # residuals of the first min(N, 2^20) tokens define the buckets


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    C: int
    P: int
    length: Tuple            # ("uniform", lo, hi) | ("tnormal", mean, sd, lo, hi) | ("fixed", [l0, l1, ...])
    nbits: int
    nq: int
    nprobe: int
    t_cs: float
    ndocs: int
    k: int
    index_seed: int
    query_seed: int
    sigma_d: float = 0.15
    sigma_q: float = 0.2
    zipf_s: float = 1.1

    def replace(self, **kw) -> "WorkloadConfig":
        return dataclasses.replace(self, **kw)


# The five benchmark configurations (search triples are Table 2 of the paper).
CONFIGS: Dict[str, WorkloadConfig] = {
    "cfg1": WorkloadConfig("cfg1", C=1024, P=10_000, length=("uniform", 20, 60), nbits=2, nq=16,
                           nprobe=1, t_cs=0.5, ndocs=256, k=10, index_seed=1001, query_seed=2001),
    "cfg2": WorkloadConfig("cfg2", C=16_384, P=200_000, length=("uniform", 30, 90), nbits=2, nq=256,
                           nprobe=1, t_cs=0.5, ndocs=256, k=10, index_seed=1002, query_seed=2002),
    "cfg3": WorkloadConfig("cfg3", C=65_536, P=400_000, length=("uniform", 30, 100), nbits=2, nq=512,
                           nprobe=2, t_cs=0.45, ndocs=1024, k=100, index_seed=1003, query_seed=2003),
    "cfg4": WorkloadConfig("cfg4", C=262_144, P=8_800_000, length=("tnormal", 68.0, 20.0, 8, 180), nbits=2,
                           nq=1000, nprobe=4, t_cs=0.4, ndocs=4096, k=1000, index_seed=1004, query_seed=2004),
    "cfg5": WorkloadConfig("cfg5", C=262_144, P=20_000_000, length=("tnormal", 70.0, 20.0, 8, 180), nbits=1,
                           nq=1000, nprobe=4, t_cs=0.4, ndocs=4096, k=100, index_seed=1005, query_seed=2005),
}


def get_config(name: str) -> WorkloadConfig:
    return CONFIGS[name]


def tiny_config(C: int, P: int, lo: int, hi: int, nbits: int = 2, nq: int = 4, seed: int = 7,
                nprobe: int = 1, t_cs: float = 0.5, ndocs: int = 16, k: int = 4, **kw) -> WorkloadConfig:
    """A small configuration of the same generator for property tests."""
    return WorkloadConfig(f"tiny_C{C}_P{P}_b{nbits}_s{seed}", C=C, P=P, length=("uniform", lo, hi), nbits=nbits,
                          nq=nq, nprobe=nprobe, t_cs=t_cs, ndocs=ndocs, k=k,
                          index_seed=10_000 + seed, query_seed=20_000 + seed, **kw)


@dataclass
class Workload:
    cfg: WorkloadConfig
    noise: str
    centroids: torch.Tensor        # [C,128] f32
    doc_offsets: torch.Tensor      # [P+1] i64
    codes: torch.Tensor            # [N] i32
    residuals: torch.Tensor        # [N,16*nbits] u8
    bucket_cutoffs: torch.Tensor   # [2^nbits-1] f32 (index-time only)
    bucket_weights: torch.Tensor   # [2^nbits] f32
    ivf_offsets: torch.Tensor      # [C+1] i64
    ivf_pids: torch.Tensor         # [ivf_offsets[C]] i32
    queries: torch.Tensor          # [nq,32,128] f32
    query_src_tokens: torch.Tensor  # [nq,32] i64: token index each query token was derived from
    sample_embeddings: Optional[torch.Tensor] = None  # [n_keep,128] f32 uncompressed x of the first tokens (tests)

    @property
    def N(self) -> int:
        return int(self.codes.shape[0])

    def numpy(self) -> Dict[str, np.ndarray]:
        """Host copies of the index buffers and queries, C-contiguous."""
        out = {}
        for f in ("centroids", "doc_offsets", "codes", "residuals", "bucket_cutoffs", "bucket_weights",
                  "ivf_offsets", "ivf_pids", "queries"):
            out[f] = np.ascontiguousarray(getattr(self, f).detach().cpu().numpy())
        return out

    def to(self, device) -> "Workload":
        kw = {}
        for f in dataclasses.fields(self):
            v = getattr(self, f.name)
            kw[f.name] = v.to(device) if isinstance(v, torch.Tensor) else v
        return Workload(**kw)


def index_nbytes(N: int, nbits: int) -> int:
    """Bytes of codes + packed residuals: N * (4 + 16*nbits) (Section 3.1)."""
    return N * (4 + 16 * nbits)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed & 0x7FFF_FFFF_FFFF_FFFF)
    return g


def _draw_lengths(cfg: WorkloadConfig, device) -> torch.Tensor:
    g = _gen(device, cfg.index_seed * 7_919 + 11)
    kind = cfg.length[0]
    if kind == "uniform":
        _, lo, hi = cfg.length
        return torch.randint(lo, hi + 1, (cfg.P,), generator=g, device=device, dtype=torch.int64)
    if kind == "tnormal":
        _, mean, sd, lo, hi = cfg.length
        z = torch.randn(cfg.P, generator=g, device=device, dtype=torch.float32)
        return torch.clamp(torch.round(z * sd + mean), lo, hi).to(torch.int64)
    if kind == "fixed":
        lens = torch.tensor(list(cfg.length[1]), dtype=torch.int64, device=device)
        assert lens.numel() == cfg.P
        return lens
    raise ValueError(kind)


def _order_statistics(values: torch.Tensor, qs) -> np.ndarray:
    """Linear-interpolated quantiles (numpy.quantile's default rule), fp64 arithmetic on exact order statistics."""
    n = values.numel()
    pos = [q * (n - 1) for q in qs]
    lo = [int(math.floor(p)) for p in pos]
    hi = [min(l + 1, n - 1) for l in lo]
    need = sorted(set(lo + hi))
    if values.is_cuda:
        s, _ = torch.sort(values.reshape(-1))
        got = s[torch.tensor(need, device=values.device)].double().cpu().numpy()
    else:
        a = np.partition(values.reshape(-1).numpy(), need)
        got = a[need].astype(np.float64)
    at = dict(zip(need, got))
    return np.array([at[l] + (at[h] - at[l]) * (p - l) for p, l, h in zip(pos, lo, hi)], dtype=np.float64)


def _chunk_tokens(cfg: WorkloadConfig, noise: str, centroids, cdf, g_idx: int, n: int, device):
    """Codes, uncompressed embeddings and residuals of chunk ``g_idx`` (its first ``n`` tokens)."""
    g = _gen(device, cfg.index_seed * 1_000_003 + 1 + g_idx)
    u = torch.rand(n, generator=g, device=device, dtype=torch.float64)
    codes = torch.searchsorted(cdf, u).clamp_(max=cfg.C - 1)
    sig = cfg.sigma_d if noise == "literal" else cfg.sigma_d / math.sqrt(DIM)
    x = torch.randn(n, DIM, generator=g, device=device, dtype=torch.float32)
    x.mul_(sig)
    cen = centroids[codes]
    x.add_(cen)
    x = torch.nn.functional.normalize(x, dim=1)
    r = x - cen
    return codes, x, r


def _pack(idx: torch.Tensor, nbits: int) -> torch.Tensor:
    """Bit-pack bucket indices MSB-first: dimension order is preserved inside each byte."""
    n = idx.shape[0]
    per = 8 // nbits
    v = idx.reshape(n, DIM // per, per).to(torch.int32)
    shifts = torch.arange(per - 1, -1, -1, device=idx.device, dtype=torch.int32) * nbits
    return (v << shifts).sum(dim=2).to(torch.uint8)


def make_workload(cfg: WorkloadConfig, device="cpu", noise: str = "literal", keep_embeddings: int = 0) -> Workload:
    assert noise in ("literal", "calibrated")
    assert cfg.nbits in (1, 2)
    device = torch.device(device)
    g0 = _gen(device, cfg.index_seed)
    centroids = torch.nn.functional.normalize(
        torch.randn(cfg.C, DIM, generator=g0, device=device, dtype=torch.float32), dim=1).contiguous()
    lengths = _draw_lengths(cfg, device)
    doc_offsets = torch.zeros(cfg.P + 1, dtype=torch.int64, device=device)
    doc_offsets[1:] = torch.cumsum(lengths, 0)
    N = int(doc_offsets[-1].item())

    pz = torch.arange(1, cfg.C + 1, device=device, dtype=torch.float64).pow_(-cfg.zipf_s)
    cdf = torch.cumsum(pz, 0)
    cdf /= cdf[-1].clone()

    nchunks = (N + CHUNK_TOKENS - 1) // CHUNK_TOKENS

    def chunk_len(gi):
        return min(CHUNK_TOKENS, N - gi * CHUNK_TOKENS)

    # pass A: bucket cut-offs and weights from the residuals of the first tokens
    n_sample = min(N, QUANTILE_SAMPLE_TOKENS)
    parts = []
    gi = 0
    while gi * CHUNK_TOKENS < n_sample:
        n = min(chunk_len(gi), n_sample - gi * CHUNK_TOKENS)
        # the whole chunk is drawn so the stream matches pass B, then truncated
        _, _, r = _chunk_tokens(cfg, noise, centroids, cdf, gi, chunk_len(gi), device)
        parts.append(r[:n].reshape(-1))
        gi += 1
    sample = torch.cat(parts) if len(parts) > 1 else parts[0]
    if cfg.nbits == 2:
        qv = _order_statistics(sample, [0.25, 0.5, 0.75, 0.125, 0.375, 0.625, 0.875])
        cut, wts = qv[:3], qv[3:]
    else:
        qv = _order_statistics(sample, [0.5, 0.25, 0.75])
        cut, wts = qv[:1], qv[1:]
    del sample, parts
    bucket_cutoffs = torch.tensor(cut, dtype=torch.float64).to(torch.float32).to(device)
    bucket_weights = torch.tensor(wts, dtype=torch.float64).to(torch.float32).to(device)

    # query source tokens
    gq = _gen(device, cfg.query_seed)
    qsrc = torch.randint(0, N, (cfg.nq * QLEN,), generator=gq, device=device, dtype=torch.int64)
    qx = torch.empty(cfg.nq * QLEN, DIM, device=device, dtype=torch.float32)

    # pass B: quantise, pack, collect inverted-list pairs
    codes = torch.empty(N, dtype=torch.int32, device=device)
    residuals = torch.empty(N, 16 * cfg.nbits, dtype=torch.uint8, device=device)
    pair_parts = []
    kept = []
    for gi in range(nchunks):
        n = chunk_len(gi)
        t0 = gi * CHUNK_TOKENS
        c, x, r = _chunk_tokens(cfg, noise, centroids, cdf, gi, n, device)
        idx = torch.bucketize(r, bucket_cutoffs, right=False)      # = #{cutoffs < r}
        codes[t0:t0 + n] = c.to(torch.int32)
        residuals[t0:t0 + n] = _pack(idx, cfg.nbits)
        tok = torch.arange(t0, t0 + n, device=device, dtype=torch.int64)
        pid = torch.searchsorted(doc_offsets, tok, right=True) - 1
        pair_parts.append(torch.unique(c * cfg.P + pid))
        sel = ((qsrc >= t0) & (qsrc < t0 + n)).nonzero().squeeze(1)
        if sel.numel():
            qx[sel] = x[qsrc[sel] - t0]
        if keep_embeddings > t0:
            kept.append(x[: max(0, min(n, keep_embeddings - t0))].clone())
        del c, x, r, idx, tok, pid
    pairs = torch.unique(torch.cat(pair_parts)) if len(pair_parts) > 1 else pair_parts[0]
    del pair_parts
    ivf_pids = (pairs % cfg.P).to(torch.int32)
    counts = torch.bincount(pairs // cfg.P, minlength=cfg.C)
    del pairs
    ivf_offsets = torch.zeros(cfg.C + 1, dtype=torch.int64, device=device)
    ivf_offsets[1:] = torch.cumsum(counts, 0)

    sq = cfg.sigma_q if noise == "literal" else cfg.sigma_q / math.sqrt(DIM)
    qn = torch.randn(cfg.nq * QLEN, DIM, generator=gq, device=device, dtype=torch.float32) * sq
    queries = torch.nn.functional.normalize(qx + qn, dim=1).reshape(cfg.nq, QLEN, DIM).contiguous()

    return Workload(cfg=cfg, noise=noise, centroids=centroids, doc_offsets=doc_offsets, codes=codes,
                    residuals=residuals, bucket_cutoffs=bucket_cutoffs, bucket_weights=bucket_weights,
                    ivf_offsets=ivf_offsets, ivf_pids=ivf_pids, queries=queries,
                    query_src_tokens=qsrc.reshape(cfg.nq, QLEN),
                    sample_embeddings=(torch.cat(kept) if kept else None))


# ---------------------------------------------------------------------------------------------
# Flat index file (read by plaid_index_load).  Layout, little-endian:
#   bytes 0..7    magic "PLAIDIX1"
#   int32 dim, int32 nbits, int64 C, int64 P, int64 N, int64 ivf_len, zero padding to 64 bytes
#   then the sections centroids f32[C*dim], doc_offsets i64[P+1], codes i32[N],
#   residuals u8[N*16*nbits], bucket_weights f32[2^nbits], ivf_offsets i64[C+1],
#   ivf_pids i32[ivf_len]; every section starts at a multiple of 64 bytes.
# ---------------------------------------------------------------------------------------------
INDEX_MAGIC = b"PLAIDIX1"


def save_index_file(path: str, arrays: Dict[str, np.ndarray], nbits: int) -> None:
    C, dim = arrays["centroids"].shape
    P = arrays["doc_offsets"].shape[0] - 1
    N = arrays["codes"].shape[0]
    ivf_len = arrays["ivf_pids"].shape[0]
    hdr = INDEX_MAGIC + struct.pack("<iiqqqq", dim, nbits, C, P, N, ivf_len)
    hdr += b"\0" * (64 - len(hdr))
    order = [("centroids", np.float32), ("doc_offsets", np.int64), ("codes", np.int32), ("residuals", np.uint8),
             ("bucket_weights", np.float32), ("ivf_offsets", np.int64), ("ivf_pids", np.int32)]
    with open(path, "wb") as f:
        f.write(hdr)
        for name, dt in order:
            a = np.ascontiguousarray(arrays[name], dtype=dt)
            f.write(a.tobytes())
            pad = (-a.nbytes) % 64
            if pad:
                f.write(b"\0" * pad)
