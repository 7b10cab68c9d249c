"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs.

Runs only on a machine with an MI355X (`-m gpu`).  Sizes: the tiny configuration with all its
queries stage by stage, random small indexes sweeping the degenerate cases, and the codec alone.
"""
import contextlib
import os

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from synth import get_config, make_workload, tiny_config

import parity_util as pu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pl():
    import paper_2205_09707_amd as pl_
    pl_.load_library()   # fails loudly when libplaid.so has not been built
    assert torch.cuda.is_available(), "these tests need the GPU"
    return pl_


@contextlib.contextmanager
def _kernel_forms(form=None, stage2=None):
    """Index creation reads PLAID_SCQ_FORM ('split16' / 'matrix' / 'vector': the S_cq kernels) and PLAID_STAGE2_FORM
    ('inverted' / 'stream': the two ways to candidates and pruned scores); None leaves the library's own choice."""
    wanted = {"PLAID_SCQ_FORM": form, "PLAID_STAGE2_FORM": stage2}
    old = {k: os.environ.get(k) for k in wanted}
    for k, v in wanted.items():
        if v is None:
            os.environ.pop(k, None)
        else:
            os.environ[k] = v
    try:
        yield
    finally:
        for k, v in old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v


def _check_workload(pl, w, params_list, want=None, queries=None, copy=False, form=None, stage2=None, max_chunk=None):
    ix = pu.oracle_index(w)
    with _kernel_forms(form, stage2):
        gidx = pl.plaid_index_from_view(pu.device_arrays(w), w.cfg.nbits, device=0, copy=copy)
    if max_chunk is not None:
        pl.plaid_set_max_chunk(gidx, max_chunk)
    if form is not None:
        assert pl.plaid_get_score_kernel(gidx) == {"vector": 0, "matrix": 1, "split16": 2}[form]
    if stage2 is not None:
        assert pl.plaid_get_stage2_kernel(gidx) == {"stream": 0, "inverted": 1, "inverted11": 1, "inverted13": 2}[stage2]
    Qdev = w.queries.to("cuda:0")
    Qh = w.queries.numpy()
    nq = Qh.shape[0]
    identical = 0
    total = 0
    try:
        for params in params_list:
            print(f"[parity] {w.cfg.name} {w.noise} params={params}", flush=True)
            out = pu.run_gpu_debug(pl, gidx, Qdev, params, want=want)
            for q in (range(nq) if queries is None else queries):
                same = pu.compare_query(ix, Qh[q], params, pu.slice_query(out, q), ctx=f"{w.cfg.name}/{w.noise} {params} q{q}",
                                        approx=pu.is_approx(pl, gidx, params))
                identical += bool(same)
                total += 1
    finally:
        pl.plaid_index_free(gidx)
    print(f"[parity] largest deviations so far (split-fp16 score kernel): {pu.MEASURED}", flush=True)
    return identical, total


@pytest.mark.parametrize("form,stage2", [("split16", "inverted"), ("split16", "stream"), ("split16", "inverted13"),
                                         ("matrix", "inverted"), ("vector", "stream"), ("matrix", "stream")])
@pytest.mark.parametrize("noise", ["literal", "calibrated"])
def test_cfg1_all_stages(pl, noise, form, stage2):
    cfg = get_config("cfg1")
    w = make_workload(cfg, device="cpu", noise=noise)
    same, total = _check_workload(pl, w, [(cfg.nprobe, cfg.t_cs, cfg.ndocs, cfg.k)], form=form, stage2=stage2)
    # (every difference has already been checked to lie inside a tie of oracle scores within TOL: compare_query)
    print(f"cfg1/{noise}: {same}/{total} queries with id lists identical to the oracle's")


@pytest.mark.parametrize("form,stage2", [("split16", "inverted"), ("split16", "stream"), ("matrix", "inverted"),
                                         ("vector", "stream")])
def test_cfg1_other_operating_points(pl, form, stage2):
    """Table 2's other two triples, and thresholds low enough that many centroids survive (more than the slot sets hold:
    both forms then score candidates from their token codes)."""
    cfg = get_config("cfg1")
    w = make_workload(cfg, device="cpu", noise="calibrated")
    _check_workload(pl, w, [(2, 0.45, 1024, 100), (4, 0.4, 4096, 1000), (3, 0.2, 300, 40), (1, -np.inf, 64, 16),
                            (6, 0.5, 200, 20), (8, 0.45, 512, 50), (12, 0.5, 128, 10)], form=form, stage2=stage2)


@pytest.mark.parametrize("max_chunk", [1, 3, 5])
def test_cfg1_in_ragged_chunks(pl, max_chunk):
    """A batch larger than the per-launch limit is processed in chunks (the last one shorter): every chunk reuses the
    same workspace, so anything a kernel leaves behind in it would show up in the next chunk's results."""
    cfg = get_config("cfg1")
    w = make_workload(cfg, device="cpu", noise="calibrated")
    _check_workload(pl, w, [(cfg.nprobe, cfg.t_cs, cfg.ndocs, cfg.k), (2, 0.45, 1024, 100)], max_chunk=max_chunk)


def test_default_kernel_forms(pl):
    """An index created without an override scores with the split-fp16 matrix kernel; asked for the double-precision
    matrix kernel it gets it, because on gfx950 the device check of that instruction passes."""
    cfg = tiny_config(C=64, P=50, lo=3, hi=9, nbits=2, nq=1, seed=5)
    w = make_workload(cfg, device="cpu", noise="calibrated")
    with _kernel_forms(None, None):
        gidx = pl.plaid_index_from_view(pu.device_arrays(w), w.cfg.nbits, device=0, copy=True)
    try:
        assert pl.plaid_get_score_kernel(gidx) == 2
        assert pl.plaid_get_stage2_kernel(gidx) == 1   # a small index: the range table is tiny at 2048 passages per column
    finally:
        pl.plaid_index_free(gidx)
    with _kernel_forms("matrix", None):
        gidx = pl.plaid_index_from_view(pu.device_arrays(w), w.cfg.nbits, device=0, copy=True)
    try:
        assert pl.plaid_get_score_kernel(gidx) == 1
    finally:
        pl.plaid_index_free(gidx)


def test_score_kernel_clock_diagnostic(pl):
    """With stage timing on, the split-fp16 score kernel's workgroups add up how far the shader-clock counter and the
    100 MHz timer moved while they ran: the ratio is a clock between a few hundred MHz and the chip's 2.4 GHz.  Nothing
    is recorded with timing off, nor by the double-precision kernels."""
    w = make_workload(tiny_config(C=700, P=300, lo=2, hi=20, nbits=2, nq=6, seed=73), device="cpu", noise="calibrated")
    Qdev = w.queries.to("cuda:0")
    for form, measured in (("split16", True), ("matrix", False)):
        with _kernel_forms(form, None):
            gidx = pl.plaid_index_from_view(pu.device_arrays(w), w.cfg.nbits, device=0, copy=True)
        try:
            assert pl.plaid_get_score_kernel_clocks(gidx) == (0, 0)
            ids0, sc0 = pl.plaid_search(gidx, Qdev, 2, 0.45, 64, 10)
            assert pl.plaid_get_score_kernel_clocks(gidx) == (0, 0)
            pl.plaid_set_stage_timing(gidx, True)
            ids1, sc1 = pl.plaid_search(gidx, Qdev, 2, 0.45, 64, 10)
            core, fixed = pl.plaid_get_score_kernel_clocks(gidx)
            pl.plaid_set_stage_timing(gidx, False)
            assert torch.equal(ids0, ids1) and torch.equal(sc0, sc1)
            if measured:
                assert fixed > 0 and 200.0 < 100.0 * core / fixed < 2600.0, (core, fixed)
            else:
                assert (core, fixed) == (0, 0)
        finally:
            pl.plaid_index_free(gidx)


def test_large_centroid_components_get_a_double_precision_score_kernel(pl):
    """The split-fp16 kernel scales the centroids' leading terms by 2^11 in fp16: a table with a component of 32 or more
    is given the double-precision matrix kernel instead (and searches like the oracle); insisting on the split form
    for such a table is an error."""
    w = make_workload(tiny_config(C=64, P=300, lo=2, hi=20, nbits=2, nq=3, seed=72), device="cpu", noise="calibrated")
    arrays = pu.device_arrays(w)
    # one more centroid, in no passage (so the final scores keep their usual size): a unit vector times 400
    big = 400.0 * arrays["centroids"][5:6]
    arrays["centroids"] = torch.cat([arrays["centroids"], big]).contiguous()
    arrays["ivf_offsets"] = torch.cat([arrays["ivf_offsets"], arrays["ivf_offsets"][-1:]]).contiguous()
    assert float(arrays["centroids"].abs().max()) > 32.0
    with _kernel_forms(None, None):
        gidx = pl.plaid_index_from_view(arrays, w.cfg.nbits, device=0, copy=True)
    try:
        assert pl.plaid_get_score_kernel(gidx) == 1
        ix = orc.Index({k: v.cpu().numpy() for k, v in arrays.items()}, w.cfg.nbits)
        params = (2, 0.45, 64, 10)
        out = pu.run_gpu_debug(pl, gidx, w.queries.to("cuda:0"), params)
        for q in range(3):
            pu.compare_query(ix, w.queries[q].numpy(), params, pu.slice_query(out, q), ctx=f"large centroid q{q}", approx=False)
    finally:
        pl.plaid_index_free(gidx)
    with _kernel_forms("split16", None):
        with pytest.raises(pl.PlaidError):
            pl.plaid_index_from_view(arrays, w.cfg.nbits, device=0, copy=True)


def test_pipeline_equals_exhaustive_when_nothing_is_filtered(pl):
    """nprobe = C, t_cs = -inf, ndocs >= 4P: every passage reaches stage 4, so the library's result must be the
    exhaustive MaxSim ranking (ndocs = 4P because stage 3 keeps ndocs/4)."""
    w = make_workload(tiny_config(C=48, P=150, lo=1, hi=70, nbits=2, nq=5, seed=11), noise="calibrated")
    ix = pu.oracle_index(w)
    gidx = pl.plaid_index_from_view(pu.device_arrays(w), 2, device=0, copy=True)
    try:
        k = 20
        ids, sc = pl.plaid_search(gidx, w.queries.to("cuda:0"), 48, -np.inf, 4 * 150, k)
        ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
        allp = np.arange(150, dtype=np.int32)
        for q in range(5):
            Q = w.queries[q].numpy()
            e_ids, e_sc = orc.exhaustive(ix, Q, k)
            s_all = orc.maxsim(ix, Q, allp)
            same = pu.assert_final_matches(ids[q], sc[q], allp, s_all, k, ctx=f"exhaustive q{q}")
            if same:
                assert np.array_equal(ids[q], e_ids)
            assert np.max(np.abs(sc[q] - e_sc)) <= pu.TOL
    finally:
        pl.plaid_index_free(gidx)


SWEEP = [
    # C, P, lo, hi, nbits, seed, noise, nq, S_cq kernel, stage-2 form (None = the library's choice)
    (16, 50, 1, 9, 2, 1, "calibrated", 4, None, None),
    (16, 50, 1, 9, 1, 2, "literal", 4, None, "stream"),
    (5, 7, 1, 3, 2, 3, "calibrated", 3, None, None),          # an odd number of queries: the last column block is half empty
    (33, 200, 1, 130, 2, 4, "calibrated", 4, None, "stream"),  # passages longer than two waves of tokens
    (33, 200, 1, 130, 2, 4, "calibrated", 4, None, "inverted"),
    (70, 321, 0, 40, 1, 5, "calibrated", 4, "vector", None),  # empty passages, ragged sizes
    (1, 9, 1, 5, 2, 6, "literal", 4, None, None),             # a single centroid
    (300, 1, 5, 5, 2, 7, "calibrated", 5, None, None),        # a single passage; three row blocks, the last one ragged
    (129, 40, 2, 12, 2, 8, "calibrated", 1, "matrix", "stream"),  # one row past a row block, one query
    (40, 5000, 1, 6, 2, 9, "calibrated", 3, None, "inverted"),    # three passage ranges, the last one ragged
    (40, 5000, 1, 6, 2, 9, "calibrated", 3, None, "stream"),
    # 8192 passages per workgroup (the form large indexes take): one ragged range, then three ranges with the last ragged
    (40, 5000, 1, 6, 2, 9, "calibrated", 3, None, "inverted13"),
    (33, 20000, 1, 5, 2, 10, "calibrated", 35, None, "inverted13"),
    # more than 16 queries: the short-list selections sort in LDS (one workgroup per list) instead of counting ranks;
    # 900 and 3000 passages put the lists into the 512- and 1024-thread forms of that sort
    (33, 200, 1, 30, 2, 11, "calibrated", 20, None, None),
    (24, 900, 1, 4, 2, 12, "calibrated", 17, None, None),
    (24, 3000, 1, 4, 2, 13, "literal", 17, None, "stream"),
    # 32 queries or more: queries without a surviving centroid (t_cs = +inf in the parameter list) take the kernel that
    # covers 2^19 passages per workgroup; 16 centroids over 300 passages make every inverted list long enough for a
    # bitmap, 200 centroids over 3000 short passages none
    (16, 300, 1, 9, 2, 14, "calibrated", 33, None, "inverted"),
    (200, 3000, 1, 4, 2, 15, "literal", 40, None, "inverted"),
]


@pytest.mark.parametrize("C,P,lo,hi,nbits,seed,noise,nq,form,stage2", SWEEP)
def test_small_index_sweep(pl, C, P, lo, hi, nbits, seed, noise, nq, form, stage2):
    w = make_workload(tiny_config(C=C, P=P, lo=lo, hi=hi, nbits=nbits, nq=nq, seed=seed), noise=noise)
    S = orc.scq(w.centroids.numpy(), w.queries[0].numpy())
    qs = np.quantile(S.max(axis=1), [0.3, 0.9]).tolist()
    params = []
    for nprobe in sorted({1, min(2, C), min(9, C), C}):
        for t_cs in (-np.inf, qs[0], qs[1], np.inf):
            for ndocs, k in ((1, 1), (4, 3), (17, 5), (4 * P + 3, P + 2)):
                params.append((nprobe, float(t_cs), ndocs, k))
    # a deterministic subset keeps the run short while every value of every parameter appears
    params = params[:: 3] + params[-2:]
    # launches of many queries run all of them; the oracle, on the CPU, checks every third one and the last
    queries = None if nq <= 12 else sorted(set(range(0, nq, 3)) | {nq - 1})
    _check_workload(pl, w, params, queries=queries, form=form, stage2=stage2)


RARE = [
    # name, config, parameter list, stage-2 forms
    # two centroids: thousands of passages share each pruned score, so the stage-2 cut falls inside a tie group far
    # longer than one workgroup can sort (digit filter on the passage-id bits), and ndocs > 8192 sends stage 3's
    # selection through the multi-level radix path
    ("tie_groups", dict(C=2, P=40000, lo=1, hi=3, nbits=2, nq=2, seed=31), [(2, -np.inf, 9000, 10), (1, 0.0, 300, 5)],
     ("inverted", "stream", "inverted13")),
    # passages longer than the streaming kernel's staging buffer (2272 tokens) and than many 32-token steps of stage 4
    ("long_passages", dict(C=50, P=6, lo=2300, hi=2400, nbits=1, nq=2, seed=32), [(2, 0.1, 4, 2), (50, -np.inf, 6, 6)],
     ("stream", "inverted", "inverted13")),
    # ndocs/4 and k beyond 8192: radix selection of the stage-3 survivors and of the final ranking, sorted output
    # through the global bitonic network
    ("big_lists", dict(C=8, P=40000, lo=1, hi=2, nbits=2, nq=1, seed=33), [(8, -np.inf, 40000, 12000)], ("inverted",)),
]


@pytest.mark.parametrize("name,cfgkw,params,forms", RARE, ids=[r[0] for r in RARE])
def test_rare_paths(pl, name, cfgkw, params, forms):
    w = make_workload(tiny_config(**cfgkw), noise="calibrated")
    for stage2 in forms:
        _check_workload(pl, w, params, stage2=stage2)


def test_two_long_tie_groups_in_one_score_bin(pl):
    """Two nearly equal centroids, each the only one of some 240 000 passages: two pruned scores that differ in their
    last bits, so both tie groups land in one bin of the stage-2 histogram and the ndocs cut falls inside the second.
    In a launch of nine queries on an index of more than 2^19 passages the boundary list then passes two digit filters
    (score bits, then passage-id bits)."""
    rng = np.random.default_rng(71)
    P, nq = 600000, 9
    c0 = rng.standard_normal(128)
    c0 /= np.linalg.norm(c0)
    c1 = c0 + 5e-5 * rng.standard_normal(128)
    c1 /= np.linalg.norm(c1)
    c2 = rng.standard_normal(128)
    c2 /= np.linalg.norm(c2)
    centroids = np.stack([c0, c1, c2]).astype(np.float32)
    kind = rng.integers(0, 10, size=P)               # 4 in 10 hold centroid 0 only, 4 in 10 centroid 1 only, the rest more
    lengths = np.where(kind < 8, 1, 2)
    doc_offsets = np.zeros(P + 1, dtype=np.int64)
    np.cumsum(lengths, out=doc_offsets[1:])
    N = int(doc_offsets[-1])
    codes = np.zeros(N, dtype=np.int32)
    first = doc_offsets[:-1]
    codes[first] = np.where(kind < 4, 0, np.where(kind < 8, 1, 2))
    two = np.nonzero(lengths == 2)[0]
    codes[first[two] + 1] = rng.integers(0, 2, size=len(two))
    residuals = rng.integers(0, 256, size=(N, 32), dtype=np.uint8)
    weights = np.array([-0.03, -0.01, 0.01, 0.03], dtype=np.float32)
    ivf_offsets, ivf_pids = orc.build_ivf(codes, doc_offsets, 3)
    arrays = dict(centroids=centroids, doc_offsets=doc_offsets, codes=codes, residuals=residuals, bucket_weights=weights,
                  ivf_offsets=ivf_offsets, ivf_pids=ivf_pids)
    Q = c0[None, None, :] + 0.3 * rng.standard_normal((nq, 32, 128))
    Q = (Q / np.linalg.norm(Q, axis=2, keepdims=True)).astype(np.float32)
    ix = orc.Index(arrays, 2)
    gidx = pl.plaid_index_from_view({k: torch.from_numpy(v).to("cuda:0") for k, v in arrays.items()}, 2, device=0, copy=True)
    try:
        Qdev = torch.from_numpy(Q).to("cuda:0")
        for params in [(1, -np.inf, 300000, 10), (3, 0.3, 400000, 5)]:
            out = pu.run_gpu_debug(pl, gidx, Qdev, params)
            for q in (0, 4, 8):
                pu.compare_query(ix, Q[q], params, pu.slice_query(out, q), ctx=f"tie bins {params} q{q}",
                                 approx=pu.is_approx(pl, gidx, params))
    finally:
        pl.plaid_index_free(gidx)


@pytest.mark.parametrize("form", ["split16", "matrix", "vector"])
def test_all_zero_query_token(pl, form):
    """A query token of zeros scores 0 against every centroid: all tiles of the score kernel tie on their column
    maximum (more tiles than the probe kernel lists per token), and the probes are the lowest centroid ids."""
    w = make_workload(tiny_config(C=2200, P=300, lo=2, hi=12, nbits=2, nq=3, seed=41), noise="calibrated")
    w.queries[:, 0, :] = 0.0
    w.queries[1, 7, :] = 0.0
    _check_workload(pl, w, [(1, 0.3, 40, 5), (2, 0.3, 40, 5), (4, -np.inf, 64, 8), (7, 0.2, 30, 4)], form=form)


def test_codec_bit_exact(pl):
    """Unpacked bucket indices and reconstructed vectors (Section 4.5) are bit-identical to the oracle's."""
    for nbits, seed in ((2, 21), (1, 22)):
        w = make_workload(tiny_config(C=64, P=300, lo=0, hi=50, nbits=nbits, nq=1, seed=seed), noise="calibrated")
        ix = pu.oracle_index(w)
        gidx = pl.plaid_index_from_view(pu.device_arrays(w), nbits, device=0, copy=False)
        try:
            rng = np.random.default_rng(seed)
            pids = np.concatenate([rng.permutation(300)[:120], [0, 299, 299]]).astype(np.int32)
            lens = (w.doc_offsets[1:] - w.doc_offsets[:-1]).numpy()
            total = int(lens[pids].sum())
            offs, vec, ind = pl.plaid_decompress_passages(gidx, torch.from_numpy(pids).to("cuda:0"), total)
            offs, vec, ind = offs.cpu().numpy(), vec.cpu().numpy(), ind.cpu().numpy()
            assert offs[-1] == total
            do = w.doc_offsets.numpy()
            for a, p in enumerate(pids):
                D, idx = orc.decompress(ix, int(do[p]), int(do[p + 1]))
                assert np.array_equal(ind[offs[a]:offs[a + 1]], idx), f"bucket indices of passage {p}"
                assert np.array_equal(pu.bits(vec[offs[a]:offs[a + 1]]), pu.bits(D)), f"vectors of passage {p}"
            with pytest.raises(pl.PlaidError):
                pl.plaid_decompress_passages(gidx, torch.from_numpy(pids).to("cuda:0"), total - 1)
        finally:
            pl.plaid_index_free(gidx)


def test_argument_errors(pl):
    w = make_workload(tiny_config(C=8, P=10, lo=1, hi=4, nbits=2, nq=2, seed=9), noise="literal")
    gidx = pl.plaid_index_from_view(pu.device_arrays(w), 2, device=0, copy=True)
    Q = w.queries.to("cuda:0")
    try:
        for bad in ((0, 0.5, 4, 2), (9, 0.5, 4, 2), (1, 0.5, 0, 2), (1, 0.5, 4, 0), (1, float("nan"), 4, 2)):
            with pytest.raises(pl.PlaidError) as e:
                pl.plaid_search(gidx, Q, *bad)
            assert e.value.status == pl.plaid.PLAID_EINVAL
        # the handle still works after rejected calls
        ids, sc = pl.plaid_search(gidx, Q, 1, 0.5, 4, 2)
        torch.cuda.synchronize()
        assert ids.shape == (2, 2)
    finally:
        pl.plaid_index_free(gidx)


def test_device_arrays_are_validated(pl):
    """An index handed over in device memory gets the structural checks host arrays get: a code, a passage id or an
    offset that a search kernel would follow out of bounds is PLAID_EINVAL at index creation, with or without a copy."""
    w = make_workload(tiny_config(C=20, P=300, lo=1, hi=9, nbits=2, nq=1, seed=17), noise="calibrated")

    def broken(name, fn):
        arrs = pu.device_arrays(w)
        t = arrs[name].clone()
        fn(t)
        arrs[name] = t
        return arrs

    C, P, N = 20, 300, int(w.N)
    head = int(torch.argmax(w.ivf_offsets[1:] - w.ivf_offsets[:-1]))    # a list with at least two entries
    e0 = int(w.ivf_offsets[head])

    def swap(t):
        t[e0], t[e0 + 1] = t[e0 + 1].clone(), t[e0].clone()

    def dup(t):
        t[e0 + 1] = t[e0]
    cases = [("codes", lambda t: t.__setitem__(N // 2, C)), ("codes", lambda t: t.__setitem__(0, -1)),
             ("ivf_pids", lambda t: t.__setitem__(3, P)), ("ivf_pids", lambda t: t.__setitem__(5, -2)),
             ("ivf_pids", swap), ("ivf_pids", dup),
             ("doc_offsets", lambda t: t.__setitem__(7, int(t[8]) + 1)), ("doc_offsets", lambda t: t.__setitem__(0, 1)),
             ("ivf_offsets", lambda t: t.__setitem__(4, int(t[5]) + 1)), ("ivf_offsets", lambda t: t.__setitem__(0, 2))]
    for copy in (False, True):
        for name, fn in cases:
            with pytest.raises(pl.PlaidError) as e:
                pl.plaid_index_from_view(broken(name, fn), 2, device=0, copy=copy)
            assert e.value.status == pl.plaid.PLAID_EINVAL, (name, copy)
        ok = pl.plaid_index_from_view(pu.device_arrays(w), 2, device=0, copy=copy)   # the unbroken arrays are accepted
        pl.plaid_index_free(ok)


def test_index_file_round_trip(pl, tmp_path):
    from synth import save_index_file
    w = make_workload(tiny_config(C=32, P=80, lo=1, hi=20, nbits=2, nq=3, seed=13), noise="calibrated")
    path = str(tmp_path / "tiny.plaid")
    save_index_file(path, w.numpy(), 2)
    a = pl.plaid_index_load(path, 0)
    b = pl.plaid_index_from_view(pu.device_arrays(w), 2, device=0, copy=False)
    try:
        Q = w.queries.to("cuda:0")
        ia, sa = pl.plaid_search(a, Q, 2, 0.3, 16, 4)
        ib, sb = pl.plaid_search(b, Q, 2, 0.3, 16, 4)
        torch.cuda.synchronize()
        assert torch.equal(ia, ib) and torch.equal(sa, sb)
        assert pl.plaid_index_info(a) == pl.plaid_index_info(b)
    finally:
        pl.plaid_index_free(a)
        pl.plaid_index_free(b)


def test_repeatable(pl):
    """The same call twice gives bit-identical outputs (no order-dependent arithmetic anywhere)."""
    cfg = get_config("cfg1")
    w = make_workload(cfg, device="cpu", noise="calibrated")
    gidx = pl.plaid_index_from_view(pu.device_arrays(w), 2, device=0, copy=False)
    try:
        Q = w.queries.to("cuda:0")
        a = pl.plaid_search(gidx, Q, 2, 0.45, 1024, 100)
        b = pl.plaid_search(gidx, Q, 2, 0.45, 1024, 100)
        one = [pl.plaid_search(gidx, Q[q:q + 1], 2, 0.45, 1024, 100) for q in range(Q.shape[0])]
        torch.cuda.synchronize()
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
        assert torch.equal(a[0], torch.cat([o[0] for o in one])) and torch.equal(a[1], torch.cat([o[1] for o in one]))
    finally:
        pl.plaid_index_free(gidx)
