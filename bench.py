#!/usr/bin/env python3
"""Benchmark of the PLAID search path on one MI355X.

A step is one pass of the whole path (S_cq, probes, candidates, both centroid-interaction stages,
decompression + MaxSim, top-k) over the configuration's full query batch, submitted as a single
plaid_search call with the index and the queries already resident in HBM.  The JSON line also
carries the batch-1 latency distribution (one query per call), the roofline of the kernel that
takes the largest share of a step (algorithmic work / event-timed duration; the other two large
kernels are listed beside it), and the CPU oracle timed on the host cores on a bounded sample of
the same queries.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg3] [--noise literal]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
FP64_MFMA_PEAK_TFLOPS = 78.6   # MI355X published dense fp64 matrix rate (the vector fp64 rate is the same figure)
FP32_MFMA_PEAK_TFLOPS = 157.3  # MI355X published dense fp32 matrix rate
FP16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X published dense fp16 / bf16 matrix rate

# HBM bytes per launch of each kernel as measured with `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` are read from the
# profile summary that holds them (lines "traffic <config> <noise> <stage> <bytes per launch> <kernel ms in that run>"),
# never typed in here: a stage without such a line reports null.
PROFILE_WITH_TRAFFIC = os.path.join(ROOT, "profiles", "bench_cfg3.txt")


def profiled_traffic():
    """(config, noise, stage) -> (HBM bytes per launch, kernel ms per launch in the profiled run) from the profile summary."""
    out = {}
    try:
        for line in open(PROFILE_WITH_TRAFFIC):
            f = line.split()
            if len(f) == 6 and f[0] == "traffic":
                out[(f[1], f[2], f[3])] = (int(f[4]), float(f[5]))
    except OSError:
        pass
    return out


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_work(pl, idx, w_dev, Q, params, cfg):
    """What the method must move, from the library's own candidate and survivor lists.
    Stage 2 (Eq. 3-5), code-stream figure: per candidate passage 8 bytes of offsets + 4 bytes per token code; for a query
    none of whose centroids passes Eq. 5 every bag is empty whatever the codes hold, and only the candidate bitmap is read
    and written.  Inverted-list figure (what the inverted form of candidate generation + stage 2 must move instead): 4 bytes
    per entry of the inverted lists of the probed and the surviving centroids (for a query without a surviving centroid,
    which only needs the candidate set, a list longer than a bitmap over the passages counts as that bitmap), 8 bytes
    per key written (queries with a surviving centroid) and the candidate and empty-bag words.
    Stage 3 (Eq. 3-4): per passage kept by stage 2, 8 bytes of offsets and 4 bytes per token code, plus the 128-byte S_cq
    row of every DISTINCT centroid among those tokens (a row shared by several tokens of a query has to be fetched once).
    Stage 4 (Section 4.5, Eq. 1): per surviving passage 8 bytes of offsets and per token its 4-byte code and its packed
    residual (16 * nbits bytes), plus the 128-byte S_cq row of every distinct centroid among those tokens."""
    import torch
    nprobe, t_cs, ndocs, k = params
    lens = (w_dev.doc_offsets[1:] - w_dev.doc_offsets[:-1])
    s2 = 0
    s4 = 0
    s4_tokens = 0
    n_skipped = 0
    s3 = 0
    inv = 0
    ivf_len = (w_dev.ivf_offsets[1:] - w_dev.ivf_offsets[:-1])
    ncand = []
    step = 512  # the library's chunk size, so that these launches look like the timed ones to a profiler
    bitmap_bytes = 4 * ((cfg.P + 31) // 32)

    def token_codes(pids):
        """codes of all tokens of the passages `pids` (1-D long tensor)"""
        ln = lens[pids]
        starts = w_dev.doc_offsets[pids]
        total = int(ln.sum())
        if total == 0:
            return w_dev.codes[:0], 0
        seg = torch.repeat_interleave(torch.arange(pids.numel(), device=pids.device), ln)
        first = torch.cumsum(ln, 0) - ln
        pos = torch.arange(total, device=pids.device) - first[seg] + starts[seg]
        return w_dev.codes[pos], total
    for q0 in range(0, Q.shape[0], step):
        _, _, b = pl.plaid_search_debug(idx, Q[q0:q0 + step], nprobe, t_cs, ndocs, k,
                                        want=("S_cq", "probed", "cand", "n_cand", "sel2_ids", "n2", "sel3_ids", "n3"))
        torch.cuda.synchronize()
        keep = b["S_cq"].max(dim=2).values >= t_cs                              # [queries, C]: centroids passing Eq. 5
        survivors = keep.sum(dim=1).tolist()
        del b["S_cq"]
        for j in range(keep.shape[0]):
            lists = keep[j].clone() if survivors[j] <= 63 else torch.zeros_like(keep[j])
            lists[b["probed"][j].flatten().long()] = True
            list_bytes = 4 * ivf_len[lists]
            if survivors[j] == 0:
                list_bytes = torch.clamp(list_bytes, max=bitmap_bytes)
            inv += int(list_bytes.sum()) + 2 * bitmap_bytes
        for j in range(b["cand"].shape[0]):
            n = int(b["n_cand"][j])
            c = b["cand"][j, :n].long()
            if survivors[j] > 0:
                s2 += 8 * n + 4 * int(lens[c].sum())
                # (inverted form: one 4-byte score word per candidate; more than 63 survivors: the candidates' codes too)
                inv += 4 * n if survivors[j] <= 63 else 4 * n + 4 * int(lens[c].sum())
            else:
                s2 += 8 * ((cfg.P + 31) // 32)
                n_skipped += 1
            ncand.append(n)
            n2 = int(b["n2"][j])
            tc, t = token_codes(b["sel2_ids"][j, :n2].long())
            s3 += 8 * n2 + 4 * t + 128 * int(torch.unique(tc).numel())
            n3 = int(b["n3"][j])
            tc, t = token_codes(b["sel3_ids"][j, :n3].long())
            s4_tokens += t
            s4 += 8 * n3 + t * (4 + 16 * cfg.nbits) + 128 * int(torch.unique(tc).numel())
    return {"stage2_bytes": s2, "stage2_inverted_bytes": inv, "stage3_bytes": s3, "stage4_bytes": s4, "stage4_tokens": s4_tokens,
            "mean_candidates": float(sum(ncand)) / max(1, len(ncand)), "queries_without_survivors": n_skipped}


def measure(pl, torch, np, cfg, noise, args, latency=True):
    """Generate the workload on the GPU, time K steps of the full batch (and, if asked, batch-1 latency) and derive the
    rooflines.  Returns a dict of results plus the objects the caller still needs."""
    dev = torch.device("cuda:0")
    t0 = time.time()
    w = make_workload_(cfg, device=dev, noise=noise)
    torch.cuda.synchronize()
    log(f"[bench] generated {cfg.name}/{noise}: C={cfg.C} P={cfg.P} N={w.N} nbits={cfg.nbits} "
        f"ivf={w.ivf_pids.numel()} in {time.time() - t0:.1f}s")
    names = ("centroids", "doc_offsets", "codes", "residuals", "bucket_weights", "ivf_offsets", "ivf_pids")
    idx = pl.plaid_index_from_view({n: getattr(w, n) for n in names}, cfg.nbits, device=0, copy=False)
    Q = w.queries
    nq = Q.shape[0]
    params = (cfg.nprobe, cfg.t_cs, cfg.ndocs, cfg.k)
    out_ids = torch.empty((nq, cfg.k), dtype=torch.int32, device=dev)
    out_sc = torch.empty((nq, cfg.k), dtype=torch.float32, device=dev)
    # ---- throughput: K steps of the full batch, stage events on (they cost one sync per query chunk)
    # queries per internal launch: the library's own choice (512, fewer when the per-query workspace is large: cfg4, cfg5)
    _, CHUNK = pl.plaid_workspace_bytes(cfg.C, cfg.P, nq, cfg.nprobe, cfg.ndocs, cfg.k)
    launches = (nq + CHUNK - 1) // CHUNK
    pl.plaid_set_stage_timing(idx, True)
    for _ in range(args.warmup):
        pl.plaid_search(idx, Q, *params, out_ids=out_ids, out_scores=out_sc)
    torch.cuda.synchronize()
    stage_acc = {}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        pl.plaid_search(idx, Q, *params, out_ids=out_ids, out_scores=out_sc)
        for s, ms in pl.plaid_get_stage_ms(idx).items():
            stage_acc[s] = stage_acc.get(s, 0.0) + ms
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    qps = nq * args.steps / dt
    stage_ms = {s: v / args.steps for s, v in stage_acc.items()}
    log(f"[bench] batch of {nq}: {ms_per_step:.3f} ms/step, {qps:.0f} queries/s; stage ms/step {stage_ms}")
    # shader-clock and 100 MHz timer ticks of the score kernel's workgroups in the last timed step (read outside the timed
    # region: the call copies from the device)
    clock_ticks = pl.plaid_get_score_kernel_clocks(idx)
    scq_clock_mhz = round(100.0 * clock_ticks[0] / clock_ticks[1], 0) if clock_ticks[1] else None
    pl.plaid_set_stage_timing(idx, False)

    # ---- batch-1 latency: one query per call, host clock around call + stream sync
    nlat = min(args.latency_queries, nq) if latency else 0
    for q in range(min(20, nq) if nlat else 0):
        pl.plaid_search(idx, Q[q:q + 1], *params, out_ids=out_ids[q:q + 1], out_scores=out_sc[q:q + 1])
    torch.cuda.synchronize()
    best = None
    enq = None
    for _trial in range(3 if nlat else 0):
        lat = np.empty(nlat)
        enq_t = np.empty(nlat)
        for q in range(nlat):
            t1 = time.perf_counter()
            pl.plaid_search(idx, Q[q:q + 1], *params, out_ids=out_ids[q:q + 1], out_scores=out_sc[q:q + 1])
            t2 = time.perf_counter()
            torch.cuda.synchronize()
            lat[q] = (time.perf_counter() - t1) * 1e3
            enq_t[q] = (t2 - t1) * 1e3
        if best is None or lat.mean() < best.mean():
            best, enq = lat, enq_t
    lat = best if nlat else np.zeros(1)
    enq = enq if nlat else np.zeros(1)
    if nlat:
        log(f"[bench] batch-1 latency over {nlat} queries (best of 3 trials): p50 {np.percentile(lat, 50):.4f} ms, "
            f"p99 {np.percentile(lat, 99):.4f} ms, mean {lat.mean():.4f} ms; host enqueue p50 {np.percentile(enq, 50):.4f} ms")

    # ---- the same, replaying a HIP graph of the search (plaid_search_static records into a graph because it allocates
    # nothing): the host enqueues one graph instead of a dozen kernels.  A reference figure: never fails the benchmark.
    lat_graph = None
    if nlat and not args.no_graph_latency:
        try:
            k_out = out_ids.shape[1]
            Qb = Q[0:1].clone()
            gi = torch.empty((1, k_out), dtype=torch.int32, device=Q.device)
            gs = torch.empty((1, k_out), dtype=torch.float32, device=Q.device)
            pl.plaid_search_static(idx, Qb, *params, gi, gs)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                pl.plaid_search_static(idx, Qb, *params, gi, gs)
            torch.cuda.synchronize()
            lg = np.empty(nlat)
            same = True
            for q in range(nlat):
                Qb.copy_(Q[q:q + 1])
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                graph.replay()
                torch.cuda.synchronize()
                lg[q] = (time.perf_counter() - t1) * 1e3
                same = same and bool(torch.equal(gi[0], out_ids[q]))
            lat_graph = {"p50": round(float(np.percentile(lg, 50)), 4), "p99": round(float(np.percentile(lg, 99)), 4),
                         "mean": round(float(lg.mean()), 4), "queries": int(nlat), "ids_equal_to_eager_search": same}
            log(f"[bench] batch-1 latency, graph replay: p50 {lat_graph['p50']:.4f} ms, p99 {lat_graph['p99']:.4f} ms; "
                f"ids equal to the eager search: {same}")
            del graph
        except Exception as e:
            log(f"[bench] graph-replay latency not measured: {e}")

    # ---- rooflines of the three large kernels; the one with the largest share of the step is the headline
    roofline = None
    rooflines = {}
    if not args.no_roofline:
        work = algorithmic_work(pl, idx, w, Q, params, cfg)
        traffic_table = profiled_traffic()

        def entry(stage, kernel, bound, amount, unit_scale, peak, unit, extra):
            t = stage_ms[stage] * 1e-3
            ach = amount / t / unit_scale if t > 0 else 0.0
            prof = traffic_table.get((cfg.name, noise, stage))
            e = {"bound": bound, "kernel": kernel, "achieved": round(ach, 1), "peak": peak, "unit": unit,
                 "frac": round(ach / peak, 4),
                 # hardware bytes per launch from the rocprofv3 counter runs recorded in the named profile summary (not
                 # measured in this run), and the rate they give over the kernel time of that same profiled run
                 "traffic": prof[0] if prof else None,
                 "traffic_source": os.path.relpath(PROFILE_WITH_TRAFFIC, ROOT) if prof else None,
                 "traffic_gbs_in_profiled_run": round(prof[0] / (prof[1] * 1e-3) / 1e9, 1) if prof and prof[1] > 0 else None,
                 "kernel_ms_per_step": round(stage_ms[stage], 4), "launches_per_step": launches, "queries_per_launch": CHUNK,
                 "kernel_ms_per_launch": round(stage_ms[stage] / launches, 4)}
            e.update(extra)
            log(f"[bench] {stage}: {ach:.1f} {unit} = {ach / peak:.1%} of {peak:g} ({bound}); {stage_ms[stage]:.3f} ms/step")
            return e

        scq_flop = 2.0 * cfg.C * 128 * 32 * nq
        form = pl.plaid_get_score_kernel(idx)
        if form == 2 and cfg.nprobe <= 8:
            # split-fp16 matrix kernel: three fp16 products per term of Eq. 2, far below the matrix rate's ceiling; what
            # bounds it is the write of S_cq itself (128 bytes per centroid and query) next to one read of the centroids'
            # operands (512 bytes each) per launch and of the queries' (16 KB each)
            scq_bytes = nq * cfg.C * 128 + launches * cfg.C * 512 + nq * 16384
            t_scq = stage_ms["scq"] * 1e-3
            rooflines["scq"] = entry(
                "scq", "S_cq = C.Q^T (Eq. 2): fp16 matrix instruction on operands split into two fp16 terms, fp32 accumulation",
                "hbm", scq_bytes, 1e9, HBM_PEAK_GBS, "GB/s",
                {"algorithmic_bytes_per_step": scq_bytes, "algorithmic_bytes_per_launch": scq_bytes // launches, "dtype": "f16x2/f32",
                 "matrix_flop_per_step": 3 * scq_flop,
                 "fp16_mfma_tflops": round(3 * scq_flop / t_scq / 1e12, 1) if t_scq > 0 else None,
                 "fp16_mfma_frac": round(3 * scq_flop / t_scq / 1e12 / FP16_MFMA_PEAK_TFLOPS, 4) if t_scq > 0 else None,
                 # the clock the chip held while this kernel ran (shader-clock counter over the 100 MHz timer, read inside
                 # the kernel by every workgroup): the published peaks are quoted at the top clock
                 "shader_clock_mhz_during_kernel": scq_clock_mhz})
        else:
            rooflines["scq"] = entry(
                "scq", "S_cq = C.Q^T (Eq. 2) in double through the fp64 matrix instruction" if form == 1
                else "S_cq = C.Q^T (Eq. 2), fp64 fused multiply-add chain", "mfma", scq_flop, 1e12, FP64_MFMA_PEAK_TFLOPS, "TFLOP/s",
                {"algorithmic_flop_per_step": scq_flop, "algorithmic_flop_per_launch": scq_flop / launches, "dtype": "f64"})
        inverted = bool(pl.plaid_get_stage2_kernel(idx))
        s2_bytes = work["stage2_inverted_bytes"] if inverted else work["stage2_bytes"]
        rooflines["stage2_ci"] = entry(
            "stage2_ci", ("candidates + stage-2 centroid interaction (Section 4.1, Eq. 3-5) from the inverted lists" if inverted
                          else "stage-2 centroid interaction (Eq. 3-5) streaming the candidates' codes"), "hbm", s2_bytes, 1e9,
            HBM_PEAK_GBS, "GB/s",
            {"algorithmic_bytes_per_step": s2_bytes, "algorithmic_bytes_per_launch": s2_bytes // launches,
             "code_stream_bytes_per_step": work["stage2_bytes"],
             "mean_candidates_per_query": work["mean_candidates"],
             "queries_without_surviving_centroid": work["queries_without_survivors"]})
        rooflines["stage3_ci"] = entry(
            "stage3_ci", "stage-3 centroid interaction without pruning (Eq. 3-4): codes and S_cq rows of the ndocs survivors",
            "hbm", work["stage3_bytes"], 1e9, HBM_PEAK_GBS, "GB/s",
            {"algorithmic_bytes_per_step": work["stage3_bytes"], "algorithmic_bytes_per_launch": work["stage3_bytes"] // launches})
        rooflines["stage4_maxsim"] = entry(
            "stage4_maxsim", "stage-4 decompression + MaxSim (Section 4.5, Eq. 1) over the ndocs/4 survivors", "hbm",
            work["stage4_bytes"], 1e9, HBM_PEAK_GBS, "GB/s",
            {"algorithmic_bytes_per_step": work["stage4_bytes"], "algorithmic_bytes_per_launch": work["stage4_bytes"] // launches,
             "tokens_per_step": work["stage4_tokens"],
             # three fp16 matrix products per fp32 product (two-term operand splits): 3 x 2 x 32 x 128 flop per token
             "fp16_mfma_tflops": round(3 * work["stage4_tokens"] * 8192 / (stage_ms["stage4_maxsim"] * 1e-3) / 1e12, 2),
             "fp16_mfma_frac": round(3 * work["stage4_tokens"] * 8192 / (stage_ms["stage4_maxsim"] * 1e-3) / 1e12
                                     / FP16_MFMA_PEAK_TFLOPS, 4)})
        dominant = max(rooflines, key=lambda s: stage_ms[s])
        roofline = dict(rooflines[dominant])
        roofline["stage"] = dominant

    return {"w": w, "idx": idx, "Q": Q, "nq": nq, "params": params, "out_ids": out_ids, "qps": qps, "ms_per_step": ms_per_step,
            "stage_ms": stage_ms, "lat": lat, "enq": enq, "nlat": nlat, "lat_graph": lat_graph, "roofline": roofline,
            "rooflines": rooflines}


def memory_shortfall(torch, cfg):
    """None when the configuration's index fits the free device memory three times over (generation temporaries, the
    library's workspace), else the reason it does not."""
    mean_len = {"cfg1": 40, "cfg2": 60, "cfg3": 65, "cfg4": 68, "cfg5": 70}.get(cfg.name, 70)
    index_bytes = cfg.P * mean_len * (4 + 16 * cfg.nbits + 4)
    free_dev, _ = torch.cuda.mem_get_info(0)
    if free_dev < 3 * index_bytes:
        return f"{free_dev / 2**30:.0f} GiB of free device memory, {3 * index_bytes / 2**30:.0f} GiB wanted for {cfg.name}"
    return None


def measure_ablation(pl, torch, np, cfg, args):
    """The ablation of Section 5.3 / Figure 6 on this chip, calibrated noise, hyperparameters of the k = 1000 setting of
    Table 2 as in the paper (nprobe 4, t_cs 0.4, ndocs 4096): vanilla ColBERTv2 retrieval (ncandidates 2^16), then with one
    stage of centroid interaction without pruning (the pipeline at t_cs = -inf), then with centroid pruning (the full
    pipeline).  The paper's fourth rung, its optimised kernels, has no counterpart here: every rung runs the same HIP
    kernels.  Throughput over a batch of 128 queries, best of three."""
    dev = torch.device("cuda:0")
    w = make_workload_(cfg, device=dev, noise="calibrated")
    names = ("centroids", "doc_offsets", "codes", "residuals", "bucket_weights", "ivf_offsets", "ivf_pids")
    idx = pl.plaid_index_from_view({n: getattr(w, n) for n in names}, cfg.nbits, device=0, copy=False)
    Q = w.queries[:128].contiguous()
    nprobe, t_cs, ndocs, k, ncand = 4, 0.4, 4096, 1000, 1 << 16

    def best_of(fn):
        fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            best = dt if best is None or dt < best else best
        return best / Q.shape[0] * 1e3
    rungs = [("vanilla ColBERTv2 retrieval", lambda: pl.plaid_search_vanilla(idx, Q, nprobe, ncand, k)),
             ("+ centroid interaction (stage 3, no pruning)", lambda: pl.plaid_search(idx, Q, nprobe, float("-inf"), ndocs, k)),
             ("+ centroid pruning (stage 2): the full pipeline", lambda: pl.plaid_search(idx, Q, nprobe, t_cs, ndocs, k))]
    out = {"workload": f"{cfg.name} (calibrated noise), {Q.shape[0]} queries per call", "nprobe": nprobe, "t_cs": t_cs, "ndocs": ndocs,
           "k": k, "ncandidates": ncand, "rungs": []}
    base = None
    for name, fn in rungs:
        ms = best_of(fn)
        base = ms if base is None else base
        out["rungs"].append({"rung": name, "ms_per_query": round(ms, 4), "speedup_over_vanilla": round(base / ms, 2)})
        log(f"[bench] ablation, {name}: {ms:.4f} ms per query ({base / ms:.2f}x vanilla)")
    pl.plaid_index_free(idx)
    del w
    torch.cuda.empty_cache()
    return out


def measured_copy_gbs(torch):
    """Bandwidth a plain device-to-device copy of 1 GiB reaches on this machine (bytes read + bytes written per second):
    the achievable figure to read the 8 TB/s vendor peak against.  None if the measurement itself fails."""
    try:
        dev = torch.device("cuda:0")
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            dst.copy_(src)
        b.record()
        torch.cuda.synchronize()
        gbs = 5 * 2 * src.numel() * 4 / (a.elapsed_time(b) * 1e-3) / 1e9
        del src, dst
        torch.cuda.empty_cache()
        return round(gbs, 1)
    except Exception as e:  # a reference figure only: never fail the benchmark over it
        log(f"[bench] copy bandwidth not measured: {e}")
        return None


def measure_index_build(pl, torch, np, cfg, noise, cpu: bool):
    """The index-construction calls (the step before the search path) at the configuration's sizes: inverted lists of all
    N tokens, residual encoding and nearest-centroid assignment of the first 2^20 token vectors.  Each call synchronises
    internally, so it is timed on the host clock (best of three).  Returns a dict for the JSON line."""
    dev = torch.device("cuda:0")
    w = make_workload_(cfg, device=dev, noise=noise, keep_embeddings=1 << 20)
    x = w.sample_embeddings
    n = int(x.shape[0])
    codes_n = w.codes[:n].contiguous()
    cut = w.bucket_cutoffs.to(dev)

    def best_of(fn, reps=3):
        best = None
        for _ in range(reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            out = fn()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            best = dt if best is None or dt < best else best
        return best, out

    out = {"workload": f"{cfg.name} ({noise} noise)", "tokens_total": int(w.N), "vectors_sampled": n}
    t, (off, pids) = best_of(lambda: pl.plaid_build_ivf(w.codes, w.doc_offsets, cfg.C))
    ivf_bytes = 2 * 4 * int(w.N) + 2 * 8 * (cfg.P + 1) + 4 * int(pids.numel()) + 8 * (cfg.C + 1)
    out["build_ivf"] = {"seconds": round(t, 5), "tokens_per_s": round(int(w.N) / t, 1), "entries": int(pids.numel()),
                        "algorithmic_bytes": ivf_bytes, "achieved_gbs": round(ivf_bytes / t / 1e9, 1),
                        "frac_of_hbm_peak": round(ivf_bytes / t / 1e9 / HBM_PEAK_GBS, 4),
                        "identical_to_generator": bool(torch.equal(off, w.ivf_offsets) and torch.equal(pids, w.ivf_pids))}
    t, res = best_of(lambda: pl.plaid_encode_residuals(w.centroids, x, codes_n, cut, cfg.nbits))
    # a vector, its code and its packed residual per token, plus the 512-byte row of every distinct centroid among them
    enc_bytes = n * (512 + 4 + 16 * cfg.nbits) + 512 * int(torch.unique(codes_n).numel())
    out["encode_residuals"] = {"seconds": round(t, 5), "tokens_per_s": round(n / t, 1), "algorithmic_bytes": enc_bytes,
                               "achieved_gbs": round(enc_bytes / t / 1e9, 1),
                               "frac_of_hbm_peak": round(enc_bytes / t / 1e9 / HBM_PEAK_GBS, 4),
                               "identical_to_generator": bool(torch.equal(res, w.residuals[:n]))}
    t, codes = best_of(lambda: pl.plaid_assign_centroids(w.centroids, x), reps=2)
    flop = 2.0 * cfg.C * 128 * n
    asg = {"seconds": round(t, 5), "tokens_per_s": round(n / t, 1), "algorithmic_flop": flop,
           "share_equal_to_drawn_codes": round(float((codes == codes_n).float().mean()), 4)}
    if os.environ.get("PLAID_SCQ_FORM", "split16") == "split16":
        # the search path's split-fp16 score kernel, three fp16 matrix products per fp32 product, without its score
        # stores (the probe kernel re-evaluates the rows of the best tile in double): bound by the matrix rate
        asg.update({"bound": "mfma", "fp16_matrix_tflops": round(3 * flop / t / 1e12, 1),
                    "frac_of_fp16_matrix_peak": round(3 * flop / t / 1e12 / FP16_MFMA_PEAK_TFLOPS, 4)})
    else:
        asg.update({"bound": "mfma", "achieved_tflops": round(flop / t / 1e12, 1),
                    "frac_of_fp64_matrix_peak": round(flop / t / 1e12 / FP64_MFMA_PEAK_TFLOPS, 4)})
    out["assign_centroids"] = asg
    for k_ in ("build_ivf", "encode_residuals", "assign_centroids"):
        log(f"[bench] index construction, {k_}: {out[k_]}")
    if cpu:
        from oracle import oracle as orc
        ch, dh = w.codes.cpu().numpy(), w.doc_offsets.cpu().numpy()
        t0 = time.perf_counter()
        orc.build_ivf(ch, dh, cfg.C)
        t_ivf = time.perf_counter() - t0
        xh, cenh = x.cpu().numpy(), w.centroids.cpu().numpy()
        t0 = time.perf_counter()
        orc.encode(xh, ch[:n], cenh, w.bucket_cutoffs.cpu().numpy(), cfg.nbits)
        t_enc = time.perf_counter() - t0
        ng = 8   # groups of 32 vectors: the oracle's S_cq routine is a plain triple loop
        t0 = time.perf_counter()
        for g_ in range(ng):
            orc.top_nprobe(orc.scq(cenh, xh[32 * g_:32 * g_ + 32]), 1)
        t_asg = time.perf_counter() - t0
        out["cpu_oracle"] = {"kind": "oracle", "cores": 1,
                             "build_ivf_tokens_per_s": round(int(w.N) / t_ivf, 1),
                             "encode_residuals_tokens_per_s": round(n / t_enc, 1),
                             "assign_centroids_tokens_per_s": round(32 * ng / t_asg, 1),
                             "sample": f"all {int(w.N)} tokens / the same {n} vectors / the first {32 * ng} vectors"}
        log(f"[bench] index construction, CPU oracle: {out['cpu_oracle']}")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="cfg3", help="cfg1 .. cfg5 (synth/workload.py)")
    ap.add_argument("--noise", default="literal", choices=["literal", "calibrated"])
    ap.add_argument("--latency-queries", type=int, default=512, help="queries timed one per call for p50/p99")
    ap.add_argument("--cpu-sample", type=int, default=512, help="queries the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--single-noise", action="store_true", help="skip the run on the other reading of the noise scale")
    ap.add_argument("--no-index-build", action="store_true", help="skip the timing of the index-construction calls")
    ap.add_argument("--no-graph-latency", action="store_true", help="skip the HIP-graph replay of the batch-1 search")
    ap.add_argument("--no-ablation", action="store_true", help="skip the vanilla-retrieval ablation ladder (Section 5.3)")
    ap.add_argument("--no-operating-points", action="store_true",
                    help="skip the k = 10 (cfg2), k = 1000 (cfg4) and 1-bit (cfg5) operating points reported beside the headline")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run four 1 GiB device-to-device copies (reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2205_09707_amd as pl
    from synth import get_config, make_workload
    global make_workload_
    make_workload_ = make_workload

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    pl.load_library()
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)     # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        log("[bench] copy calibration: 4 copies, each reads 1 GiB (1048576 KiB) and writes 1 GiB")
        return
    cfg = get_config(args.config)
    r = measure(pl, torch, np, cfg, args.noise, args)
    w, idx, Q, nq, params, out_ids = r["w"], r["idx"], r["Q"], r["nq"], r["params"], r["out_ids"]
    qps, ms_per_step, stage_ms, lat, enq, nlat = r["qps"], r["ms_per_step"], r["stage_ms"], r["lat"], r["enq"], r["nlat"]
    roofline, rooflines, lat_graph = r["roofline"], r["rooflines"], r["lat_graph"]

    # ---- CPU oracle on a bounded sample of the same queries (rank 0, N = 1)
    cpu = None
    if args.cpu_sample > 0:
        from oracle import oracle as orc
        ns = min(args.cpu_sample, nq)
        ix = orc.Index(w.numpy(), cfg.nbits)
        Qh = np.ascontiguousarray(Q[:ns].cpu().numpy())
        t1 = time.perf_counter()
        o_ids, o_sc, used = orc.search_batch(ix, Qh, *params, nthreads=0)
        dt_cpu = time.perf_counter() - t1
        g_ids = out_ids[:ns].cpu().numpy()
        agree = float(np.mean(g_ids == o_ids))
        # one thread, one query at a time: the oracle's per-query latency (8 queries)
        lat1 = []
        for qq in range(min(8, ns)):
            t2 = time.perf_counter()
            orc.search(ix, Qh[qq], *params)
            lat1.append((time.perf_counter() - t2) * 1e3)
        cpu = {"value": round(ns / dt_cpu, 3), "unit": "queries/s", "cores": int(used), "kind": "oracle",
               "single_thread_latency_ms_p50": round(float(np.percentile(lat1, 50)), 2),
               "sample": f"first {ns} of the {nq} queries of {cfg.name}/{args.noise}, whole pipeline, one query per thread",
               "seconds": round(dt_cpu, 2), "id_agreement_with_gpu": agree}
        log(f"[bench] CPU oracle: {ns} queries in {dt_cpu:.2f}s on {used} threads; id agreement with GPU {agree:.4f}")

    forms = {"score_kernel": ("vector", "matrix", "split16")[pl.plaid_get_score_kernel(idx)],
             "stage2_kernel": "inverted" if pl.plaid_get_stage2_kernel(idx) else "stream"}
    n_embeddings = int(w.N)
    pl.plaid_index_free(idx)
    del w, idx, Q, r
    torch.cuda.empty_cache()

    # ---- the other reading of the generator's noise scale, throughput and rooflines only (never mixed into `value`)
    other = None
    if not args.single_noise:
        on = "calibrated" if args.noise == "literal" else "literal"
        r2 = measure(pl, torch, np, cfg, on, args, latency=False)
        pl.plaid_index_free(r2["idx"])
        other = {"noise": on, "value": round(r2["qps"], 2), "unit": "queries/s", "ms_per_step": round(r2["ms_per_step"], 4),
                 "stage_ms_per_step": {s_: round(v, 4) for s_, v in r2["stage_ms"].items()},
                 "roofline_by_stage": r2["rooflines"] or None}
        del r2
    copy_gbs = measured_copy_gbs(torch)
    log(f"[bench] plain 1 GiB device copy: {copy_gbs} GB/s read + written (vendor HBM peak {HBM_PEAK_GBS:g})")
    # ---- the other operating points of the metric (k = 10 and k = 1000; the headline configuration has k = 100):
    # throughput of the full batch and batch-1 latency, both readings of the noise scale
    points = None
    if not args.no_operating_points and args.config == "cfg3":
        points = {}
        for name in ("cfg2", "cfg4", "cfg5"):
            c2 = get_config(name)
            short = memory_shortfall(torch, c2)
            if short:
                points[name] = {"skipped": short}
                log(f"[bench] operating point {name} skipped: {short}")
                continue
            a2 = argparse.Namespace(**vars(args))
            a2.no_roofline, a2.steps, a2.warmup = True, max(2, args.steps // 3), 1
            a2.latency_queries = min(args.latency_queries, 128)
            points[name] = {"k": c2.k, "nprobe": c2.nprobe, "t_cs": c2.t_cs, "ndocs": c2.ndocs}
            # (cfg5: the largest index, 1-bit residuals; the calibrated reading only, to keep the default run short)
            for nz in (("calibrated",) if name == "cfg5" else ("literal", "calibrated")):
                r3 = measure(pl, torch, np, c2, nz, a2, latency=True)
                l3 = r3["lat"]
                points[name][nz] = {
                    "workload": f"{name} ({nz} noise): C={c2.C}, P={c2.P}, N={int(r3['w'].N)}, {c2.nbits}-bit, {r3['nq']} queries",
                    "value": round(r3["qps"], 2), "unit": "queries/s", "ms_per_step": round(r3["ms_per_step"], 4), "steps": a2.steps,
                    "stage2_kernel": "inverted" if pl.plaid_get_stage2_kernel(r3["idx"]) else "stream",
                    "stage_ms_per_step": {s_: round(v, 4) for s_, v in r3["stage_ms"].items()},
                    "latency_batch1_ms": {"p50": round(float(np.percentile(l3, 50)), 4), "p99": round(float(np.percentile(l3, 99)), 4),
                                          "mean": round(float(l3.mean()), 4), "queries": int(r3["nlat"]), "trials": 3,
                                          "graph_replay": r3["lat_graph"]}}
                pl.plaid_index_free(r3["idx"])
                del r3
                torch.cuda.empty_cache()
    ablation = None
    if not args.no_ablation and args.config == "cfg3":
        ablation = measure_ablation(pl, torch, np, cfg, args)
    build = None
    if not args.no_index_build:
        build = measure_index_build(pl, torch, np, cfg, args.noise, cpu=args.cpu_sample > 0)
    line = {
        "metric": "queries_per_sec", "value": round(qps, 2), "unit": "queries/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if forms["score_kernel"] == "split16" else "f64/f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} ({args.noise} noise): C={cfg.C} centroids, P={cfg.P} passages, N={n_embeddings} "
                               f"embeddings, {cfg.nbits}-bit residuals, {nq} queries x 32 x 128",
                   "nprobe": cfg.nprobe, "t_cs": cfg.t_cs, "ndocs": cfg.ndocs, "k": cfg.k,
                   "queries_per_step": nq, "index_generated_on": "cuda", **forms,
                   "arithmetic": ("S_cq: fp16 matrix instruction on two-term fp16 splits of the fp32 operands, f32 accumulation, every "
                                  "decision near its threshold re-evaluated in f64; centroid-interaction sums in f64; MaxSim in f32"
                                  if forms["score_kernel"] == "split16" else
                                  "S_cq and the centroid-interaction sums accumulate in f64 (stored f32); MaxSim in f32")},
        "latency_batch1_ms": {"p50": round(float(np.percentile(lat, 50)), 4), "p99": round(float(np.percentile(lat, 99)), 4),
                              "mean": round(float(lat.mean()), 4), "queries": int(nlat), "trials": 3, "host_enqueue_p50": round(float(np.percentile(enq, 50)), 4),
                              "qps": round(1e3 / float(lat.mean()), 1) if nlat else None, "graph_replay": lat_graph},
        "stage_ms_per_step": {s: round(v, 4) for s, v in stage_ms.items()},
        "roofline": roofline, "roofline_by_stage": rooflines or None, "cpu_baseline": cpu,
        "other_noise_reading": other, "operating_points": points, "ablation": ablation, "index_construction": build,
        "hbm": {"vendor_peak_gbs": HBM_PEAK_GBS, "measured_copy_gbs": copy_gbs},
        # the paper's own figures, for context only: other hardware, real corpora, per-query latency (Tables 3 and 6)
        "paper_context": {"hardware": "one NVIDIA TITAN V / 8 threads of a Xeon Gold 6132", "unit": "ms per query",
                          "ms_marco_v1_8.8M_passages": {"k=10": {"gpu": 11.5, "cpu8": 31.5}, "k=100": {"gpu": 20.2, "cpu8": 52.9},
                                                        "k=1000": {"gpu": 38.4, "cpu8": 101.3},
                                                        "vanilla_colbertv2_p4_c65536": {"gpu": 259.6, "cpu8": 4568.5}},
                          "ms_marco_v2_138M_passages_1bit": {"k=10": {"gpu": 47.1, "cpu8": 136.4}, "k=100": {"gpu": 96.1, "cpu8": 181.9}},
                          "nearest_synthetic_config": {"ms_marco_v1": "cfg4 (operating_points)", "ms_marco_v2": "cfg5 = one GPU's share"}},
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
