#!/usr/bin/env python3
"""Benchmark of the PLAID search path on one MI355X.

A step is one pass of the whole path (S_cq, probes, candidates, both centroid-interaction stages,
decompression + MaxSim, top-k) over the configuration's full query batch, submitted as a single
plaid_search call with the index and the queries already resident in HBM.  The JSON line also
carries the batch-1 latency distribution (one query per call), the roofline of the dominant
kernel (stage-2 centroid interaction, HBM-bound: algorithmic bytes / event-timed duration), and
the CPU oracle timed on the host cores on a bounded sample of the same queries.

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

# HBM bytes per launch of the stage-2 kernel (64 queries), from `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` runs of this
# file, each scaled by the counter's reading on a 1 GiB device copy (fetch reads half the bytes: x2; write: x1).
# Source and date of every figure: profiles/s2_stream_<config>_<noise>.txt.  None = not measured.
MEASURED_TRAFFIC_PER_LAUNCH = {
    ("cfg3", "literal"): int((980377.8 * 2.0 + 11660.3 * 1.0) * 1024),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_stage2_bytes(pl, idx, w_dev, Q, params):
    """Sum over queries of (8 bytes of passage offsets + 4 bytes per token code) over the candidate passages:
    what the pruned centroid interaction must read (codes of every candidate, Eq. 3-5)."""
    import torch
    nprobe, t_cs, ndocs, k = params
    lens = (w_dev.doc_offsets[1:] - w_dev.doc_offsets[:-1])
    total = 0
    ncand = []
    step = 64   # the library's chunk size, so that these launches look like the timed ones to a profiler
    for q0 in range(0, Q.shape[0], step):
        _, _, b = pl.plaid_search_debug(idx, Q[q0:q0 + step], nprobe, t_cs, ndocs, k, want=("cand", "n_cand"))
        torch.cuda.synchronize()
        for j in range(b["cand"].shape[0]):
            n = int(b["n_cand"][j])
            c = b["cand"][j, :n].long()
            total += 8 * n + 4 * int(lens[c].sum())
            ncand.append(n)
    return total, ncand


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="cfg3", help="cfg1 .. cfg5 (synth/workload.py)")
    ap.add_argument("--noise", default="literal", choices=["literal", "calibrated"])
    ap.add_argument("--latency-queries", type=int, default=512, help="queries timed one per call for p50/p99")
    ap.add_argument("--cpu-sample", type=int, default=16, help="queries the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--no-roofline", action="store_true")
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
    t0 = time.time()
    w = make_workload(cfg, device=dev, noise=args.noise)
    torch.cuda.synchronize()
    log(f"[bench] generated {cfg.name}/{args.noise}: C={cfg.C} P={cfg.P} N={w.N} nbits={cfg.nbits} "
        f"ivf={w.ivf_pids.numel()} in {time.time() - t0:.1f}s")
    names = ("centroids", "doc_offsets", "codes", "residuals", "bucket_weights", "ivf_offsets", "ivf_pids")
    idx = pl.plaid_index_from_view({n: getattr(w, n) for n in names}, cfg.nbits, device=0, copy=False)
    Q = w.queries
    nq = Q.shape[0]
    params = (cfg.nprobe, cfg.t_cs, cfg.ndocs, cfg.k)
    out_ids = torch.empty((nq, cfg.k), dtype=torch.int32, device=dev)
    out_sc = torch.empty((nq, cfg.k), dtype=torch.float32, device=dev)

    # ---- throughput: K steps of the full batch, stage events on (they cost one sync per query chunk)
    CHUNK = 64   # queries per internal launch
    pl.plaid_set_max_chunk(idx, CHUNK)
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
    pl.plaid_set_stage_timing(idx, False)

    # ---- batch-1 latency: one query per call, host clock around call + stream sync
    nlat = min(args.latency_queries, nq)
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
    log(f"[bench] batch-1 latency over {nlat} queries (best of 3 trials): p50 {np.percentile(lat, 50):.4f} ms, "
        f"p99 {np.percentile(lat, 99):.4f} ms, mean {lat.mean():.4f} ms; host enqueue p50 {np.percentile(enq, 50):.4f} ms")

    # ---- roofline of the dominant kernel (stage-2 centroid interaction over all candidates)
    roofline = None
    if not args.no_roofline:
        alg_bytes, ncand = algorithmic_stage2_bytes(pl, idx, w, Q, params)
        t_s2 = stage_ms["stage2_ci"] * 1e-3
        achieved = alg_bytes / t_s2 / 1e9 if t_s2 > 0 else 0.0
        roofline = {"bound": "hbm", "kernel": "stage-2 centroid interaction (Eq. 3-5) over all candidates",
                    "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": MEASURED_TRAFFIC_PER_LAUNCH.get((cfg.name, args.noise)),
                    "algorithmic_bytes_per_step": alg_bytes, "kernel_ms_per_step": round(stage_ms["stage2_ci"], 4),
                    "launches_per_step": launches, "queries_per_launch": CHUNK,
                    "algorithmic_bytes_per_launch": alg_bytes // launches,
                    "kernel_ms_per_launch": round(stage_ms["stage2_ci"] / launches, 4),
                    "mean_candidates_per_query": float(np.mean(ncand))}
        log(f"[bench] stage 2: {alg_bytes / 1e6:.1f} MB algorithmic per step in {stage_ms['stage2_ci']:.3f} ms "
            f"-> {achieved:.0f} GB/s ({achieved / HBM_PEAK_GBS:.1%} of {HBM_PEAK_GBS:.0f})")

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
        cpu = {"value": round(ns / dt_cpu, 3), "unit": "queries/s", "cores": int(used), "kind": "oracle",
               "sample": f"first {ns} of the {nq} queries of {cfg.name}/{args.noise}, whole pipeline, one query per thread",
               "seconds": round(dt_cpu, 2), "id_agreement_with_gpu": agree}
        log(f"[bench] CPU oracle: {ns} queries in {dt_cpu:.2f}s on {used} threads; id agreement with GPU {agree:.4f}")

    pl.plaid_index_free(idx)
    line = {
        "metric": "queries_per_sec", "value": round(qps, 2), "unit": "queries/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} ({args.noise} noise): C={cfg.C} centroids, P={cfg.P} passages, N={w.N} "
                               f"embeddings, {cfg.nbits}-bit residuals, {nq} queries x 32 x 128",
                   "nprobe": cfg.nprobe, "t_cs": cfg.t_cs, "ndocs": cfg.ndocs, "k": cfg.k,
                   "queries_per_step": nq, "index_generated_on": "cuda"},
        "latency_batch1_ms": {"p50": round(float(np.percentile(lat, 50)), 4), "p99": round(float(np.percentile(lat, 99)), 4),
                              "mean": round(float(lat.mean()), 4), "queries": int(nlat), "trials": 3, "host_enqueue_p50": round(float(np.percentile(enq, 50)), 4),
                              "qps": round(1e3 / float(lat.mean()), 1) if nlat else None},
        "stage_ms_per_step": {s: round(v, 4) for s, v in stage_ms.items()},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
