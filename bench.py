#!/usr/bin/env python3
"""Benchmark of the IVFPQ search path on one MI355X.

A "step" is one pass of the whole hot path -- probe selection, lookup-table build, PQ-code scan,
top-k -- over one batch of 10,000 synthetic queries that already sits in HBM.  The default workload is
the size of the paper's experiments (Sec. III): 10^8 integer-valued 128-d vectors in 50,000 clusters,
32 sub-spaces of 8-bit codes (32-byte codes, 3.2 GB), 64 probes, k = 100; inputs are seeded and synthetic.

Prints ONE JSON line: queries/s of the headline table dtype (median of the timed steps), with
  roofline     -- the dominant kernel (the scan over the probes other than the nearest one) against the unit
                  that binds it, the LDS: table lookups per second of the run that makes every lookup of
                  Eq. (1), timed live with HIP events on the stream the kernel runs on, against a
                  conflict-free LDS (256 CUs x 32 lanes x 2.4 GHz); the algorithmic PQ-code bytes against
                  the HBM peak and this box's plain streaming-read rate are secondary keys;
  cpu_baseline -- the CPU oracle timed on a bounded sample of the same queries and index (best of 3).
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0                   # MI355X published HBM3E bandwidth, GB/s
LDS_PEAK_LOOKUPS = 256 * 32 * 2.4e9     # conflict-free wave-wide LDS reads: 32 lanes per clock and CU

# HBM traffic of the dominant kernel per launch, bytes.  NOT measured by this process: recorded from two
# rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter reads for a plain
# copy of known size); the summary file under profiles/ holds the command and the raw figures.
PROFILED_TRAFFIC = {
    # (workload, table dtype): (bytes per launch of the dominant kernel, early exit off; summary file)
    ("intgrid_100m_p8", "e5m3"): (4658953375, "profiles/scan_kernel_intgrid_100m_p8_e5m3_hbm_traffic.txt"),
    ("unitnorm_10m", "e5m3"): (745721453, "profiles/scan_kernel_unitnorm_10m_e5m3_hbm_traffic.txt"),
    ("intgrid_1m", "e5m3"): (300197912, "profiles/scan_kernel_intgrid_1m_e5m3_hbm_traffic.txt"),
    ("intgrid_100m_p4", "e5m3"): (5692997573, "profiles/scan_kernel_intgrid_100m_p4_e5m3_hbm_traffic.txt"),
}


# Which unit the dominant kernel keeps busiest.  NOT measured by this process either: busy shares of the vector
# ALU and of the LDS from a recorded rocprofv3 --pmc run of the same command (early exit off).
PROFILED_UNITS = {
    ("intgrid_100m_p8", "e5m3"): ({"valu_busy": 0.94, "lds_busy": 0.56}, "profiles/scan_kernel_intgrid_100m_p8_lds_counters.txt"),
    ("unitnorm_10m", "e5m3"): ({"valu_busy": 0.90, "lds_busy": 0.68}, "profiles/scan_kernel_unitnorm_10m_lds_counters.txt"),
    ("intgrid_1m", "e5m3"): ({"valu_busy": 0.95, "lds_busy": 0.92}, "profiles/scan_kernel_intgrid_1m_lds_counters.txt"),
    ("intgrid_100m_p4", "e5m3"): ({"valu_busy": 0.97, "lds_busy": 0.28}, "profiles/scan_kernel_intgrid_100m_p4_lds_counters.txt"),
}


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def exact_topk_gpu(data_np, queries_t, k, chunk=1_000_000):
    """Harness-side ground truth: exact k nearest by float64 distances, chunked over the data."""
    import torch
    q = queries_t.double()
    qn = (q * q).sum(1, keepdim=True)
    best_d = torch.full((q.shape[0], k), float("inf"), dtype=torch.float64, device="cuda")
    best_i = torch.full((q.shape[0], k), -1, dtype=torch.int64, device="cuda")
    for lo in range(0, data_np.shape[0], chunk):
        x = torch.from_numpy(data_np[lo:lo + chunk]).cuda().double()
        d2 = qn + (x * x).sum(1)[None, :] - 2.0 * (q @ x.T)
        dd, ii = torch.topk(d2, min(k, x.shape[0]), dim=1, largest=False)
        cat_d = torch.cat([best_d, dd], 1)
        cat_i = torch.cat([best_i, ii + lo], 1)
        dd, sel = torch.topk(cat_d, k, dim=1, largest=False)
        best_d, best_i = dd, torch.gather(cat_i, 1, sel)
    return best_i, best_d


def tie_aware_recall(found_ids_t, data_np, queries_t, gt_d, k):
    """|V & V_GT| / |V_GT| where a returned vector counts if its true distance does not exceed the
    true k-th distance (integer-valued data have exact distance ties)."""
    import numpy as np
    import torch
    ids = found_ids_t.cpu().numpy()
    q = queries_t.double()
    thr = gt_d[:, k - 1] * (1 + 1e-12)
    safe = np.where(ids >= 0, ids, 0)
    x = torch.from_numpy(data_np[safe.reshape(-1)]).cuda().double().reshape(ids.shape[0], ids.shape[1], -1)
    d2 = ((x - q[:, None, :]) ** 2).sum(-1)
    ok = (d2 <= thr[:, None]) & torch.from_numpy(ids >= 0).cuda()
    return int(ok.sum().item()) / float(ids.shape[0] * k)


def measure_read_ceiling(torch, pkg, gib=4):
    """GB/s of the library's plain streaming-read kernel over a buffer far larger than the caches."""
    buf = torch.empty(gib << 30, dtype=torch.uint8, device="cuda")
    buf.zero_()
    best = 0.0
    for n_wg in (2048, 4096, 8192, 16384):
        pkg.ivfpq_stream_read(buf, n_wg)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            pkg.ivfpq_stream_read(buf, n_wg)
        b.record()
        torch.cuda.synchronize()
        best = max(best, 5 * buf.numel() / (a.elapsed_time(b) * 1e-3) / 1e9)
    del buf
    return best


INDEX_FILES = ("centroids", "codebooks", "list_offsets", "codes", "ids")


def load_cached_index(np, pkg, w, path):
    arrays = [np.load(os.path.join(path, f"{name}.npy"), mmap_mode=None, allow_pickle=False) for name in INDEX_FILES]
    return pkg.Index.ivfpq_index_from_arrays(w.d, w.n_lists, w.pq_dim, w.pq_bits, *arrays), arrays


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="intgrid_100m_p8")
    ap.add_argument("--lut", default="e5m3", choices=["fp32", "fp16", "e5m3", "e4m4"])
    ap.add_argument("--e4m4-bias", type=int, default=None,
                    help="exponent bias of the e4m4 table dtype (default: 1 for the integer-valued sets, 16 for the unit-norm sets)")
    ap.add_argument("--all-luts", action="store_true", help="also time the e4m4 table")
    ap.add_argument("--fp8-variants", action="store_true",
                    help="also time the 8-bit tables with a truncating encode and with a per-table exponent bias "
                         "(reported under by_lut as e5m3+trunc, e5m3+pertable, e4m4+pertable)")
    ap.add_argument("--probe-sweep", default="", metavar="P1,P2,...",
                    help="also time fp32 / fp16 / e5m3 at these numbers of probes (the recall-vs-throughput curves of "
                         "Sec. III, Figs. 5-6, on the synthetic stand-in); reported under by_probes")
    ap.add_argument("--batch-sweep", default="", metavar="N1,N2,...",
                    help="also time batches of these sizes (the first rows of the query set), each call on its own and "
                         "replayed from a captured HIP graph: milliseconds per call; reported under by_batch")
    ap.add_argument("--early-exit", type=int, choices=(0, 1), default=None,
                    help="force the filtered scan's early exit off / on for every run (default: the library's, on)")
    ap.add_argument("--lds-pad", type=int, default=0, metavar="BYTES",
                    help="extra LDS requested per scan workgroup (occupancy experiment: a small table at a large table's footprint)")
    ap.add_argument("--scan-share", type=int, default=0, choices=(0, 1, 2, 4), help="ivfpq_set_tuning(IVFPQ_TUNE_SCAN_SHARE)")
    ap.add_argument("--scan-threads", type=int, default=0, help="ivfpq_set_tuning(IVFPQ_TUNE_SCAN_THREADS)")
    ap.add_argument("--no-full-run", action="store_true",
                    help="skip the extra headline run without early exit (profiling runs: keeps the number of search calls fixed)")
    ap.add_argument("--refine-from", type=int, default=0, metavar="K2",
                    help="also time search with k=K2 followed by ivfpq_refine down to k (exact re-ranking with the "
                         "stored vectors; reported under by_lut as <lut>+refineK2)")
    ap.add_argument("--kmeans-iters", type=int, default=6, help="Lloyd iterations of the (untimed) index build")
    ap.add_argument("--n-probes", type=int, default=None)
    ap.add_argument("--k", type=int, default=None)
    ap.add_argument("--recall-queries", type=int, default=1000)
    ap.add_argument("--no-recall", action="store_true", help="skip the ground truth and recall (profiling runs)")
    ap.add_argument("--cpu-queries", type=int, default=0, help="queries of the CPU oracle sample (0: sized for a few seconds per pass)")
    ap.add_argument("--builder", default="device", choices=["device", "host"],
                    help="index construction (untimed): ivfpq_build_device (HIP kernels) or ivfpq_build_host (CPU)")
    ap.add_argument("--index-cache", default="", metavar="DIR",
                    help="directory with the saved index arrays of this workload: loaded if present (no data generation unless "
                         "recall is wanted, no build), written after the build otherwise.  Profiler runs use it so that the "
                         "profiled process makes a few dozen launches instead of the builder's thousands")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="only run a plain elementwise copy (read BYTES, write BYTES) three times and exit: "
                         "reference for scaling the FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--only-headline", action="store_true", help="skip the other table dtypes (for profiling runs)")
    ap.add_argument("--profile-run", action="store_true",
                    help="for runs under rocprofv3: --only-headline --no-cpu-baseline --no-full-run --no-recall, one stage-timing "
                         "repetition and no streaming-read measurement, so that the process makes warmup + steps + 1 search calls "
                         "and nothing else on the GPU besides the probe lists for the byte count")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.profile_run:
        args.only_headline = args.no_cpu_baseline = args.no_full_run = args.no_recall = True
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; the path shards by query across GPUs with no "
              "communication, and no multi-GPU figure is produced.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth_inputs as si
    import paper_2301_06672_amd as pkg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the search path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    pkg.lib()
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = args.copy_calibration // 4
        x = torch.ones(n, dtype=torch.float32, device="cuda")
        y = torch.empty_like(x)
        for _ in range(3):
            torch.mul(x, 2.0, out=y)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n * 4, "bytes_written": n * 4, "launches": 3}))
        return
    w = si.WORKLOADS[args.workload]
    n_probes = args.n_probes or w.n_probes
    k = args.k or w.k
    lut_ids = {"fp32": pkg.LUT_FP32, "fp16": pkg.LUT_FP16, "e5m3": pkg.LUT_FP8_E5M3, "e4m4": pkg.LUT_FP8_E4M4}
    e4m4_bias = args.e4m4_bias if args.e4m4_bias is not None else (1 if w.kind == "intgrid" else 16)

    cache = args.index_cache
    cached = bool(cache) and all(os.path.exists(os.path.join(cache, f"{n}.npy")) for n in INDEX_FILES)
    want_recall = not args.no_recall
    data = None
    t0 = time.time()
    queries_np = si.queries(w)
    if want_recall or not cached or args.refine_from:
        data = si.dataset(w)
        log(f"generated {w.name}: data {data.shape}, queries {queries_np.shape} in {time.time() - t0:.1f}s")
    t0 = time.time()
    builder = args.builder
    x_dev = None
    if cached:
        idx, (cent, cb, offs, codes, ids_arr) = load_cached_index(np, pkg, w, cache)
        builder = f"cached ({cache})"
        log(f"index loaded from {cache} in {time.time() - t0:.1f}s")
    else:
        if builder == "host":
            idx = pkg.Index.ivfpq_build_host(data, w.n_lists, w.pq_dim, w.pq_bits, args.kmeans_iters, seed=1)
        else:
            x_dev = torch.from_numpy(data).cuda()
            torch.cuda.synchronize()
            t1 = time.time()
            idx = pkg.Index.ivfpq_build_device(x_dev, w.n_lists, w.pq_dim, w.pq_bits, args.kmeans_iters, seed=1)
            log(f"ivfpq_build_device alone (data resident): {time.time() - t1:.2f}s")
            if not args.refine_from:
                x_dev = None
            torch.cuda.empty_cache()
        log(f"index build ({builder}, {args.kmeans_iters} Lloyd iterations) {time.time() - t0:.1f}s")
        cent, cb, offs, codes, ids_arr = idx.ivfpq_index_export()
        if cache:
            os.makedirs(cache, exist_ok=True)
            for name, arr in zip(INDEX_FILES, (cent, cb, offs, codes, ids_arr)):
                np.save(os.path.join(cache, f"{name}.npy"), arr)
            log(f"index saved to {cache}")
    t0 = time.time()
    idx.ivfpq_upload()
    log(f"ivfpq_upload (codes re-laid out on the host, copied to the device) {time.time() - t0:.2f}s")
    idx.ivfpq_set_e4m4_bias(e4m4_bias)
    if args.early_exit is not None:
        idx.ivfpq_set_tuning(pkg.TUNE_EARLY_EXIT, 1 if args.early_exit else -1)
    if args.lds_pad:
        idx.ivfpq_set_tuning(pkg.TUNE_LDS_PAD, args.lds_pad)
    if args.scan_share:
        idx.ivfpq_set_tuning(pkg.TUNE_SCAN_SHARE, args.scan_share)
    if args.scan_threads:
        idx.ivfpq_set_tuning(pkg.TUNE_SCAN_THREADS, args.scan_threads)
    sizes = np.diff(offs)

    q = torch.from_numpy(queries_np).cuda()
    nq = q.shape[0]
    out = (torch.empty((nq, k), dtype=torch.int64, device="cuda"),
           torch.empty((nq, k), dtype=torch.float32, device="cuda"))

    # Exact algorithmic work of one step, from the probe lists: every probed cluster's vectors once per
    # (query, probe).  The cluster scanned unfiltered by the first scan launch is the nearest probe that holds
    # at least k vectors (the nearest one if none does); the dominant kernel scans all the others.
    probes, _ = idx.ivfpq_select_probes(q, n_probes)
    probes_np = probes.cpu().numpy().view(np.uint32)
    probe_sizes = sizes[probes_np]                                   # [nq][n_probes]
    pivot = np.argmax(probe_sizes >= k, axis=1)                      # 0 where no probe holds k vectors
    scanned_vectors = int(probe_sizes.sum())
    nearest_vectors = int(probe_sizes[np.arange(nq), pivot].sum())
    filtered_vectors = scanned_vectors - nearest_vectors
    code_bytes = scanned_vectors * w.code_bytes

    # ground truth for recall on a query subset (harness work, outside the timed region)
    nr = min(args.recall_queries, nq)
    gt_d = None
    if want_recall:
        t0 = time.time()
        _, gt_d = exact_topk_gpu(data, q[:nr], k)
        log(f"exact ground truth of {nr} queries in {time.time() - t0:.1f}s")

    def run(lut_name, steps, warmup, n_probes=n_probes):
        base, _, variant = lut_name.partition("+")
        lut = lut_ids[base]
        if base in ("e5m3", "e4m4"):
            idx.ivfpq_set_fp8_encoding(lut, 15 if base == "e5m3" else e4m4_bias,
                                       pkg.ROUND_TRUNCATE if variant == "trunc" else pkg.ROUND_NEAREST,
                                       variant == "pertable")
        for _ in range(warmup):
            idx.ivfpq_search(q, n_probes, k, lut, out=out)
        # exactly `steps` steps between two synchronisations; every step also sits between two events recorded
        # on the search stream, whose median is the figure reported (the mean over the bracket is kept beside it)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        torch.cuda.synchronize()
        t = time.perf_counter()
        marks[0].record()
        for i in range(steps):
            idx.ivfpq_search(q, n_probes, k, lut, out=out)
            marks[i + 1].record()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
        med = statistics.median(per_step)
        # stage and kernel times of further (untimed) steps, from HIP events the library records on the search
        # stream around its launches: median over the repetitions
        idx.ivfpq_set_stage_timing(True)
        reps = 1 if args.profile_run else 5
        seen = {}
        for _ in range(reps):
            idx.ivfpq_search(q, n_probes, k, lut, out=out)
            torch.cuda.synchronize()
            for name, v in idx.ivfpq_stage_times_ms().items():
                seen.setdefault(name, []).append(v)
        idx.ivfpq_set_stage_timing(False)
        stage = {name: statistics.median(v) for name, v in seen.items()}
        rec = tie_aware_recall(out[0][:nr], data, q[:nr], gt_d, k) if want_recall else None
        return {"qps": nq / (med * 1e-3), "ms_per_step": med, "ms_per_step_mean": 1e3 * dt / steps,
                "ms_per_step_min": min(per_step), "ms_per_step_max": max(per_step), "recall": rec, "stage_ms": stage}

    def fmt(r):
        rec = "n/a" if r["recall"] is None else f"{r['recall']:.4f}"
        return (f"{r['qps']:.0f} q/s, median {r['ms_per_step']:.3f} ms/step (mean {r['ms_per_step_mean']:.3f}, "
                f"min {r['ms_per_step_min']:.3f}, max {r['ms_per_step_max']:.3f}), recall@{k}={rec}, "
                f"stages {{{', '.join(f'{a}: {b:.3f}' for a, b in r['stage_ms'].items())}}}")

    results = {}
    order = [args.lut] if args.only_headline else ["fp32", "fp16", "e5m3"]
    if not args.only_headline and (args.all_luts or args.lut == "e4m4"):
        order.append("e4m4")
    if args.fp8_variants and not args.only_headline:
        order += ["e5m3+trunc", "e5m3+pertable", "e4m4+pertable"]
    other_steps = max(10, args.steps // 2)
    for name in order:
        results[name] = run(name, args.steps if name == args.lut else other_steps, args.warmup)
        log(f"lut={name}: {fmt(results[name])}")
    # the same headline run with the filtered scan adding up every sub-space of every vector (no exit once a
    # group's partial sums are all over the bound): same results, the rate a kernel without that test has, and
    # the run whose lookup count is known exactly (what the roofline fraction is taken from)
    if args.no_full_run or args.early_exit == 0:
        full = results[args.lut]
        full_is_exact = args.early_exit == 0
    else:
        idx.ivfpq_set_tuning(pkg.TUNE_EARLY_EXIT, -1)
        full = run(args.lut, other_steps, 1)
        idx.ivfpq_set_tuning(pkg.TUNE_EARLY_EXIT, 0 if args.early_exit is None else 1)
        full_is_exact = True
        log(f"lut={args.lut} without early exit: {fmt(full)}")
    by_probes = {}
    for P in [int(v) for v in args.probe_sweep.split(",") if v]:
        if P < 1 or P > min(w.n_lists, pkg.MAX_PROBES):
            continue
        by_probes[P] = {}
        for name in ("fp32", "fp16", "e5m3"):
            r = run(name, other_steps, 1, n_probes=P)
            by_probes[P][name] = {"qps": round(r["qps"], 1), "recall": None if r["recall"] is None else round(r["recall"], 4)}
        log(f"n_probes={P}: " + "  ".join(f"{n} {v['qps']:.0f} q/s @ {v['recall']}" for n, v in by_probes[P].items()))
    by_batch = {}
    for nb in [int(v) for v in args.batch_sweep.split(",") if v]:
        nb = max(1, min(nb, nq))
        lut = lut_ids[args.lut]
        if args.lut in ("e5m3", "e4m4"):
            idx.ivfpq_set_fp8_encoding(lut, 15 if args.lut == "e5m3" else e4m4_bias)
        qb = q[:nb].contiguous()
        ob = (torch.empty((nb, k), dtype=torch.int64, device="cuda"), torch.empty((nb, k), dtype=torch.float32, device="cuda"))
        reps = 50 if nb <= 1024 else 10
        for _ in range(3):
            idx.ivfpq_search(qb, n_probes, k, lut, out=ob)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            idx.ivfpq_search(qb, n_probes, k, lut, out=ob)
        torch.cuda.synchronize()
        eager_ms = 1e3 * (time.perf_counter() - t) / reps
        want = ob[0].clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            idx.ivfpq_search(qb, n_probes, k, lut, out=ob)
        g.replay()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = 1e3 * (time.perf_counter() - t) / reps
        same = bool(torch.equal(ob[0], want))
        del g
        by_batch[nb] = {"eager_ms": round(eager_ms, 4), "graph_ms": round(graph_ms, 4), "graph_matches_eager": same}
        log(f"batch {nb}: {eager_ms:.3f} ms per call, {graph_ms:.3f} ms replayed from a HIP graph (same ids: {same})")
    if args.refine_from:
        # search with a longer result list, then re-rank it exactly with the stored vectors
        k2 = args.refine_from
        if x_dev is None:
            x_dev = torch.from_numpy(data).cuda()
        lut = lut_ids[args.lut]
        if args.lut in ("e5m3", "e4m4"):
            idx.ivfpq_set_fp8_encoding(lut, 15 if args.lut == "e5m3" else e4m4_bias)
        out2 = (torch.empty((nq, k2), dtype=torch.int64, device="cuda"), torch.empty((nq, k2), dtype=torch.float32, device="cuda"))

        def one():
            idx.ivfpq_search(q, n_probes, k2, lut, out=out2)
            return pkg.ivfpq_refine(x_dev, q, out2[0], k)
        for _ in range(args.warmup):
            one()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(args.steps):
            rid, _ = one()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        name = f"{args.lut}+refine{k2}"
        results[name] = {"qps": nq * args.steps / dt, "ms_per_step": 1e3 * dt / args.steps,
                         "recall": tie_aware_recall(rid[:nr], data, q[:nr], gt_d, k) if want_recall else None, "stage_ms": {}}
        log(f"lut={name}: {results[name]['qps']:.0f} q/s, {results[name]['ms_per_step']:.3f} ms/step, recall@{k}={results[name]['recall']}")
    head = results[args.lut]

    ws_bytes = idx.ivfpq_search_workspace_bytes(nq, n_probes, k, lut_ids[args.lut])
    ceiling = 0.0 if args.profile_run else measure_read_ceiling(torch, pkg)
    log(f"plain streaming read on this box: {ceiling:.0f} GB/s")
    # The dominant kernel: the scan over every probe but the one scanned unfiltered (one launch per step when the
    # batch is one query tile).  Its units are known exactly for the run without early exit.
    kern_ms_full = full["stage_ms"]["scan_filtered_kernel"]
    kern_ms = head["stage_ms"]["scan_filtered_kernel"]
    lookups = filtered_vectors * w.pq_dim
    kern_bytes = filtered_vectors * w.code_bytes
    traffic = PROFILED_TRAFFIC.get((w.name, args.lut))
    roofline = None
    if kern_ms_full > 0:
        rate = lookups / (kern_ms_full * 1e-3)
        roofline = {
            "bound": "lds",
            "kernel": idx.ivfpq_scan_kernel_info(lut_ids[args.lut]),
            "achieved": round(rate, 1), "peak": LDS_PEAK_LOOKUPS, "unit": "table lookups/s",
            "frac": round(rate / LDS_PEAK_LOOKUPS, 4),
            "lookups_per_step": lookups, "kernel_ms_per_step": round(kern_ms_full, 4),
            "launches_per_step": "one per query tile; one tile at this workload unless the workspace limit is lowered",
            "run": "every lookup of Eq. (1) made (early exit off)" if full_is_exact else
                   "default run: the early exit skips an unknown share of the lookups counted here, so achieved and frac are upper bounds",
            "recorded_unit_shares": None if (w.name, args.lut) not in PROFILED_UNITS else
                dict(PROFILED_UNITS[(w.name, args.lut)][0], source=PROFILED_UNITS[(w.name, args.lut)][1] +
                     ": recorded rocprofv3 --pmc run, not measured by this process; the vector ALU, not the LDS, is what "
                     "the 8-bit table's kernel keeps busiest"),
            "traffic": None if traffic is None else traffic[0],
            "traffic_source": None if traffic is None else
                f"{traffic[1]}: recorded rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, not measured by this process",
            # secondary: the algorithmic PQ-code bytes of the same kernel against HBM (pairs run grouped by cluster,
            # so most of these bytes come from the L2, not from HBM: compare traffic)
            "hbm_algorithmic": {"bytes_per_step": kern_bytes, "achieved": round(kern_bytes / (kern_ms_full * 1e-3) / 1e9, 1),
                                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(kern_bytes / (kern_ms_full * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                "streaming_read_ceiling": round(ceiling, 1)},
            "default_run": {"kernel_ms_per_step": round(kern_ms, 4),
                            "note": "with the early exit (library default) a 64-vector group stops adding once all its partial sums "
                                    "are over the query's bound: same results, fewer lookups made"},
            "whole_scan_stage": {"scanned_vectors_per_step": scanned_vectors, "code_bytes_per_step": code_bytes,
                                 "stage_ms": round(head["stage_ms"]["scan"], 4), "stage_ms_without_early_exit": round(full["stage_ms"]["scan"], 4)},
            "note": "achieved = table lookups the kernel makes per step (vectors of every probed cluster but the one scanned "
                    "unfiltered x sub-spaces, exact from the probe lists) / its launch time (HIP events recorded around the launch "
                    "on the search stream, median of 5); peak = one lookup per lane per clock on a 32-lane LDS pipe per CU "
                    "(256 x 32 x 2.4e9): a 256-entry row of 1-byte entries spans 64 dwords on 32 banks, so 0.5 is the structural limit",
        }

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oidx = oracle.make_index(w.d, w.n_lists, w.pq_dim, w.pq_bits, cent, cb, offs, codes, ids_arr)
        cores = oracle.num_threads()
        # a first small pass sizes the sample so that one pass takes about 4 s; then best of 3
        probe_n = min(nq, 4 * cores)
        t = time.perf_counter()
        _, _, table_stats = oracle.search(oidx, queries_np[:probe_n], n_probes, k, lut_ids[args.lut], e4m4_bias=e4m4_bias,
                                          return_stats=True)
        rate0 = probe_n / (time.perf_counter() - t)
        nc = args.cpu_queries or int(min(nq, max(cores, rate0 * 4.0)))
        nc = max(cores, nc // cores * cores)
        times = []
        for _ in range(3):
            t = time.perf_counter()
            oracle.search(oidx, queries_np[:nc], n_probes, k, lut_ids[args.lut], e4m4_bias=e4m4_bias)
            times.append(time.perf_counter() - t)
        n1 = max(1, nc // cores)                # about the same wall time on one thread
        oracle.set_num_threads(1)
        t = time.perf_counter()
        oracle.search(oidx, queries_np[:n1], n_probes, k, lut_ids[args.lut], e4m4_bias=e4m4_bias)
        dt1 = time.perf_counter() - t
        oracle.set_num_threads(cores)
        cpu = {"value": round(nc / min(times), 1), "unit": "queries/s", "cores": cores, "kind": "oracle",
               "sample": f"first {nc} of the {nq} queries, same index, lut={args.lut}, best of 3 passes "
                         f"({', '.join(f'{x:.1f}' for x in times)} s wall)",
               "one_thread": {"value": round(n1 / dt1, 1), "sample": f"first {n1} queries, one pass, {dt1:.1f}s wall"},
               # entries of the 8-bit tables that fell under the smallest / over the largest code (oracle's count)
               "table_entries": {"sample": f"tables of the first {probe_n} queries",
                                 "entries": int(probe_n) * int(n_probes) * int(w.pq_dim) * (1 << int(w.pq_bits)),
                                 "floored": table_stats["floored"], "saturated": table_stats["saturated"]}}
        log(f"cpu oracle: {cpu}")

    def rnd(x, nd=4):
        return None if x is None else round(x, nd)

    line = {
        "metric": f"queries/sec at recall@{k} ({args.lut} LUT)",
        "value": round(head["qps"], 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(head["ms_per_step"], 4),
        "ms_per_step_stat": "median of the timed steps (HIP events around each step)",
        "ms_per_step_mean": round(head["ms_per_step_mean"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: N={w.n} d={w.d} nq={nq} n_lists={w.n_lists} pq_dim={w.pq_dim} "
                               f"pq_bits={w.pq_bits} n_probes={n_probes} k={k}",
                   "lut_dtype": args.lut, "e4m4_bias": e4m4_bias, "kmeans_iters": args.kmeans_iters, "builder": builder,
                   "workspace_bytes": ws_bytes, "recall_queries": nr if want_recall else 0},
        "recall_at_k": rnd(head["recall"]),
        "by_lut": {n: {"qps": round(r["qps"], 1), "recall": rnd(r["recall"]),
                       "stage_ms": {a: round(b, 4) for a, b in r["stage_ms"].items()}} for n, r in results.items()},
        "without_early_exit": None if full is head else {
            "qps": round(full["qps"], 1), "ms_per_step": round(full["ms_per_step"], 4),
            "stage_ms": {a: round(b, 4) for a, b in full["stage_ms"].items()}},
        "early_exit": "library default (on)" if args.early_exit is None else bool(args.early_exit),
        "roofline": roofline,
        "cpu_baseline": cpu,
        **({"by_probes": by_probes} if by_probes else {}),
        **({"by_batch": by_batch} if by_batch else {}),
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
