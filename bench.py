#!/usr/bin/env python3
"""Benchmark of the batched IVF top-k retrieval path on one MI355X.

A step is one pass of the whole hot path (coarse quantisation, probe selection,
regrouping, list scan, k-selection) over one batch of synthetic queries, with the
index and the queries already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5] [--others C1,C2,C3,C4]

The default workload is C5 (100 M x 768 fp16, nq 128, nprobe 128, k 100): the
configuration the benchmark's target is quoted on, and it fits one GPU.  The other
configurations are measured after it in the same run and reported under
`other_configs` of the same line.

Timing definitions (all reported; `value` is the first):
  queued        K searches issued back to back with ivf_search_queued (stages of
                neighbouring searches overlap), one synchronisation at the end, mean
  plain_queued  the same with ivf_search (each search a chain on one stream), mean
  single        K searches, each followed by a stream synchronisation, median
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per k_scan launch from hardware counters (FETCH_SIZE x 2.000 + WRITE_SIZE, both
# scaled against the library's plain copy kernel), and the summary each comes from.
# Workloads that have not been counted report null.
TRAFFIC_BYTES = {"C5": 1.66754e7 * 2.000 * 1024 + 8283.61 * 1024,
                 "C5-int8": 8.38864e6 * 2.000 * 1024 + 5432.68 * 1024}
TRAFFIC_SOURCE = {"C5": "profiles/k_scan_C5_pmc_traffic.md",
                  "C5-int8": "profiles/k_scan_C5_int8_trace_and_traffic.md"}


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def cpu_baseline(lw, q, got_ids, got_scores, nprobe, k, target_seconds):
    """The CPU oracle, as it stands, timed on the host cores for a bounded sample of
    the same batch; the sampled rows are also compared with the GPU's.  The oracle reads
    lists regenerated from the seeded recipe, never the library's own storage."""
    import numpy as np
    from oracle import check as CK
    from oracle import ivf_oracle as O
    from paper_2504_15302_amd.loader import host_lists

    w = lw.w

    def run(rows):
        qs = q[rows]
        t0 = time.perf_counter()
        cs = O.coarse(qs, lw.centroids)
        pr = O.probe_select(cs, nprobe)
        t_coarse = time.perf_counter() - t0
        vec, ids, off, cmap = host_lists(lw, pr.ravel())
        cpr = np.vectorize(cmap.get)(pr).astype(np.int32)
        t1 = time.perf_counter()
        oi, os_ = O.scan_select(vec, ids, off, qs, cpr, k + 8)
        t_scan = time.perf_counter() - t1
        CK.check_topk(got_ids[rows], got_scores[rows], oi, os_, k, CK.SCORE_REL[w.storage])
        return t_coarse + t_scan

    # the oracle spreads queries over its threads, so the pilot uses one query per thread
    threads = O.threads()
    npilot = min(q.shape[0], threads)
    t_pilot = run(list(range(npilot)))
    waves = max(1, int(target_seconds / max(t_pilot, 1e-6)))
    n = min(q.shape[0], npilot * waves)
    rows = list(range(n))
    t = run(rows) if n > npilot else t_pilot
    return {"value": n / t, "unit": "queries/s", "cores": O.threads(), "kind": "oracle",
            "sample": f"first {n} of the {q.shape[0]} queries of batch 0 (fp64 coarse + probe "
                      f"selection + exact scan of their probed lists + sort), search only, "
                      f"lists regenerated from the seed into host RAM beforehand; {t:.1f} s; rows checked "
                      f"against the GPU result",
            "seconds": t}


def budget_change(idx, w, lw, q_dev, out_ids, out_scores, first, log):
    """Times a change of residency between the placement at hand and a quarter of the lists
    HBM-resident, both ways: with the blocking call, and in the background with searches
    issued back to back meanwhile (each compared with the rows from before the change)."""
    import numpy as np
    import torch
    lens = np.diff(lw.offsets)
    order = np.lexsort((np.arange(w.nlist), -lens))
    keep = order[: w.nlist // 4]
    quarter = int(((lens[keep] + 63) // 64).sum()) * 64 * w.row_bytes
    start = idx.info().device_list_bytes
    nb = len(q_dev)

    def searches_per_s(n=8):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            idx.search(q_dev[i % nb], w.nprobe, w.k, out_ids, out_scores)
        torch.cuda.synchronize()
        return n / (time.perf_counter() - t0)

    out = {"quarter_budget_bytes": quarter, "start_device_bytes": int(start), "legs": []}
    for mode in ("blocking", "background"):
        for target, name in ((quarter, "shrink to a quarter of the lists"), (start, "grow back")):
            steady_before = searches_per_s()
            t0 = time.perf_counter()
            n_search = 0
            ok = True
            if mode == "blocking":
                idx.set_device_budget(target)
            else:
                idx.set_device_budget_async(target)
                while idx.budget_progress()[2]:
                    idx.search(q_dev[0], w.nprobe, w.k, out_ids, out_scores)
                    torch.cuda.synchronize()
                    n_search += 1
                    if n_search % 16 == 1:
                        ok = ok and np.array_equal(out_ids.cpu().numpy(), first[0]) and \
                            np.array_equal(out_scores.cpu().numpy(), first[1])
            dt = time.perf_counter() - t0
            info = idx.info()
            moved = info.moved_h2d_bytes + info.moved_d2h_bytes
            leg = {"mode": mode, "change": name, "seconds": dt, "moved_pcie_GB": moved / 1e9,
                   "moved_inside_hbm_GB": info.moved_d2d_bytes / 1e9,
                   "pcie_GBps": moved / 1e9 / dt if dt > 0 else None,
                   "device_pool_GB_after": info.device_pool_bytes / 1e9,
                   "searches_per_s_before": steady_before}
            if mode == "background":
                leg.update({"searches_during": n_search, "searches_per_s_during": n_search / dt if dt > 0 else None,
                            "rows_unchanged": bool(ok)})
            log(f"budget change: {leg}")
            out["legs"].append(leg)
    return out


def workload_label(w):
    return (f"{w.name}: IVF-Flat inner product, N={w.n}, d={w.d}, {w.storage} storage, nlist={w.nlist}, "
            f"nq={w.nq}, nprobe={w.nprobe}, k={w.k}"
            + (f", {w.resident_list_frac:.0%} of lists HBM-resident" if w.resident_list_frac else ""))


def pinned_h2d_rate():
    """The box's own pinned host-to-device copy rate (1 GiB copies): the denominator for
    lists that cross PCIe."""
    import torch
    hsrc = torch.empty(1 << 30, dtype=torch.uint8, pin_memory=True)
    ddst = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    ddst.copy_(hsrc, non_blocking=True)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(4):
        ddst.copy_(hsrc, non_blocking=True)
    e1.record()
    torch.cuda.synchronize()
    return 4 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9


def measure(idx, w, steps, warmup, nb, direct=True, stages=True, components=None, tight=False):
    """All timing definitions for one workload on an index that is already placed.
    Returns (report dict, query batches on host and device, first batch's results, output buffers)."""
    import numpy as np
    import torch
    from paper_2504_15302_amd import workloads as W

    q_host = [W.queries(w, batch=b, components=components, tight=tight) for b in range(nb)]
    q_dev = [torch.from_numpy(q).cuda() for q in q_host]
    out_ids = torch.empty((w.nq, w.k), dtype=torch.int64, device="cuda")
    out_scores = torch.empty((w.nq, w.k), dtype=torch.float32, device="cuda")
    # every search of the measurement goes to one stream of the benchmark's own (the legacy
    # default stream synchronises implicitly with other streams)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()

    idx.set_timing(2)
    stats, firsts = [], []
    for b in range(nb):                      # also the first warm-up of every batch
        idx.search(q_dev[b], w.nprobe, w.k, out_ids, out_scores, stream=stream)
        torch.cuda.synchronize()
        stats.append(idx.last_search_stats())
        firsts.append((out_ids.cpu().numpy().copy(), out_scores.cpu().numpy().copy()))
    first = firsts[0]
    for i in range(max(warmup, 3)):          # every scratch set of the queued path gets its size here
        idx.search_queued(q_dev[i % nb], w.nprobe, w.k, out_ids, out_scores, stream=stream)
    torch.cuda.synchronize()

    # timed region (the headline): K queued searches; only the scan carries HIP events
    idx.set_timing(2)
    t0 = time.perf_counter()
    for i in range(steps):
        idx.search_queued(q_dev[i % nb], w.nprobe, w.k, out_ids, out_scores, stream=stream)
    torch.cuda.synchronize()
    ms_queued = (time.perf_counter() - t0) / steps * 1e3
    last = (out_ids.cpu().numpy(), out_scores.cpu().numpy())
    kept = min(steps, 64)
    scan_ms, scan_bytes, stream_ms = [], [], []
    for back in range(kept):
        step = steps - 1 - back
        ms = idx.stage_ms(back)
        st = stats[step % nb]
        scan_ms.append(ms["scan"])
        stream_ms.append(ms["stream"])
        # with host lists read in place, the one scan launch covers both HBM and PCIe bytes
        scan_bytes.append(st.scan_bytes if direct else st.scan_bytes_resident)
    same = firsts[(steps - 1) % nb]          # the plain search of the batch that the last step used
    rows_ok = bool(np.array_equal(last[0], same[0]) and np.array_equal(last[1], same[1]))

    # the same K steps with plain ivf_search, queued back to back
    for i in range(2):
        idx.search(q_dev[i % nb], w.nprobe, w.k, out_ids, out_scores, stream=stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        idx.search(q_dev[i % nb], w.nprobe, w.k, out_ids, out_scores, stream=stream)
    torch.cuda.synchronize()
    ms_plain = (time.perf_counter() - t0) / steps * 1e3
    plain_scan_ms = float(np.mean([idx.stage_ms(b)["scan"] for b in range(kept)]))
    plain_stream_ms = float(np.mean([idx.stage_ms(b)["stream"] for b in range(kept)]))

    # one search at a time, each synchronised: median
    singles = []
    for i in range(steps):
        t0 = time.perf_counter()
        idx.search(q_dev[i % nb], w.nprobe, w.k, out_ids, out_scores, stream=stream)
        torch.cuda.synchronize()
        singles.append((time.perf_counter() - t0) * 1e3)
    ms_single = float(np.median(singles))

    avg_scan_ms = float(np.mean(scan_ms))
    avg_scan_bytes = float(np.mean(scan_bytes))
    achieved = avg_scan_bytes / (avg_scan_ms * 1e-3) / 1e9 if avg_scan_ms > 0 else 0.0
    rep = {
        "queries_per_s": w.nq / (ms_queued * 1e-3),
        "ms_per_step": ms_queued,
        "timing": {"queued_ms": ms_queued, "plain_queued_ms": ms_plain, "single_sync_median_ms": ms_single,
                   "queries_per_s_plain_queued": w.nq / (ms_plain * 1e-3),
                   "queries_per_s_single": w.nq / (ms_single * 1e-3),
                   "rows_of_last_step_equal_plain_search": rows_ok},
        "scan": {"GBps": achieved, "frac_of_hbm_peak": achieved / HBM_PEAK_GBS, "ms_per_launch": avg_scan_ms,
                 "bytes_per_launch": avg_scan_bytes, "launches_timed": kept,
                 "ms_per_launch_plain_search": plain_scan_ms,
                 "GBps_plain_search": avg_scan_bytes / (plain_scan_ms * 1e-3) / 1e9 if plain_scan_ms > 0 else None},
        "unique_lists_per_batch": int(stats[0].unique_lists),
        "pairs_per_batch": int(stats[0].pairs),
        "queries_per_probed_list": stats[0].pairs / max(1, stats[0].unique_lists),
        # what the scan kernel asks memory for: one read of a block per group of up to four
        # queries that probe its list (equal to the algorithmic bytes when no list has more)
        "scan_requested_bytes_per_batch": int(stats[0].scan_items) * 64 * w.row_bytes,
        "scan_bytes_per_batch": int(stats[0].scan_bytes),
        "scan_bytes_streamed_per_batch": int(stats[0].scan_bytes_streamed),
        "_stream_ms": float(np.mean(stream_ms)),
        "_plain_stream_ms": plain_stream_ms,
        "_streamed": float(np.mean([stats[(steps - 1 - b) % nb].scan_bytes_streamed for b in range(kept)])),
    }
    if stages:
        # every stage, on a few more plain searches (seven event records per search)
        idx.set_timing(1)
        extra = min(steps, 8)
        for i in range(extra):
            idx.search(q_dev[i % nb], w.nprobe, w.k, out_ids, out_scores, stream=stream)
        torch.cuda.synchronize()
        stage_sum = {}
        for back in range(extra):
            for name, v in idx.stage_ms(back).items():
                stage_sum[name] = stage_sum.get(name, 0.0) + v
        rep["stages_ms"] = {name: v / extra for name, v in stage_sum.items()}
        rep["stages_note"] = (f"plain ivf_search with events around every stage, {extra} searches after the timed "
                              "region (the events add ~18 us per search)")
        c = rep["stages_ms"]["coarse"]
        rep["coarse_tflops_fp32"] = 2.0 * w.nq * w.nlist * w.d / (c * 1e-3) / 1e12 if c > 0 else 0.0
    idx.set_timing(0)
    return rep, q_host, q_dev, first, (out_ids, out_scores)


def worker_report(idx, w, q_host, first, log, batches=24):
    """The retrieval worker over the same index (single requests in, batches formed by the
    worker with the batch-size rule, rows out by ticket): requests per second under a backlog
    of `batches` x nq requests, host queries and results in pinned memory (PCIe-inclusive)."""
    import numpy as np
    from paper_2504_15302_amd import ivf
    nb = len(q_host)
    wk = ivf.Worker(idx, w.nprobe, w.k, w.nq)
    try:
        for t in [wk.submit(q_host[0][i]) for i in range(w.nq)]:          # warm-up: one batch
            wk.wait(t)
        n = batches * w.nq
        t0 = time.perf_counter()
        tickets = [wk.submit(q_host[(i // w.nq) % nb][i % w.nq]) for i in range(n)]
        got = [wk.wait(t) for t in tickets]
        dt = time.perf_counter() - t0
        st = wk.stats()
        rows_ok = all(np.array_equal(got[i][0], first[0][i]) and np.array_equal(got[i][1], first[1][i])
                      for i in range(w.nq))                              # the first nq requests are batch 0
    finally:
        wk.stop()
    log(f"worker: {n / dt:.0f} queries/s over {n} single requests")
    return {"queries_per_s": n / dt, "requests": n, "batches_formed": int(st.batches) - 1,
            "largest_batch": int(st.largest_batch), "rows_of_batch_0_equal_plain_search": bool(rows_ok),
            "note": "ivf_worker_*: requests submitted one by one from the host, queries and results in pinned "
                    "host memory, batches formed by the worker; PCIe-inclusive"}


def pcie_report(rep, direct, h2d):
    streamed = rep["_streamed"]
    # direct reads happen inside the scan; staged copies are a stage of their own (searches
    # of the staged mode always run on one stream: the figure of the plain-search region)
    t_stream = rep["scan"]["ms_per_launch"] if direct else rep["_plain_stream_ms"]
    rate = streamed / 1e9 / (t_stream * 1e-3) if t_stream > 0 else None
    return {"streamed_GB_per_batch": streamed / 1e9, "GBps_over_stream_stage": rate,
            "stream_stage_ms": t_stream,
            "mode": "scan reads pinned host memory directly" if direct else "hipMemcpyAsync to staging on a side stream",
            "pinned_h2d_copy_GBps_1GiB": h2d, "frac_of_h2d_copy": rate / h2d if rate else None}


def measure_others(others, args, nb, log):
    """C1..C4 beside the headline workload: the same measurement on indexes of their own, built
    and released one after the other (C4 is C3's index under a budget)."""
    import torch
    from paper_2504_15302_amd import workloads as W
    from paper_2504_15302_amd.loader import load_workload
    out = {}
    built = {}
    h2d = None
    for name in others:
        ow = W.CONFIGS[name]
        key = (ow.n, ow.d, ow.nlist, ow.storage, ow.seed)
        if key not in built:
            for olw in built.values():
                olw.index.close()
            built.clear()
            torch.cuda.empty_cache()
            log(f"building {ow.name}: {ow.n} x {ow.d} {ow.storage}, nlist {ow.nlist}")
            built[key] = load_workload(ow, groups_per_chunk=32, log=log)
        olw = built[key]
        if ow.resident_list_frac is not None:
            set_quarter_budget(olw.index, ow, olw)
        else:
            olw.index.set_device_budget(2**62)
        orep, _, _, _, _ = measure(olw.index, ow, args.steps, args.warmup, nb, True)
        entry = {"workload": workload_label(ow)}
        entry.update(public(orep))
        if orep["scan_bytes_streamed_per_batch"] > 0:
            h2d = h2d or pinned_h2d_rate()
            entry["pcie"] = pcie_report(orep, True, h2d)
            entry["scan"]["note"] = "PCIe-bound: see pcie; the HBM fraction is not meaningful here"
        out[name] = entry
        log(f"{name}: {entry['queries_per_s']:.0f} queries/s queued, scan {entry['scan']['GBps']:.0f} GB/s")
    for olw in built.values():
        olw.index.close()
    built.clear()
    torch.cuda.empty_cache()
    return out


def set_quarter_budget(idx, w, lw):
    import numpy as np
    lens = np.diff(lw.offsets)
    order = np.lexsort((np.arange(w.nlist), -lens))
    keep = order[: int(w.nlist * w.resident_list_frac)]
    budget = int(((lens[keep] + 63) // 64).sum()) * 64 * w.row_bytes
    idx.set_device_budget(budget)
    log(f"device budget {budget / 2**30:.2f} GiB: {idx.info().resident_lists} lists resident")


def public(rep):
    return {k: v for k, v in rep.items() if not k.startswith("_")}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C5")
    ap.add_argument("--others", default=None,
                    help="comma-separated workloads measured afterwards and reported under other_configs "
                         "(default: C1,C2,C3,C4 when the workload is C5 and no experiment flag is given; 'none' skips)")
    ap.add_argument("--batches", type=int, default=4, help="query batches rotated between steps")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="0 skips the CPU baseline")
    ap.add_argument("--option", action="append", default=[], help="library option name=value")
    ap.add_argument("--n", type=int, default=0, help="override the number of vectors (experiments only)")
    ap.add_argument("--uniform-list-len", type=int, default=0,
                    help="experiment: every list of the workload exactly this many vectors long (n = nlist x length)")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="also launch the library's plain copy kernel over this many MiB (reference "
                         "point for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="also time ivf_search at batch sizes 8..nq, fit T(B) = a*B^c and report the "
                         "backlog-aware batch-size choice (ivf_sched_*)")
    ap.add_argument("--k-sweep", action="store_true",
                    help="also time the search for k = 1..10 (the paper's range of retrieved chunks)")
    ap.add_argument("--budget-change", action="store_true",
                    help="also time a change of the device budget (to a quarter of the lists and back), "
                         "blocking and in the background while searches go on")
    ap.add_argument("--skew-components", type=int, default=0,
                    help="draw every query batch from this many mixture components only (about nq/m queries "
                         "then probe the same lists); 0 = the benchmark's uniform batches")
    ap.add_argument("--skew-tight", action="store_true",
                    help="with --skew-components: the queries of a component are near copies of one another, "
                         "so that all their probed lists are shared, not only the home list")
    ap.add_argument("--read-ceiling-gib", type=int, default=24,
                    help="size of the plain streaming-read measurement (0 skips it)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported, use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2504_15302_amd import workloads as W
    from paper_2504_15302_amd.loader import load_workload

    experiment = bool(args.option or args.n or args.batch_sweep or args.k_sweep or args.budget_change
                      or args.calibrate_copy_mib or args.skew_components or args.uniform_list_len)
    if args.others is None:
        others = ["C1", "C2", "C3", "C4"] if (args.workload == "C5" and not experiment) else []
    else:
        others = [o for o in args.others.split(",") if o and o != "none"]

    # The small configurations first: where the driver places an index decides about 5 % of
    # their scan rate, and after the 150 GB of the headline workload have been allocated and
    # freed the placement is the worse one.
    other_results = measure_others(others, args, max(1, args.batches), log) if others else None

    w = W.CONFIGS[args.workload]
    if args.n:
        w = W.scaled(w, n=args.n, name=w.name + f"-n{args.n}")
    if args.uniform_list_len:
        w = W.scaled(w, n=w.nlist * args.uniform_list_len, uniform_lists=True, name=w.name + f"-len{args.uniform_list_len}")
    log(f"building {w.name}: {w.n} x {w.d} {w.storage}, nlist {w.nlist}")
    lw = load_workload(w, groups_per_chunk=32, log=log)
    idx = lw.index
    log(f"index ready in {lw.seconds:.1f}s")
    for opt in args.option:
        name, val = opt.split("=")
        idx.set_option(name, int(val))
    if w.resident_list_frac is not None:
        set_quarter_budget(idx, w, lw)
    direct = not any(o.replace(" ", "") == "host_direct=0" for o in args.option)   # library default: direct
    nb = max(1, args.batches)

    if args.calibrate_copy_mib:
        nbytes = args.calibrate_copy_mib << 20
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            idx.debug_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    read_ceiling = None
    if args.read_ceiling_gib:
        # plain read kernel with the scan's access pattern: what this machine can deliver
        nbytes = (args.read_ceiling_gib << 30) // 98304 * 98304
        try:
            src = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
            sink = torch.zeros(16, dtype=torch.int32, device="cuda")
            idx.debug_read(src, sink)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                idx.debug_read(src, sink)
            e1.record()
            torch.cuda.synchronize()
            read_ceiling = 5 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
            del src, sink
        except torch.OutOfMemoryError:
            log("no room for the read-ceiling buffer; skipped")
        torch.cuda.empty_cache()

    rep, q_host, q_dev, first, (out_ids, out_scores) = measure(idx, w, args.steps, args.warmup, nb, direct,
                                                               components=args.skew_components or None,
                                                               tight=args.skew_tight)
    sc = rep["scan"]
    result = {
        "metric": "queries/sec and list-scan HBM GB/s (% of peak), batched IVF top-k search",
        "value": rep["queries_per_s"], "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rep["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 accumulate over " + {"fp32": "f32", "fp16": "f16", "int8": "i8 codes + f32 scale",
                                           "pq8": "product-quantisation codes (u8) with f32 tables over"}[w.storage] + " storage",
        "data": "synthetic (seeded Gaussian mixture, generated on the GPU; random-init, no dataset)",
        "config": {"workload": workload_label(w),
                   "query_batches_rotated": nb,
                   "unique_lists_per_batch": rep["unique_lists_per_batch"],
                   "scan_bytes_per_batch": rep["scan_bytes_per_batch"],
                   "scan_bytes_streamed_per_batch": rep["scan_bytes_streamed_per_batch"],
                   "pairs_per_batch": rep["pairs_per_batch"],
                   "queries_per_probed_list": rep["queries_per_probed_list"],
                   "scan_requested_bytes_per_batch": rep["scan_requested_bytes_per_batch"],
                   "skew_components": args.skew_components or None, "skew_tight": bool(args.skew_tight),
                   "step": "one ivf_search_queued call; K calls issued back to back, one synchronisation at the end"},
        "roofline": {"bound": "hbm", "kernel": "k_pq_tables + k_pq_scan (LDS-gather-bound: the HBM figure is context only)"
                     if w.storage == "pq8" else "k_scan / k_scan_split (scan of the probed lists)",
                     "achieved": sc["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": sc["GBps"] / HBM_PEAK_GBS,
                     "traffic": TRAFFIC_BYTES.get(w.name) if not experiment else None,
                     "traffic_source": TRAFFIC_SOURCE[w.name] + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, "
                                       "bytes per launch; a constant from that summary, not counted in this run)"
                     if (w.name in TRAFFIC_BYTES and not experiment) else None,
                     "bytes_per_launch": sc["bytes_per_launch"], "ms_per_launch": sc["ms_per_launch"],
                     "launches_timed": sc["launches_timed"],
                     "ms_per_launch_plain_search": sc["ms_per_launch_plain_search"],
                     "achieved_plain_search": sc["GBps_plain_search"],
                     "plain_read_same_pattern_GBps": read_ceiling},
        "timing": rep["timing"],
        "stages_ms": rep.get("stages_ms"),
        "stages_note": rep.get("stages_note"),
        "coarse_tflops_fp32": rep.get("coarse_tflops_fp32"),
        "index_build_seconds": lw.seconds,
    }
    if rep["scan_bytes_streamed_per_batch"] > 0:
        result["roofline"]["note"] = ("this workload is PCIe-bound: most probed bytes come from pinned host memory; "
                                      "see the pcie object, the HBM figure is not meaningful here")
        result["pcie"] = pcie_report(rep, direct, pinned_h2d_rate())
    if args.batch_sweep:
        from paper_2504_15302_amd import ivf as ivf_mod
        sizes = [b for b in (8, 16, 32, 64, 128, 256) if b <= w.nq]
        times = []
        for b in sizes:
            qs = [q[:b].contiguous() for q in q_dev]
            oi, os_ = out_ids[:b].contiguous(), out_scores[:b].contiguous()
            for i in range(2):
                idx.search(qs[i % nb], w.nprobe, w.k, oi, os_)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(8):
                idx.search(qs[i % nb], w.nprobe, w.k, oi, os_)
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t0) / 8 * 1e3)
        a, c = ivf_mod.sched_fit(sizes, times)
        best, lat = ivf_mod.sched_choose(a, c, w.nq, sizes)
        result["batch_scheduling"] = {
            "batch_sizes": sizes, "ms_per_search": times, "fit_a_ms": a, "fit_c": c,
            "queue": w.nq, "chosen_batch": best, "avg_latency_ms_from_queue_start": lat,
            "single_batch_beats_two": ivf_mod.sched_single_batch_is_best(c, 2)}
    if args.k_sweep:
        sweep = {}
        for k in range(1, 11):
            oi = torch.empty((w.nq, k), dtype=torch.int64, device="cuda")
            os_ = torch.empty((w.nq, k), dtype=torch.float32, device="cuda")
            for i in range(2):
                idx.search(q_dev[i % nb], w.nprobe, k, oi, os_)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(8):
                idx.search(q_dev[i % nb], w.nprobe, k, oi, os_)
            torch.cuda.synchronize()
            sweep[str(k)] = w.nq / ((time.perf_counter() - t0) / 8)
        result["k_sweep_queries_per_s"] = sweep
    if args.budget_change:
        result["budget_change"] = budget_change(idx, w, lw, q_dev, out_ids, out_scores, first, log)
    if not experiment and direct:
        result["worker"] = worker_report(idx, w, q_host, first, log)
    if args.cpu_seconds > 0:
        log("timing the CPU oracle on a sample of batch 0")
        result["cpu_baseline"] = cpu_baseline(lw, q_host[0], first[0], first[1], w.nprobe, w.k, args.cpu_seconds)
    else:
        result["cpu_baseline"] = None

    if other_results is not None:
        result["other_configs"] = other_results
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
