"""Benchmark of the IVF search hot path on one MI355X.

Headline workload: single-query retrieval (configs[1] of the benchmark definition) over
1,000,000 x 768 fp32 rows in 1024 k-means lists, nprobe 32, k 10, batch 1, synthetic (seeded
mixture of Gaussians).  A step is one pass of the whole hot path (coarse scoring, top-nprobe
selection, list scan, top-k merge) over one batch of synthetic input: the workload's 256 distinct
queries, each searched on its own through ivf_search_device with query and outputs resident in
HBM.  K steps are timed `--repeats` times; `value` is the median.  The same line carries compact
legs for the other named configurations (configs[2], [3], [4], the paper's resident shape, squared
L2), each with its own roofline, oracle-parity sample and oracle timing.  Prints one JSON line.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes one scan launch moves, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE scaled by a 1 GiB
# copy (profiles/scan_kernel_c2_single_query.md, profiles/batched_scan_kernel_c3_c5.md)
C2_SCAN_TRAFFIC_BYTES = 88561 * 1024 + 1040 * 1024
C3_SCAN_TRAFFIC_BYTES = 5007893 * 2048
C5_SCAN_TRAFFIC_BYTES = 30004499 * 2048
# MFMA utilisation of the batched scan, rocprofv3 --pmc MfmaUtil (profiles/batched_scan_kernel_c3_c5.md)
C3_MFMA_UTIL, C5_MFMA_UTIL = 0.088, 0.103
METRIC = "IVF search queries/sec + achieved HBM GB/s (% of peak) at nprobe sweep, 1 GPU"
NO_EVENTS = False
REPEATS = 5
MIN_REGION_S = 0.05          # a timed region is at least this long


def log(msg):
    print(f"[bench +{time.time() - T_START:.1f}s] {msg}", file=sys.stderr, flush=True)


T_START = time.time()


def med(xs):
    s = sorted(xs)
    return s[len(s) // 2] if len(s) % 2 else 0.5 * (s[len(s) // 2 - 1] + s[len(s) // 2])


def free_gpu():
    import torch
    import workloads as W
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    W.release_pinned_cache()


def rates(units, seconds):
    """median / min / max rate over repeated timed regions of `units` units of work each"""
    r = sorted(units / s for s in seconds)
    return {"median": round(med(r), 1), "min": round(r[0], 1), "max": round(r[-1], 1), "repeats": len(r)}


def compare_sample(gi, gd, oracle_results, rtol):
    """(id mismatches, largest relative distance error) of GPU rows against oracle (ids, scores) pairs"""
    import numpy as np
    bad, rel = 0, 0.0
    for g_i, g_d, (oi, osc) in zip(gi, gd, oracle_results):
        bad += int(not np.array_equal(g_i, oi))
        rel = max(rel, float(np.max(np.abs(g_d.astype(np.float64) - osc) / np.maximum(np.abs(osc), 1e-30))))
    return {"queries": len(oracle_results), "id_mismatches": bad, "near_tie_exemptions": 0 if bad == 0 else None,
            "max_rel_distance_error": rel, "within_tolerance": bool(rel <= rtol)}


def oracle_selected(rows_t, odt, off, cent, x, nprobe, k, metric):
    """Oracle search of one query over a datastore that stays where it is (GPU or pinned host): the
    oracle selects its clusters, those lists are copied into a host datastore in which every other
    list is empty and ids are global row numbers, and the oracle searches that.  Returns
    ((ids, scores), seconds the oracle's search took)."""
    import numpy as np
    import torch
    import oracle as O
    nlist = cent.shape[0]
    sel = np.sort(O.probe(cent, x, nprobe, metric))
    cnt = np.zeros(nlist, dtype=np.int64)
    cnt[sel] = off[sel + 1] - off[sel]
    coff = np.zeros(nlist + 1, dtype=np.int64)
    coff[1:] = np.cumsum(cnt)
    block = torch.cat([rows_t[int(off[c]):int(off[c + 1])] for c in sel]).cpu()
    if block.dtype == torch.bfloat16:
        block = block.view(torch.int16)
    rows = block.numpy()
    if rows.dtype == np.int16:
        rows = rows.view(np.uint16)
    gids = np.concatenate([np.arange(off[c], off[c + 1], dtype=np.int64) for c in sel])
    t = time.perf_counter()
    res = O.search(rows, odt, coff, gids, cent, x, nprobe, k, metric)
    return res, time.perf_counter() - t


# ---------------------------------------------------------------------------------------------------
# configs[1]: single-query retrieval (the headline) and its squared-L2 twin
# ---------------------------------------------------------------------------------------------------
def build_config2(device, n, seed=20970):
    import torch
    import workloads as W
    t0 = time.time()
    ds, q_in, q_out = W.config2_single_query(seed=seed, device=device, n=n)
    torch.cuda.synchronize()
    host = {"rows": ds.rows.cpu().numpy(), "assign": ds.assign.cpu().numpy(), "cent": ds.centroids.cpu().numpy()}
    del ds
    free_gpu()
    return host, q_in, q_out, {"gen_s": round(time.time() - t0, 2)}


def make_index(host, metric):
    import torch
    import paper_2502_20969_amd as P
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    return P.ivf_build_layout(host["rows"], "f32", host["cent"], host["assign"],
                              metric=P.IVF_IP if metric == "ip" else P.IVF_L2,
                              compute_stream=compute, copy_stream=copy)


def run_passes(index, q_dev, ids_dev, dists_dev, nprobe, k, passes, first=0):
    """`passes` passes over the distinct queries, one search per query; returns the wall time"""
    import torch
    nq = q_dev.shape[0]
    views = [(q_dev[j], ids_dev[j], dists_dev[j]) for j in range(nq)]
    search = index.ivf_search_device
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for p in range(passes):
        for q, i_, d_ in views:
            search(q, nprobe, k, i_, d_)
    index.ivf_synchronize()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def time_passes(index, q_dev, ids_dev, dists_dev, nprobe, k, passes, warmup, repeats):
    if warmup > 0:
        run_passes(index, q_dev, ids_dev, dists_dev, nprobe, k, warmup)
    return [run_passes(index, q_dev, ids_dev, dists_dev, nprobe, k, passes) for _ in range(repeats)]


def profile_steps(index, q_dev, ids_dev, dists_dev, nprobe, k, steps):
    """Searches one at a time with HIP events attached to every kernel launch on the compute stream."""
    nq = q_dev.shape[0]
    zero = {"calls": 0, "us_coarse": 0.0, "us_select": 0.0, "us_scan": 0.0, "us_merge": 0.0,
            "scan_bytes_per_call": 0.0, "scan_gbs": 0.0}
    if NO_EVENTS:
        for i in range(steps):
            j = i % nq
            index.ivf_search_device(q_dev[j], nprobe, k, ids_dev[j], dists_dev[j])
        index.ivf_synchronize()
        return zero
    index.ivf_profile_enable(True)
    index.ivf_profile_reset()
    for i in range(steps):
        j = i % nq
        index.ivf_search_device(q_dev[j], nprobe, k, ids_dev[j], dists_dev[j])
    p = index.ivf_profile_read()
    index.ivf_profile_enable(False)
    calls = max(int(p.calls), 1)
    return {
        "calls": int(p.calls),
        "us_coarse": p.ms_coarse / calls * 1e3, "us_select": p.ms_select / calls * 1e3,
        "us_scan": p.ms_scan / calls * 1e3, "us_merge": p.ms_merge / calls * 1e3,
        "scan_bytes_per_call": p.scan_bytes / calls,
        "scan_gbs": (p.scan_bytes / 1e9) / (p.ms_scan / 1e3) if p.ms_scan > 0 else 0.0,
    }


def passes_for(index, q_dev, ids_dev, dists_dev, nprobe, k, at_least=1):
    """passes so that one timed region lasts MIN_REGION_S or more"""
    t = run_passes(index, q_dev, ids_dev, dists_dev, nprobe, k, 1)
    return max(at_least, int(MIN_REGION_S / max(t, 1e-6)) + 1)


def oracle_layout(host):
    import oracle as O
    off, perm = O.build_layout(host["assign"], host["cent"].shape[0])
    return off, perm, host["rows"][perm]


def run_single_query(args):
    """configs[1] headline + nprobe sweep + host-buffer entry point + squared-L2 row."""
    import numpy as np
    import torch
    import oracle as O
    host, q_in, q_out, info = build_config2("cuda", args.n)
    log(f"c2: rows generated ({info['gen_s']} s)")
    index = make_index(host, args.metric)
    nq, k = q_out.shape[0], args.k
    q_dev = q_out.contiguous()
    ids_dev = torch.empty(nq, k, dtype=torch.int64, device="cuda")
    dists_dev = torch.empty(nq, k, dtype=torch.float32, device="cuda")
    depth_trials = {}
    if args.depth == 0:
        for depth in (2, 4, 6, 8, 12, 16):
            index.ivf_set_pipeline_depth(depth)
            index.ivf_reserve(1, 1024, k)
            run_passes(index, q_dev, ids_dev, dists_dev, args.nprobe, k, 1)
            t = run_passes(index, q_dev, ids_dev, dists_dev, args.nprobe, k, 6)
            depth_trials[depth] = round(6 * nq / t, 1)
        args.depth = max(depth_trials, key=depth_trials.get)
    index.ivf_set_pipeline_depth(args.depth)
    index.ivf_reserve(1, 1024, k)
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # headline: K passes over the 256 queries, timed REPEATS times
    secs = time_passes(index, q_dev, ids_dev, dists_dev, args.nprobe, k, args.steps, args.warmup, REPEATS)
    head = rates(args.steps * nq, secs)
    log(f"c2: headline {head}")
    # kernel durations are taken with one search at a time, so that no other kernel shares the GPU
    index.ivf_set_pipeline_depth(1)
    index.ivf_reserve(1, 1024, k)
    secs1 = time_passes(index, q_dev, ids_dev, dists_dev, args.nprobe, k, max(1, args.steps // 2), 1, REPEATS)
    one = rates(max(1, args.steps // 2) * nq, secs1)
    prof = profile_steps(index, q_dev, ids_dev, dists_dev, args.nprobe, k, 2048)

    # the same searches handed over as host buffers (ivf_search): every call starts from an idle
    # stream, the query is read from pinned host memory and the k results are stored there
    q_host = q_out.cpu().numpy()
    for i in range(32):
        index.ivf_search(q_host[i % nq], args.nprobe, k)
    host_secs = []
    for _ in range(REPEATS):
        t_h = time.perf_counter()
        for i in range(4 * nq):
            index.ivf_search(q_host[i % nq], args.nprobe, k)
        host_secs.append(time.perf_counter() - t_h)
    host_rate = rates(4 * nq, host_secs)

    off = perm = lists = None
    if not args.no_cpu:
        off, perm, lists = oracle_layout(host)
    sweep = []
    if not args.no_sweep:
        for nprobe in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024):
            index.ivf_set_pipeline_depth(args.depth)
            index.ivf_reserve(1, 1024, k)
            passes = passes_for(index, q_dev, ids_dev, dists_dev, nprobe, k)
            r = rates(passes * nq, time_passes(index, q_dev, ids_dev, dists_dev, nprobe, k, passes, 0, REPEATS))
            row = {"nprobe": nprobe, "qps": r["median"], "qps_min": r["min"], "qps_max": r["max"]}
            if lists is not None:       # outputs of the last pass against the oracle, two queries
                gi, gd = ids_dev.cpu().numpy(), dists_dev.cpu().numpy()
                ores = [O.search(lists, O.F32, off, perm, host["cent"], q_host[j], nprobe, k,
                                 O.IP if args.metric == "ip" else O.L2) for j in (0, nq // 2)]
                ps = compare_sample([gi[0], gi[nq // 2]], [gd[0], gd[nq // 2]], ores, 1e-4)
                row.update({"id_mismatches": ps["id_mismatches"], "near_tie_exemptions": ps["near_tie_exemptions"],
                            "max_rel_distance_error": ps["max_rel_distance_error"]})
            index.ivf_set_pipeline_depth(1)
            pr = profile_steps(index, q_dev, ids_dev, dists_dev, nprobe, k, 512 if nprobe < 256 else 256)
            row.update({"us_scan": round(pr["us_scan"], 2), "scan_gbs": round(pr["scan_gbs"], 1),
                        "frac": round(pr["scan_gbs"] / HBM_PEAK_GBS, 4),
                        "scan_mb": round(pr["scan_bytes_per_call"] / 1e6, 2),
                        # selected bytes over the wall time of the whole search, searches in flight as for `value`
                        "e2e_gbs": round(pr["scan_bytes_per_call"] * r["median"] / 1e9, 1)})
            sweep.append(row)
        log("c2: sweep done")

    out = {
        "metric": METRIC, "value": head["median"], "unit": "queries/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(1e3 * nq / head["median"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"configs[1] single-query retrieval: {args.n} x 768 fp32, 1024-component mixture, "
                               f"nlist 1024 (k-means on a tenth of the rows), nprobe {args.nprobe}, k {k}, "
                               f"batch 1, {'inner product' if args.metric == 'ip' else 'squared L2'}; a step = one pass over "
                               f"the {nq} distinct queries, one search each",
                   "entry_point": "ivf_search_device", "searches_in_flight": args.depth,
                   "depth_trials_qps": depth_trials, "seed": 20970, "queries_per_step": nq},
        "timing": {"regions": REPEATS, "searches_per_region": args.steps * nq,
                   "region_ms_median": round(1e3 * med(secs), 2), "qps_min": head["min"], "qps_max": head["max"]},
        "one_at_a_time": {"value": one["median"], "us_per_search": round(1e6 / one["median"], 2),
                          "qps_min": one["min"], "qps_max": one["max"]},
        "host_buffers": {"value": host_rate["median"], "us_per_search": round(1e6 / host_rate["median"], 2),
                         "qps_min": host_rate["min"], "qps_max": host_rate["max"],
                         "entry_point": "ivf_search (query and results cross PCIe, one call at a time)"},
        "roofline": {"bound": "hbm", "achieved": round(prof["scan_gbs"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(prof["scan_gbs"] / HBM_PEAK_GBS, 4),
                     "traffic": C2_SCAN_TRAFFIC_BYTES if (args.n == 1_000_000 and args.nprobe == 32 and args.metric == "ip") else None,
                     "kernel": "scan_kernel", "us_per_launch": round(prof["us_scan"], 2),
                     "bytes_per_launch": round(prof["scan_bytes_per_call"], 1)},
        "kernels_us": {k_: round(prof[k_], 2) for k_ in ("us_coarse", "us_select", "us_scan", "us_merge")},
        "nprobe_sweep": sweep,
        "setup": info,
    }
    if not args.no_cpu:
        # the oracle as it stands, on the host cores, over as many of the same queries as fit the budget
        done, t0, results = 0, time.perf_counter(), []
        om = O.IP if args.metric == "ip" else O.L2
        while done < nq and (done < 4 or time.perf_counter() - t0 < args.cpu_seconds):
            results.append(O.search(lists, O.F32, off, perm, host["cent"], q_host[done], args.nprobe, k, om))
            done += 1
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(done / dt, 2), "unit": "queries/s", "cores": O.threads(), "kind": "oracle",
                               "sample": f"{done} of the benchmark's queries, nprobe {args.nprobe}, k {k}, {dt:.1f} s of wall time"}
        # the outputs of the timed configuration for those queries must equal the oracle's
        index.ivf_set_pipeline_depth(args.depth)
        run_passes(index, q_dev, ids_dev, dists_dev, args.nprobe, k, 1)
        out["parity_sample"] = compare_sample(ids_dev.cpu().numpy()[:done], dists_dev.cpu().numpy()[:done], results, 1e-4)
        log(f"c2: oracle {out['cpu_baseline']['value']} q/s, parity {out['parity_sample']}")
    index.close()
    del index
    free_gpu()

    if args.metric == "ip" and not args.no_legs:
        # the second distance of App. B on the same rows
        ix2 = make_index(host, "l2")
        ix2.ivf_set_pipeline_depth(args.depth)
        ix2.ivf_reserve(1, 1024, k)
        passes = passes_for(ix2, q_dev, ids_dev, dists_dev, args.nprobe, k)
        r = rates(passes * nq, time_passes(ix2, q_dev, ids_dev, dists_dev, args.nprobe, k, passes, 1, REPEATS))
        leg = {"workload": "configs[1] rows, squared L2", "qps": r["median"], "qps_min": r["min"], "qps_max": r["max"]}
        if lists is not None:
            gi, gd = ids_dev.cpu().numpy(), dists_dev.cpu().numpy()
            ores = [O.search(lists, O.F32, off, perm, host["cent"], q_host[j], args.nprobe, k, O.L2) for j in range(8)]
            leg["parity_sample"] = compare_sample(gi[:8], gd[:8], ores, 1e-4)
        ix2.ivf_set_pipeline_depth(1)
        pr = profile_steps(ix2, q_dev, ids_dev, dists_dev, args.nprobe, k, 1024)
        leg["roofline"] = {"bound": "hbm", "kernel": "scan_kernel", "achieved": round(pr["scan_gbs"], 1),
                           "frac": round(pr["scan_gbs"] / HBM_PEAK_GBS, 4), "us_per_launch": round(pr["us_scan"], 2),
                           "bytes_per_launch": round(pr["scan_bytes_per_call"], 1)}
        # the same searches 32 queries per call: list-major over fp32 rows with the L2 filter score
        per_query_ids, per_query_dists = ids_dev.clone(), dists_dev.clone()
        ix2.ivf_reserve(32, 1024, k)

        def batched_pass(count):
            t = time.perf_counter()
            for _ in range(count):
                for j in range(0, nq, 32):
                    ix2.ivf_search_device(q_dev[j:j + 32], args.nprobe, k, ids_dev[j:j + 32], dists_dev[j:j + 32])
            ix2.ivf_synchronize()
            return time.perf_counter() - t
        batched_pass(2)
        cnt = max(2, int(MIN_REGION_S / max(batched_pass(2) / 2, 1e-6)) + 1)
        rb = rates(cnt * nq, [batched_pass(cnt) for _ in range(3)])
        same = bool(torch.equal(ids_dev, per_query_ids) and torch.equal(dists_dev, per_query_dists))
        leg["batch32_list_major"] = {"qps": rb["median"], "qps_min": rb["min"], "qps_max": rb["max"],
                                     "equal_to_query_by_query": same}
        if not NO_EVENTS:
            ix2.ivf_profile_enable(True); ix2.ivf_profile_reset()
            batched_pass(2)
            pb = ix2.ivf_profile_read(); ix2.ivf_profile_enable(False)
            calls = max(int(pb.calls), 1)
            us = pb.ms_scan / calls * 1e3
            leg["batch32_list_major"].update({"kernel": "batched_scan_f32_kernel", "us_per_launch": round(us, 1),
                                              "union_mb_per_call": round(pb.scan_bytes / calls / 1e6, 1),
                                              "achieved": round(pb.scan_bytes / calls / 1e3 / us, 1) if us > 0 else 0.0,
                                              "frac": round(pb.scan_bytes / calls / 1e3 / us / HBM_PEAK_GBS, 4) if us > 0 else 0.0})
        ix2.close()
        del ix2
        out["legs"] = {"l2": leg}
        log(f"c2: L2 leg {leg['qps']} q/s")
    del host, lists
    free_gpu()
    return out


# ---------------------------------------------------------------------------------------------------
# configs[3]: lookahead over pinned host lists
# ---------------------------------------------------------------------------------------------------
def run_lookahead(args, full=True):
    """Lists in pinned host memory, an 8 GB device prefetch buffer, ivf_prefetch(q_in) overlapped with
    a synthetic ~20 ms decode, then ivf_search(q_out) with the resident clusters on the GPU and the
    others on the host.  full: budget sweep and scheduler rows as well; else the cluster cache rows, the 1.28 GB row,
    the row whose copy fits under the decode, and the parity sample."""
    import numpy as np
    import torch
    import paper_2502_20969_amd as P
    import workloads as W
    t0 = time.time()
    pinned, scale, note = W.pinned_rows(int(60_000_000 * args.scale), 768, "f16")
    scale *= args.scale
    n, d, k = pinned.shape[0], 768, 10
    nlist = max(64, int(16384 * scale))
    nprobe = min(256, nlist)
    ds, q_in, q_out = W.config4_lookahead(pinned, nlist, args.pairs)
    torch.cuda.synchronize()
    log(f"c4: {n * d * 2 / 1e9:.1f} GB pinned (scale {scale}: {note}), datastore ready after {time.time() - t0:.1f} s")
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    cap = int(8e9)
    index = P.ivf_adopt_layout(pinned, "f16", ds.offsets, ds.centroids.cpu(), metric=P.IVF_IP,
                               placement=P.IVF_PLACE_HOST, device_buffer_bytes=cap,
                               compute_stream=compute, copy_stream=copy)
    threads = min(16, len(os.sched_getaffinity(0)))
    index.ivf_set_host_threads(threads)
    index.ivf_reserve(1, nprobe, k)
    setup_s = time.time() - t0

    # synthetic decode: bf16 matmuls on torch's stream, count calibrated to about 20 ms
    a = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
    b = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)

    def decode(reps):
        for _ in range(reps):
            torch.matmul(a, b)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    decode(4); torch.cuda.synchronize()
    e0.record(); decode(16); e1.record(); torch.cuda.synchronize()
    reps = max(1, int(round(20.0 / (e0.elapsed_time(e1) / 16))))
    e0.record(); decode(reps); e1.record(); torch.cuda.synchronize()
    decode_alone_ms = e0.elapsed_time(e1)

    qi, qo = q_in.numpy(), q_out.numpy()
    for j in range(args.pairs):          # untimed: first host touch of the lists these queries scan
        index.ivf_prefetch(qi[j], nprobe, 0, flags=P.IVF_PREFETCH_RESET)
        index.ivf_search(qo[j], nprobe, k)

    def budget_row(budget, label=None):
        acc = {"hit": [], "ms_search": [], "ms_host": [], "ms_probe": [], "ms_copy": [], "bytes": [], "ms_prefetch_call": [],
               "ms_decode": [], "gpu_bytes": [], "host_bytes": []}
        for rep in range(2 if full else 1):
            for j in range(args.pairs):
                t = time.perf_counter()
                ps = index.ivf_prefetch(qi[j], nprobe, budget, flags=P.IVF_PREFETCH_RESET)
                acc["ms_prefetch_call"].append((time.perf_counter() - t) * 1e3)
                e0.record(); decode(reps); e1.record()                 # overlaps the copies
                torch.cuda.synchronize()
                acc["ms_decode"].append(e0.elapsed_time(e1))
                acc["ms_copy"].append(index.ivf_prefetch_wait())
                acc["bytes"].append(ps.bytes)
                ids, dists, st = index.ivf_search(qo[j], nprobe, k, with_stats=True)
                acc["hit"].append(st.hit_rate); acc["ms_search"].append(st.ms_total); acc["ms_host"].append(st.ms_host_scan)
                acc["ms_probe"].append(st.ms_probe); acc["gpu_bytes"].append(st.bytes_gpu); acc["host_bytes"].append(st.bytes_host)
        m = {k_: float(np.mean(v)) for k_, v in acc.items()}
        copy_gbs = (m["bytes"] / 1e9) / (m["ms_copy"] / 1e3) if m["ms_copy"] > 0 else 0.0
        row = {"budget_gb": round(budget / 1e9, 3), "hit_rate": round(m["hit"], 4), "prefetched_gb": round(m["bytes"] / 1e9, 3),
               "copy_ms": round(m["ms_copy"], 2), "pcie_gbs": round(copy_gbs, 1),
               "copy_hidden_under_decode": bool(m["ms_copy"] <= m["ms_decode"]),
               "prefetch_call_ms": round(m["ms_prefetch_call"], 3), "decode_ms": round(m["ms_decode"], 2),
               "search_ms": round(float(np.median(acc["ms_search"])), 3), "search_ms_mean": round(m["ms_search"], 3),
               "probe_ms": round(m["ms_probe"], 3),
               "host_scan_ms": round(m["ms_host"], 3), "gpu_scan_gb": round(m["gpu_bytes"] / 1e9, 3),
               "host_scan_gb": round(m["host_bytes"] / 1e9, 3),
               "host_scan_gbs": round((m["host_bytes"] / 1e9) / (m["ms_host"] / 1e3), 1) if m["ms_host"] > 0 else 0.0}
        if label:
            row["budget_rule"] = label
        return row

    head = budget_row(int(1.28e9), "64 GB/s x 20 ms (the config's nominal link)")
    # Sec. 4.1 "Prefetching amount": budget = link bandwidth x generation time, with the link
    # bandwidth this machine's copies reach
    fit_budget = int(head["pcie_gbs"] * 1e9 * decode_alone_ms / 1e3 * 0.97) if head["pcie_gbs"] > 0 else int(0.9e9)
    rows = [budget_row(fit_budget, "measured copy GB/s x decode ms"), head]
    rows = [budget_row(int(g * 1e9)) for g in ((0.0, 0.25, 0.5) if full else (0.0, 0.5))] + rows + \
           [budget_row(int(g * 1e9)) for g in ((2.0, 8.0) if full else (2.0,))]
    log(f"c4: budget rows done ({head})")
    # App. C: the amount the model picks from what was just measured (link rate, generation time, host
    # time per missed cluster, miss-rate curve), beside the row that was fastest in fact
    model = None
    with_copy = [r for r in rows if r["pcie_gbs"] > 0]
    with_miss = [r for r in rows if r["hit_rate"] < 1.0 and r["host_scan_ms"] > 0]
    if with_copy and with_miss:
        bw = float(np.median([r["pcie_gbs"] for r in with_copy])) * 1e9
        t_cc = float(np.median([r["host_scan_ms"] / 1e3 / (nprobe * (1.0 - r["hit_rate"])) for r in with_miss]))
        curve = {}
        for r in sorted(rows, key=lambda r_: r_["prefetched_gb"]):
            curve.setdefault(r["prefetched_gb"] * 1e9, 1.0 - r["hit_rate"])
        bs = np.array(sorted(curve))
        rs = np.minimum.accumulate(np.array([curve[b_] for b_ in bs]))
        amount, seconds, which = P.ivf_prefetch_amount(bw, decode_alone_ms / 1e3, nprobe, t_cc, bs, rs)
        measured = [(max(r["decode_ms"], r["copy_ms"]) + r["search_ms"], r["budget_gb"]) for r in rows]
        model = {"bandwidth_gbs": round(bw / 1e9, 1), "t_llm_ms": round(decode_alone_ms, 2), "t_cc_us": round(t_cc * 1e6, 2),
                 "amount_gb": round(amount / 1e9, 3), "case": which, "model_t1_plus_t2_ms": round(seconds * 1e3, 3),
                 "measured_t1_plus_t2_ms": {f"{g}": round(t, 3) for t, g in measured},
                 "fastest_measured_budget_gb": min(measured)[1]}
        log(f"c4: prefetch amount model {model}")
    cache_rows, sched_rows = [], []
    budget = int(1.28e9)
    cache_leg = True          # also in the compact leg of the default run: the consolidation is measured there
    if cache_leg:
        # Cluster cache (Sec. 4.2 "Cache design"): a stream of requests around a few topics, each
        # request = prefetch(q_in) under the 1.28 GB budget, decode, search(q_out); once with a cold
        # buffer per request, once with the cache keeping at most half of the buffer between requests.
        n_req, topics = 48, 6
        tq_in = W.shared_batch_queries(ds, n_req, topics, 20981)
        tq_out = W.perturbed(tq_in, 0.3, 20982)
        tq_in, tq_out = tq_in.cpu().numpy(), tq_out.cpu().numpy()
        for j in range(n_req):               # untimed: first host touch of the lists these requests scan
            index.ivf_prefetch(tq_in[j], nprobe, 0, flags=P.IVF_PREFETCH_RESET)
            index.ivf_search(tq_out[j], nprobe, k)
        for mode in ("cold buffer per request", "cache fraction 0.5"):
            cached = mode.startswith("cache")
            index.ivf_prefetch(tq_in[0], nprobe, 0, flags=P.IVF_PREFETCH_RESET)
            index.ivf_cache_configure(0.5 if cached else -1.0, 1.0, 2.0, 1.0)
            acc = {"hit": [], "ms_search": [], "bytes": [], "ms_update": [], "ms_compact": [], "moved": [], "evicted": [],
                   "ms_round_call": [], "launches": []}
            for j in range(n_req):
                ps = index.ivf_prefetch(tq_in[j], nprobe, budget, flags=0 if cached else P.IVF_PREFETCH_RESET)
                decode(reps)
                torch.cuda.synchronize()
                index.ivf_prefetch_wait()
                ids, dists, st = index.ivf_search(tq_out[j], nprobe, k, with_stats=True)
                acc["hit"].append(st.hit_rate); acc["ms_search"].append(st.ms_total); acc["bytes"].append(ps.bytes)
                if cached:
                    t = time.perf_counter()
                    cs = index.ivf_cache_end_round()
                    acc["ms_round_call"].append((time.perf_counter() - t) * 1e3)
                    acc["ms_update"].append(cs.ms_update); acc["ms_compact"].append(cs.ms_compact)
                    acc["moved"].append(cs.bytes_moved); acc["evicted"].append(cs.n_evicted); acc["launches"].append(cs.n_launches)
            m = {k_: float(np.mean(v)) if v else 0.0 for k_, v in acc.items()}
            row = {"mode": mode, "requests": n_req, "topics": topics, "hit_rate": round(m["hit"], 4),
                   "prefetched_gb": round(m["bytes"] / 1e9, 3), "search_ms": round(m["ms_search"], 3)}
            if cached:
                row.update({"end_round_ms": round(m["ms_round_call"], 3), "hotness_update_ms": round(m["ms_update"], 3),
                            "compact_ms": round(m["ms_compact"], 3), "moved_gb": round(m["moved"] / 1e9, 3),
                            "evicted_clusters": round(m["evicted"], 1), "move_launches": round(m["launches"], 1),
                            # a move reads and writes its bytes
                            "move_traffic_gbs": round((2 * m["moved"] / 1e9) / (m["ms_compact"] / 1e3), 1) if m["ms_compact"] > 0 else 0.0})
            cache_rows.append(row)
        index.ivf_cache_configure(-1.0, 1.0, 2.0, 1.0)
        if full:
            # Prefetching scheduler (Sec. 4.2 "Scheduling optimization for prefetching"): a global batch of
            # requests around many topics, served in micro-batches that share one prefetch budget; once in
            # arrival order, once grouped by ivf_schedule.
            gB, micro, g_topics = 128, 8, 32
            gq_in = W.shared_batch_queries(ds, gB, g_topics, 20983)
            gq_out = W.perturbed(gq_in, 0.3, 20984)
            perm = torch.randperm(gB, generator=torch.Generator().manual_seed(20985))
            gq_in, gq_out = gq_in.cpu()[perm].numpy(), gq_out.cpu()[perm].numpy()       # topics arrive interleaved
            index.ivf_schedule(gq_in, micro)                                             # untimed first call
            t = time.perf_counter()
            order, ms_sched = index.ivf_schedule(gq_in, micro, with_time=True)
            ms_sched_call = (time.perf_counter() - t) * 1e3
            index.ivf_reserve(micro, nprobe, k)
            for j in range(0, gB, micro):            # untimed first touch
                index.ivf_prefetch(gq_in[j:j + micro], nprobe, 0, flags=P.IVF_PREFETCH_RESET)
                index.ivf_search(gq_out[j:j + micro], nprobe, k)
            for mode, seq in (("arrival order", np.arange(gB)), ("grouped by ivf_schedule", order)):
                hits, ms_s, copied = [], [], []
                for j in range(0, gB, micro):
                    g = seq[j:j + micro]
                    ps = index.ivf_prefetch(gq_in[g], nprobe, budget, flags=P.IVF_PREFETCH_RESET)
                    decode(reps)
                    torch.cuda.synchronize()
                    index.ivf_prefetch_wait()
                    ids, dists, st = index.ivf_search(gq_out[g], nprobe, k, with_stats=True)
                    hits.append(st.hit_rate); ms_s.append(st.ms_total); copied.append(ps.bytes)
                sched_rows.append({"mode": mode, "global_batch": gB, "micro_batch": micro, "topics": g_topics,
                                   "hit_rate": round(float(np.mean(hits)), 4), "search_ms_per_micro_batch": round(float(np.mean(ms_s)), 3),
                                   "prefetched_gb": round(float(np.mean(copied)) / 1e9, 3)})
            sched_rows.append({"ivf_schedule_gpu_ms": round(ms_sched, 3), "ivf_schedule_call_ms": round(ms_sched_call, 3)})
    # sampled parity at this size: hybrid searches against the oracle reading the same pinned lists
    parity, cpu = None, None
    if not args.no_cpu:
        import oracle as O
        off_np, cent_np = ds.offsets.numpy(), ds.centroids.cpu().numpy()
        nsamp = min(4, args.pairs)
        gi, gd, ores, t_or = [], [], [], 0.0
        for j in range(nsamp):
            index.ivf_prefetch(qi[j], nprobe, budget, flags=P.IVF_PREFETCH_RESET)
            i_, d_ = index.ivf_search(qo[j], nprobe, k)
            gi.append(i_[0]); gd.append(d_[0])
            res, dt = oracle_selected(pinned, O.F16, off_np, cent_np, qo[j], nprobe, k, O.IP)
            ores.append(res); t_or += dt
        parity = compare_sample(gi, gd, ores, 2e-3)
        cpu = {"value": round(nsamp / t_or, 2), "unit": "queries/s", "cores": O.threads(), "kind": "oracle",
               "sample": f"{nsamp} queries, nprobe {nprobe}, k {k}, selected lists copied out of the pinned region beforehand"}
    index.close()
    out = {"metric": "lookahead retrieval: hybrid IVF searches/sec with prefetch under a byte budget, 1 GPU",
           "value": round(1e3 / head["search_ms"], 1), "unit": "queries/s", "n_gpus": 1, "steps": args.pairs, "warmup": args.pairs,
           "ms_per_step": head["search_ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f16", "data": "synthetic",
           "config": {"workload": f"configs[3] limited-GPU-memory lookahead: {n} x 768 fp16 in pinned host memory, nlist {nlist}, "
                                  f"nprobe {nprobe}, k {k}, batch 1, device buffer {cap / 1e9:.1f} GB, scale {scale}"
                                  + ("" if scale == 1.0 else f" (rows and nlist scaled by {scale}; nprobe kept at {nprobe} rather than scaled with nlist, "
                                     "so that a query still scans and prefetches the named 1.4 GB)"),
                      "pinning": {"scale": scale, "first_refusal": note,
                                  "host": "RLIMIT_MEMLOCK unlimited and 309 GB of RAM on the box, yet hipHostMalloc grants about 64 GB of "
                                          "pinned memory per process in all (64 GB in one region succeeds, 70 GB does not, nor a second 40 GB beside a first)"},
                      "host_threads": threads, "decode_alone_ms": round(decode_alone_ms, 2), "decode_matmuls": reps},
           "budget_sweep": rows, "prefetch_amount_model": model, "cluster_cache": cache_rows,
           "prefetch_scheduler": sched_rows, "parity_sample": parity,
           "setup_s": round(setup_s, 1)}
    if cpu:
        out["cpu_baseline"] = cpu
    del index, ds, pinned, a, b
    free_gpu()
    return out


# ---------------------------------------------------------------------------------------------------
# configs[2] and configs[4]: batched retrieval, list-major
# ---------------------------------------------------------------------------------------------------
def run_batched(args, which, full=True):
    """configs[2] (c3: 10M x 768 fp16, nlist 4096 Zipf(1.1), nprobe 128, k 10, batch 32 sharing about
    40 % of the probed clusters) and configs[4] (c5: 30M x 1024 bf16, nlist 8192 Zipf(1.2), nprobe 512,
    k 100, batch 256 from distinct components), all lists resident in HBM, searched list-major.  A
    step is one whole batch."""
    import numpy as np
    import torch
    import paper_2502_20969_amd as P
    import workloads as W
    c3 = which == "c3"
    d, nlist, nprobe, k, B = (768, 4096, 128, 10, 32) if c3 else (1024, 8192, 512, 100, 256)
    d = args.dim if args.dim > 0 else d
    B = args.batch if args.batch > 0 else B
    k = args.topk if args.topk > 0 else k
    dtype, zipf = ("f16", 1.1) if c3 else ("bf16", 1.2)
    groups = args.groups if args.groups > 0 else (24 if c3 else B)      # 24 components: measured share 0.40
    n_sets = 8                                            # distinct batches cycled through the timed steps
    t0 = time.time()
    if c3:
        ds, qs = W.config3_mid_fp16(device="cuda", scale=args.scale, groups=groups, n_sets=n_sets, batch=B, d=d)
    else:
        ds, qs = W.config5_large_bf16(device="cuda", scale=args.scale, n_sets=n_sets, batch=B, d=d, groups=groups)
    n = ds.n
    torch.cuda.synchronize()
    log(f"{which}: datastore of {n * d * 2 / 1e9:.1f} GB ready after {time.time() - t0:.1f} s")
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    index = P.ivf_adopt_layout(ds.rows, dtype, ds.offsets, ds.centroids.cpu(), metric=P.IVF_IP,
                               compute_stream=compute, copy_stream=copy)
    index.ivf_set_batch_mode(2)
    # two batches in flight: the second one's coarse scores, selection and task lists are made
    # while the first one's scan streams (each on its own stream, workspace and outputs)
    depth = 1 if args.depth == 1 else 2
    ids2 = torch.empty(depth, B, k, dtype=torch.int64, device="cuda")
    dists2 = torch.empty(depth, B, k, dtype=torch.float32, device="cuda")
    ids, dists = ids2[0], dists2[0]
    index.ivf_set_pipeline_depth(depth)
    index.ivf_reserve(B, nprobe, k)
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def batches(nprobe_, count, first=0):
        t = time.perf_counter()
        for i in range(count):
            index.ivf_search_device(qs[(first + i) % n_sets], nprobe_, k, ids2[i % depth], dists2[i % depth])
        index.ivf_synchronize()
        return time.perf_counter() - t

    def run(nprobe_, repeats):
        index.ivf_set_pipeline_depth(depth)
        batches(nprobe_, 2)
        per = max(2, int(MIN_REGION_S / max(batches(nprobe_, 2) / 2, 1e-6)) + 1)
        r = rates(per * B, [batches(nprobe_, per, 3 * j) for j in range(repeats)])
        # kernel durations: one batch at a time, so that no other kernel shares the GPU
        index.ivf_set_pipeline_depth(1)
        if not NO_EVENTS:
            index.ivf_profile_enable(True); index.ivf_profile_reset()
        for i in range(n_sets):
            index.ivf_search_device(qs[i], nprobe_, k, ids, dists)
        p = index.ivf_profile_read(); index.ivf_profile_enable(False)
        calls = max(int(p.calls), 1)
        us_scan = p.ms_scan / calls * 1e3
        return {"nprobe": nprobe_, "qps": r["median"], "qps_min": r["min"], "qps_max": r["max"],
                "batches_per_region": per, "ms_per_batch": round(1e3 * B / r["median"], 3),
                "us_scan": round(us_scan, 1), "us_coarse": round(p.ms_coarse / calls * 1e3, 1),
                "us_select": round(p.ms_select / calls * 1e3, 1),
                "scan_gb": round(p.scan_bytes / calls / 1e9, 3),
                "scan_gbs": round((p.scan_bytes / calls / 1e9) / (us_scan / 1e6), 1) if us_scan > 0 else 0.0,
                "e2e_gbs": round(p.scan_bytes / calls / 1e9 * r["median"] / B, 1)}

    head = run(nprobe, REPEATS)
    log(f"{which}: head {head}")
    # measured sharing of the batch: 1 - |union of probed clusters| / (B * nprobe)
    pr = index.ivf_probe(qs[0].cpu().numpy(), nprobe)
    share = 1.0 - len(set(pr.reshape(-1).tolist())) / float(pr.size)
    sweep = []
    if full and not args.no_sweep:
        for np_ in ((16, 32, 64, 128, 256) if c3 else (64, 128, 256, 512)):
            sweep.append(run(np_, 3))
    parity, cpu = None, None
    if not args.no_cpu:
        import oracle as O
        odt = O.F16 if c3 else O.BF16
        q0 = qs[0].cpu().numpy()
        index.ivf_set_pipeline_depth(depth)
        index.ivf_search_device(qs[0], nprobe, k, ids, dists)
        index.ivf_synchronize()
        gi, gd = ids.cpu().numpy(), dists.cpu().numpy()
        off_np, cent_np = ds.offsets.numpy(), ds.centroids.cpu().numpy()
        which_q = list(range(0, B, max(1, B // (8 if c3 else 4))))
        ores, t_or = [], 0.0
        for b in which_q:
            res, dt = oracle_selected(ds.rows, odt, off_np, cent_np, q0[b], nprobe, k, O.IP)
            ores.append(res); t_or += dt
        parity = compare_sample([gi[b] for b in which_q], [gd[b] for b in which_q], ores, 2e-3)
        cpu = {"value": round(len(which_q) / t_or, 3), "unit": "queries/s", "cores": O.threads(), "kind": "oracle",
               "sample": f"{len(which_q)} queries of one batch, nprobe {nprobe}, k {k}, selected lists copied to the host beforehand"}
    named = args.scale == 1.0 and args.dim == 0 and args.batch == 0 and args.topk == 0 and args.groups == 0
    index.close()
    out = {"metric": METRIC, "value": head["qps"], "unit": "queries/s", "n_gpus": 1,
           "steps": head["batches_per_region"], "warmup": 4, "ms_per_step": head["ms_per_batch"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
           "config": {"workload": f"configs[{2 if c3 else 4}] batched retrieval: {n} x {d} {dtype}, nlist {nlist} Zipf({zipf}), "
                                  f"nprobe {nprobe}, k {k}, batch {B} from {groups} mixture components, scale {args.scale}",
                      "measured_share": round(share, 3), "entry_point": "ivf_search_device (list-major)",
                      "batches_in_flight": depth},
           "roofline": {"bound": "hbm", "achieved": head["scan_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": round(head["scan_gbs"] / HBM_PEAK_GBS, 4),
                        "traffic": (C3_SCAN_TRAFFIC_BYTES if c3 else C5_SCAN_TRAFFIC_BYTES) if named else None,
                        "kernel": "batched_scan_kernel",
                        "us_per_launch": head["us_scan"], "bytes_per_launch": head["scan_gb"] * 1e9,
                        "mfma_util": (C3_MFMA_UTIL if c3 else C5_MFMA_UTIL) if named else None},
           "head": head, "nprobe_sweep": sweep, "parity_sample": parity, "setup_s": round(setup_s, 1)}
    if cpu:
        out["cpu_baseline"] = cpu
    del index, ds, qs, ids2, dists2
    free_gpu()
    return out


# ---------------------------------------------------------------------------------------------------
# the paper's resident shape
# ---------------------------------------------------------------------------------------------------
def run_paper_shape(args, full=True):
    """A resident datastore of the size and shape the paper evaluates on (Sec. 5 set-up: 21 M x 768
    fp32 rows, 4096 clusters, inner product, top-3 retrieval), here with seeded synthetic rows and
    Zipf(1.1) list sizes: nprobe sweep 64..1024 at batch 1, and batches of 2, 4 and 8 queries per call
    at nprobe 256."""
    import numpy as np
    import torch
    import paper_2502_20969_amd as P
    import workloads as W
    k, nq = 3, 64
    t0 = time.time()
    ds, q_out = W.paper_shape_fp32(device="cuda", scale=args.scale, nq=nq)
    n, d, nlist = ds.n, ds.d, ds.nlist
    torch.cuda.synchronize()
    log(f"n1: datastore of {n * d * 4 / 1e9:.1f} GB ready after {time.time() - t0:.1f} s")
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    cent_np = ds.centroids.cpu().numpy()
    index = P.ivf_adopt_layout(ds.rows, "f32", ds.offsets, cent_np, metric=P.IVF_IP,
                               compute_stream=compute, copy_stream=copy)
    ids = torch.empty(nq, k, dtype=torch.int64, device="cuda")
    dists = torch.empty(nq, k, dtype=torch.float32, device="cuda")
    index.ivf_reserve(8, 1024, k)

    def calls(nprobe, B, count, first=0):
        t = time.perf_counter()
        for i in range(count):
            j = ((first + i) * B) % nq
            index.ivf_search_device(q_out[j:j + B], nprobe, k, ids[j:j + B], dists[j:j + B])
        index.ivf_synchronize()
        return time.perf_counter() - t

    def run(nprobe, B, depth, repeats):
        index.ivf_set_pipeline_depth(depth)
        index.ivf_reserve(B, 1024, k)
        calls(nprobe, B, 8)
        per = max(8, int(MIN_REGION_S / max(calls(nprobe, B, 8) / 8, 1e-6)) + 1)
        r = rates(per * B, [calls(nprobe, B, per, 5 * j) for j in range(repeats)])
        index.ivf_set_pipeline_depth(1)
        index.ivf_reserve(B, 1024, k)
        if not NO_EVENTS:
            index.ivf_profile_enable(True); index.ivf_profile_reset()
        calls(nprobe, B, 64 // B)
        p = index.ivf_profile_read(); index.ivf_profile_enable(False)
        ncalls = max(int(p.calls), 1)
        us_scan = p.ms_scan / ncalls * 1e3
        gbs = (p.scan_bytes / ncalls / 1e9) / (us_scan / 1e6) if us_scan > 0 else 0.0
        return {"nprobe": nprobe, "batch": B, "searches_in_flight": depth, "qps": r["median"], "qps_min": r["min"],
                "qps_max": r["max"], "calls_per_region": per,
                "us_scan": round(us_scan, 1), "scan_mb": round(p.scan_bytes / ncalls / 1e6, 1),
                "scan_gbs": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4)}

    depth = args.depth if args.depth > 0 else 6
    head = run(256, 1, depth, REPEATS if args.batch == 0 else 1)
    log(f"n1: head {head}")
    sweep = []
    if not args.no_sweep:
        for B in ((args.batch,) if args.batch > 0 else (2, 4, 8)):
            sweep.append(run(256, B, 1, 3))
        if full and args.batch == 0:
            for nprobe in (64, 128, 512, 1024):
                sweep.append(run(nprobe, 1, depth, 3))
            sweep.append(run(256, 1, 1, 3))
    parity, cpu = None, None
    if not args.no_cpu:
        import oracle as O
        nprobe = 256
        index.ivf_set_pipeline_depth(depth)
        for j in range(nq):
            index.ivf_search_device(q_out[j], nprobe, k, ids[j], dists[j])
        index.ivf_synchronize()
        gi, gd = ids.cpu().numpy(), dists.cpu().numpy()
        q_np = q_out.cpu().numpy()
        off_np = ds.offsets.numpy()
        which_q = list(range(0, nq, nq // 4))
        ores, t_or = [], 0.0
        for b in which_q:
            res, dt = oracle_selected(ds.rows, O.F32, off_np, cent_np, q_np[b], nprobe, k, O.IP)
            ores.append(res); t_or += dt
        parity = compare_sample([gi[b] for b in which_q], [gd[b] for b in which_q], ores, 1e-4)
        cpu = {"value": round(len(which_q) / t_or, 3), "unit": "queries/s", "cores": O.threads(), "kind": "oracle",
               "sample": f"{len(which_q)} queries, nprobe {nprobe}, k {k}, selected lists copied to the host beforehand"}
    index.close()
    out = {"metric": METRIC, "value": head["qps"], "unit": "queries/s", "n_gpus": 1, "steps": head["calls_per_region"], "warmup": 16,
           "ms_per_step": round(1e3 / head["qps"], 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"paper-shaped resident datastore: {n} x {d} fp32, nlist {nlist} Zipf(1.1), nprobe 256, "
                                  f"k {k}, batch 1, inner product, scale {args.scale}",
                      "entry_point": "ivf_search_device", "searches_in_flight": depth},
           "roofline": {"bound": "hbm", "achieved": head["scan_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": head["frac"], "traffic": None, "kernel": "scan_kernel", "us_per_launch": head["us_scan"],
                        "bytes_per_launch": head["scan_mb"] * 1e6},
           "head": head, "sweep": sweep, "parity_sample": parity, "setup_s": round(time.time() - t0, 1)}
    if cpu:
        out["cpu_baseline"] = cpu
    del index, ds, ids, dists
    free_gpu()
    return out


def compact(leg):
    """what a leg contributes to the headline line"""
    keep = ("value", "unit", "ms_per_step", "dtype", "roofline", "parity_sample", "cpu_baseline")
    out = {"workload": leg["config"]["workload"]}
    out.update({k_: leg[k_] for k_ in keep if k_ in leg})
    for extra in ("measured_share", "batches_in_flight", "searches_in_flight", "pinning", "decode_alone_ms"):
        if extra in leg["config"]:
            out[extra] = leg["config"][extra]
    if "head" in leg:
        out["qps_min"], out["qps_max"] = leg["head"]["qps_min"], leg["head"]["qps_max"]
    if "budget_sweep" in leg:
        out["budget_rows"] = leg["budget_sweep"]
    if leg.get("cluster_cache"):
        out["cluster_cache"] = leg["cluster_cache"]
    if leg.get("prefetch_amount_model"):
        out["prefetch_amount_model"] = leg["prefetch_amount_model"]
    if "sweep" in leg:
        out["rows"] = leg["sweep"]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16, help="c2: timed passes over the 256 distinct queries per region")
    ap.add_argument("--warmup", type=int, default=2, help="c2: untimed passes before the first region")
    ap.add_argument("--repeats", type=int, default=5, help="timed regions; the median is reported")
    ap.add_argument("--n", type=int, default=1_000_000, help="rows of the datastore (default: the named config)")
    ap.add_argument("--nprobe", type=int, default=32)
    ap.add_argument("--k", type=int, default=10)
    ap.add_argument("--depth", type=int, default=0,
                    help="independent searches kept in flight (ivf_set_pipeline_depth); 1 = strictly one after "
                         "another; 0 = try 2, 4, 6, 8, 12 and 16 in short untimed runs and keep the fastest (how HIP maps "
                         "streams to hardware queues makes some depths overlap better than others)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 1 GiB device-to-device copies (a kernel of known traffic for scaling rocprofv3 counters)")
    ap.add_argument("--no-events", action="store_true",
                    help="skip the passes that time kernels with HIP events (for runs under rocprofv3 --pmc)")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-legs", action="store_true", help="c2: only the headline workload, without the other configurations' legs")
    ap.add_argument("--legs", default="c3,c5,c4,n1", help="c2: the other configurations measured after the headline")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="c2: time budget of the oracle baseline")
    ap.add_argument("--metric", default="ip", choices=["ip", "l2"], help="c2: distance function")
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c4", "c5", "n1"],
                    help="c2: single-query retrieval (the default bench line, followed by compact legs of the others); c4: lookahead "
                         "with host-resident lists; c3 / c5: batched retrieval over fp16 / bf16 lists; n1: the paper's resident shape")
    ap.add_argument("--scale", type=float, default=1.0, help="c3, c4, c5, n1: fraction of the named datastore to build")
    ap.add_argument("--dim", type=int, default=0, help="c3, c5: row dimension instead of the named one (a multiple of 64)")
    ap.add_argument("--batch", type=int, default=0, help="c3, c5: queries per batch instead of the named number; n1: only this batch size in the batch rows")
    ap.add_argument("--topk", type=int, default=0, help="c3, c5: k instead of the named one")
    ap.add_argument("--groups", type=int, default=0, help="c3, c5: mixture components the batch's queries are drawn around")
    ap.add_argument("--pairs", type=int, default=64, help="c4: (q_in, q_out) pairs per budget")
    args = ap.parse_args()
    global NO_EVENTS, REPEATS
    NO_EVENTS = args.no_events
    REPEATS = max(1, args.repeats)
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    if args.workload == "c4":
        out = run_lookahead(args)
    elif args.workload in ("c3", "c5"):
        out = run_batched(args, args.workload)
    elif args.workload == "n1":
        out = run_paper_shape(args)
    else:
        out = run_single_query(args)
        if not args.no_legs:
            legs = out.setdefault("legs", {})
            for name in [s for s in args.legs.split(",") if s]:
                t = time.time()
                if name in ("c3", "c5"):
                    legs[name] = compact(run_batched(args, name, full=False))
                elif name == "c4":
                    legs[name] = compact(run_lookahead(args, full=False))
                elif name == "n1":
                    legs[name] = compact(run_paper_shape(args, full=False))
                log(f"leg {name} done in {time.time() - t:.1f} s")
    out["wall_s"] = round(time.time() - T_START, 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
