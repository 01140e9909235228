"""Benchmark of the IVF search hot path on one MI355X.

Workload: benchmark configs[1] -- single-query retrieval over 1,000,000 x 768 fp32 rows in
1024 k-means lists, nprobe 32, k 10, batch 1, synthetic (seeded mixture of Gaussians).  A step is
one whole search (coarse scoring, top-nprobe selection, list scan, top-k merge) of one query
through ivf_search_device; query and outputs are resident in HBM; 256 distinct queries are
cycled so that consecutive steps scan different lists.  Prints one JSON line.
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
METRIC = "IVF search queries/sec + achieved HBM GB/s (% of peak) at nprobe sweep, 1 GPU"


def build_config2(device, n, seed=20970):
    import torch
    import paper_2502_20969_amd as P
    import workloads as W
    t0 = time.time()
    ds, q_in, q_out = W.config2_single_query(seed=seed, device=device, n=n)
    torch.cuda.synchronize()
    rows_host = ds.rows.cpu().numpy()
    assign_host = ds.assign.cpu().numpy()
    cent_host = ds.centroids.cpu().numpy()
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    index = P.ivf_build_layout(rows_host, "f32", cent_host, assign_host, metric=P.IVF_IP,
                               compute_stream=compute, copy_stream=copy)
    info = {"gen_build_s": round(time.time() - t0, 2)}
    return index, compute, rows_host, assign_host, cent_host, q_in, q_out, info


def time_steps(index, stream, q_dev, ids_dev, dists_dev, nprobe, k, steps, warmup):
    import torch
    nq = q_dev.shape[0]
    for i in range(warmup):
        j = i % nq
        index.ivf_search_device(q_dev[j], nprobe, k, ids_dev[j], dists_dev[j])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        j = (warmup + i) % nq
        index.ivf_search_device(q_dev[j], nprobe, k, ids_dev[j], dists_dev[j])
    index.ivf_synchronize()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def profile_steps(index, stream, q_dev, ids_dev, dists_dev, nprobe, k, steps):
    """Same loop with HIP events around every kernel on the compute stream."""
    nq = q_dev.shape[0]
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


def cpu_baseline(rows_host, assign_host, cent_host, q_out, nprobe, k, budget_s=12.0):
    """The oracle as it stands, timed on the host cores over as many of the same queries as fit
    the time budget (at least 4)."""
    import numpy as np
    import oracle as O
    nlist = cent_host.shape[0]
    off, perm = O.build_layout(assign_host, nlist)
    lists = rows_host[perm]
    q = q_out.cpu().numpy()
    done, t0 = 0, time.perf_counter()
    results = []
    while done < q.shape[0] and (done < 4 or time.perf_counter() - t0 < budget_s):
        results.append(O.search(lists, O.F32, off, perm, cent_host, q[done], nprobe, k, O.IP))
        done += 1
    dt = time.perf_counter() - t0
    return {"value": done / dt, "unit": "queries/s", "cores": O.threads(), "kind": "oracle",
            "sample": f"{done} of the benchmark's queries, nprobe {nprobe}, k {k}, {dt:.1f} s of wall time"}, \
        (off, perm, lists, results)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4096)
    ap.add_argument("--warmup", type=int, default=512)
    ap.add_argument("--n", type=int, default=1_000_000, help="rows of the datastore (default: the named config)")
    ap.add_argument("--nprobe", type=int, default=32)
    ap.add_argument("--k", type=int, default=10)
    ap.add_argument("--depth", type=int, default=4,
                    help="independent searches kept in flight (ivf_set_pipeline_depth); 1 = strictly one after another")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 1 GiB device-to-device copies (a kernel of known traffic for scaling rocprofv3 counters)")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    index, stream, rows_host, assign_host, cent_host, q_in, q_out, info = build_config2("cuda", args.n)
    nq = q_out.shape[0]
    q_dev = q_out.contiguous()
    ids_dev = torch.empty(nq, args.k, dtype=torch.int64, device="cuda")
    dists_dev = torch.empty(nq, args.k, dtype=torch.float32, device="cuda")
    index.ivf_set_pipeline_depth(args.depth)
    index.ivf_reserve(1, 1024, args.k)
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    dt = time_steps(index, stream, q_dev, ids_dev, dists_dev, args.nprobe, args.k, args.steps, args.warmup)
    # kernel durations are taken with one search at a time, so that no other kernel shares the GPU
    index.ivf_set_pipeline_depth(1)
    index.ivf_reserve(1, 1024, args.k)
    dt1 = time_steps(index, stream, q_dev, ids_dev, dists_dev, args.nprobe, args.k, args.steps, args.warmup)
    prof = profile_steps(index, stream, q_dev, ids_dev, dists_dev, args.nprobe, args.k, min(args.steps, 2048))

    sweep = []
    if not args.no_sweep:
        for nprobe in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024):
            steps = max(64, min(args.steps, int(200000 / max(nprobe, 8))))
            index.ivf_set_pipeline_depth(args.depth)
            index.ivf_reserve(1, 1024, args.k)
            t = time_steps(index, stream, q_dev, ids_dev, dists_dev, nprobe, args.k, steps, 32)
            index.ivf_set_pipeline_depth(1)
            pr = profile_steps(index, stream, q_dev, ids_dev, dists_dev, nprobe, args.k, min(steps, 512))
            sweep.append({"nprobe": nprobe, "qps": round(steps / t, 1), "us_scan": round(pr["us_scan"], 2),
                          "scan_gbs": round(pr["scan_gbs"], 1), "frac": round(pr["scan_gbs"] / HBM_PEAK_GBS, 4),
                          "scan_mb": round(pr["scan_bytes_per_call"] / 1e6, 2)})

    out = {
        "metric": METRIC, "value": round(args.steps / dt, 1), "unit": "queries/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"configs[1] single-query retrieval: {args.n} x 768 fp32, 1024-component mixture, "
                               f"nlist 1024 (k-means on a tenth of the rows), nprobe {args.nprobe}, k {args.k}, "
                               f"batch 1, inner product, {nq} distinct queries cycled",
                   "entry_point": "ivf_search_device", "searches_in_flight": args.depth, "seed": 20970},
        "one_at_a_time": {"value": round(args.steps / dt1, 1), "ms_per_step": dt1 / args.steps * 1e3},
        "roofline": {"bound": "hbm", "achieved": round(prof["scan_gbs"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(prof["scan_gbs"] / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": "scan_kernel", "us_per_launch": round(prof["us_scan"], 2),
                     "bytes_per_launch": round(prof["scan_bytes_per_call"], 1)},
        "kernels_us": {k_: round(prof[k_], 2) for k_ in ("us_coarse", "us_select", "us_scan", "us_merge")},
        "nprobe_sweep": sweep,
        "setup": info,
    }
    if not args.no_cpu:
        base, (off, perm, lists, results) = cpu_baseline(rows_host, assign_host, cent_host, q_out, args.nprobe, args.k)
        out["cpu_baseline"] = base
        # the timed outputs of those queries must equal the oracle's
        torch.cuda.synchronize()
        index.ivf_profile_enable(False)
        index.ivf_set_pipeline_depth(args.depth)
        for j in range(nq):
            index.ivf_search_device(q_dev[j], args.nprobe, args.k, ids_dev[j], dists_dev[j])
        index.ivf_synchronize()
        got = ids_dev.cpu().numpy()
        bad = sum(int(not np.array_equal(got[j], results[j][0])) for j in range(len(results)))
        out["parity_sample"] = {"queries": len(results), "id_mismatches": bad}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
