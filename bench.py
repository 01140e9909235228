"""Benchmark of the IVF search hot path on one MI355X.

Workload: single-query retrieval (configs[1] of the benchmark definition) over 1,000,000 x 768
fp32 rows in 1024 k-means lists, nprobe 32, k 10, batch 1, synthetic (seeded mixture of Gaussians).  A step is
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
# HBM bytes one scan launch of the default workload moves, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE scaled by a 1 GiB copy (profiles/scan_kernel_c2_single_query.md): read + written
C2_SCAN_TRAFFIC_BYTES = 89207 * 1024 + 96 * 1024
# the same for the batched scan launch of configs[2] (default 24 components) and configs[4]
# (profiles/batched_scan_kernel_c3_c5.md): FETCH_SIZE KiB x 2.0 x 1024
C3_SCAN_TRAFFIC_BYTES = 5027107 * 2048
C5_SCAN_TRAFFIC_BYTES = 30003315 * 2048
METRIC = "IVF search queries/sec + achieved HBM GB/s (% of peak) at nprobe sweep, 1 GPU"


def build_config2(device, n, seed=20970, metric="ip"):
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
    index = P.ivf_build_layout(rows_host, "f32", cent_host, assign_host,
                               metric=P.IVF_IP if metric == "ip" else P.IVF_L2,
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


NO_EVENTS = False


def profile_steps(index, stream, q_dev, ids_dev, dists_dev, nprobe, k, steps):
    """Same loop with HIP events attached to every kernel launch on the compute stream."""
    nq = q_dev.shape[0]
    if NO_EVENTS:
        for i in range(steps):
            j = i % nq
            index.ivf_search_device(q_dev[j], nprobe, k, ids_dev[j], dists_dev[j])
        index.ivf_synchronize()
        return {"calls": 0, "us_coarse": 0.0, "us_select": 0.0, "us_scan": 0.0, "us_merge": 0.0,
                "scan_bytes_per_call": 0.0, "scan_gbs": 0.0}
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


def cpu_baseline(rows_host, assign_host, cent_host, q_out, nprobe, k, budget_s=12.0, metric="ip"):
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
        results.append(O.search(lists, O.F32, off, perm, cent_host, q[done], nprobe, k,
                                O.IP if metric == "ip" else O.L2))
        done += 1
    dt = time.perf_counter() - t0
    return {"value": done / dt, "unit": "queries/s", "cores": O.threads(), "kind": "oracle",
            "sample": f"{done} of the benchmark's queries, nprobe {nprobe}, k {k}, {dt:.1f} s of wall time"}, \
        (off, perm, lists, results)


def run_lookahead(args):
    """Lookahead configuration (configs[3]): lists in pinned host memory, an 8 GB device prefetch buffer,
    ivf_prefetch(q_in) overlapped with a synthetic ~20 ms decode, then ivf_search(q_out) with the
    resident clusters on the GPU and the others on the host.  One JSON line with a budget sweep."""
    import numpy as np
    import torch
    import paper_2502_20969_amd as P
    import workloads as W
    torch.cuda.set_device(0)
    t0 = time.time()
    scale, pinned = args.scale, None
    while pinned is None:
        # the datastore is scaled down (same d, rows per list and nprobe) when the host cannot pin it
        n, d, nlist, nprobe, k = int(60_000_000 * scale), 768, max(64, int(16384 * scale)), 256, 10
        print(f"[c4] allocating {n * d * 2 / 1e9:.1f} GB of pinned host memory", file=sys.stderr, flush=True)
        try:
            pinned = torch.empty((n, d), dtype=torch.float16, pin_memory=True)
        except RuntimeError as e:
            print(f"[c4] could not pin it ({str(e).splitlines()[0]}); halving the datastore", file=sys.stderr, flush=True)
            scale /= 2
            if scale < 0.01:
                raise
    nprobe = min(nprobe, nlist)
    sizes = W.zipf_sizes(n, nlist, 0.1, 20972)
    print(f"[c4] pinned after {time.time() - t0:.1f} s; generating rows on the GPU", file=sys.stderr, flush=True)
    ds = W.cluster_major_datastore(sizes, d, 0.3, 20973, dtype="f16", device="cuda", out=pinned, chunk=1 << 20)
    torch.cuda.synchronize()
    print(f"[c4] datastore ready after {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
    q_in, q_out = W.query_pairs(pinned, args.pairs, 0.3, 20974)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    cap = int(8e9 * min(1.0, scale * 4))
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
    print(f"[c4] warm after {time.time() - t0:.1f} s; budget sweep", file=sys.stderr, flush=True)
    rows = []
    for budget_gb in (0.0, 0.25, 0.5, 1.28, 2.0, 8.0):
        budget = int(budget_gb * 1e9 * min(1.0, scale * 4))
        acc = {"hit": [], "ms_search": [], "ms_host": [], "ms_probe": [], "ms_copy": [], "bytes": [], "ms_prefetch_call": [],
               "ms_decode": [], "gpu_bytes": [], "host_bytes": []}
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
        rows.append({"budget_gb": budget / 1e9, "hit_rate": round(m["hit"], 4), "prefetched_gb": round(m["bytes"] / 1e9, 3),
                     "copy_ms": round(m["ms_copy"], 2), "pcie_gbs": round(copy_gbs, 1),
                     "prefetch_call_ms": round(m["ms_prefetch_call"], 3), "decode_ms": round(m["ms_decode"], 2),
                     "search_ms": round(m["ms_search"], 3), "probe_ms": round(m["ms_probe"], 3),
                     "host_scan_ms": round(m["ms_host"], 3), "gpu_scan_gb": round(m["gpu_bytes"] / 1e9, 3),
                     "host_scan_gb": round(m["host_bytes"] / 1e9, 3),
                     "host_scan_gbs": round((m["host_bytes"] / 1e9) / (m["ms_host"] / 1e3), 1) if m["ms_host"] > 0 else 0.0})
    # Cluster cache (Sec. 4.2 "Cache design"): a stream of requests around a few topics, each
    # request = prefetch(q_in) under the 1.28 GB budget, decode, search(q_out); once with a cold
    # buffer per request, once with the cache keeping at most half of the buffer between requests.
    cache_rows = []
    n_req, topics = 3 * args.pairs, 6
    tq_in = W.shared_batch_queries(ds, n_req, topics, 20981)
    tq_out = W.perturbed(tq_in, 0.3, 20982)
    tq_in, tq_out = tq_in.cpu().numpy(), tq_out.cpu().numpy()
    budget = int(1.28e9 * min(1.0, scale * 4))
    for j in range(n_req):               # untimed: first host touch of the lists these requests scan
        index.ivf_prefetch(tq_in[j], nprobe, 0, flags=P.IVF_PREFETCH_RESET)
        index.ivf_search(tq_out[j], nprobe, k)
    for mode in ("cold buffer per request", "cache fraction 0.5"):
        cached = mode.startswith("cache")
        index.ivf_prefetch(tq_in[0], nprobe, 0, flags=P.IVF_PREFETCH_RESET)
        index.ivf_cache_configure(0.5 if cached else -1.0, 1.0, 2.0, 1.0)
        acc = {"hit": [], "ms_search": [], "bytes": [], "ms_update": [], "ms_compact": [], "moved": [], "evicted": [],
               "ms_round_call": []}
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
                acc["moved"].append(cs.bytes_moved); acc["evicted"].append(cs.n_evicted)
        m = {k_: float(np.mean(v)) if v else 0.0 for k_, v in acc.items()}
        row = {"mode": mode, "requests": n_req, "topics": topics, "hit_rate": round(m["hit"], 4),
               "prefetched_gb": round(m["bytes"] / 1e9, 3), "search_ms": round(m["ms_search"], 3)}
        if cached:
            row.update({"end_round_ms": round(m["ms_round_call"], 3), "hotness_update_ms": round(m["ms_update"], 3),
                        "compact_ms": round(m["ms_compact"], 3), "moved_gb": round(m["moved"] / 1e9, 3),
                        "evicted_clusters": round(m["evicted"], 1),
                        "move_gbs": round((m["moved"] / 1e9) / (m["ms_compact"] / 1e3), 1) if m["ms_compact"] > 0 else 0.0})
        cache_rows.append(row)
    index.ivf_cache_configure(-1.0, 1.0, 2.0, 1.0)
    # Prefetching scheduler (Sec. 4.2 "Scheduling optimization for prefetching"): a global batch of
    # requests around many topics, served in micro-batches that share one prefetch budget; once in
    # arrival order, once grouped by ivf_schedule.
    sched_rows = []
    gB, micro, g_topics = 8 * args.pairs, 8, 2 * args.pairs
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
    # sampled parity at this size: two hybrid searches against the oracle on the same pinned lists
    parity = None
    if not args.no_cpu:
        import oracle as O
        lists_np = pinned.numpy().view(np.uint16)
        off_np, cent_np = ds.offsets.numpy(), ds.centroids.cpu().numpy()
        bad = 0
        for j in range(min(2, args.pairs)):
            index.ivf_prefetch(qi[j], nprobe, int(1.28e9 * min(1.0, scale * 4)), flags=P.IVF_PREFETCH_RESET)
            gi, gd = index.ivf_search(qo[j], nprobe, k)
            oi, osc = O.search(lists_np, O.F16, off_np, None, cent_np, qo[j], nprobe, k, O.IP)
            bad += int(not np.array_equal(gi[0], oi)) + int(not np.allclose(gd[0], osc, rtol=2e-3))
        parity = {"queries": min(2, args.pairs), "mismatches": bad}
    head = [r for r in rows if abs(r["budget_gb"] - 1.28 * min(1.0, scale * 4)) < 1e-6][0]
    out = {"metric": "lookahead retrieval: hybrid IVF searches/sec with prefetch under a byte budget, 1 GPU",
           "value": round(1e3 / head["search_ms"], 1), "unit": "queries/s", "n_gpus": 1, "steps": args.pairs, "warmup": 0,
           "ms_per_step": head["search_ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f16", "data": "synthetic",
           "config": {"workload": f"configs[3] limited-GPU-memory lookahead: {n} x 768 fp16 in pinned host memory, nlist {nlist}, "
                                  f"nprobe {nprobe}, k {k}, batch 1, device buffer {cap / 1e9:.1f} GB, scale {scale}",
                      "host_threads": threads, "decode_alone_ms": round(decode_alone_ms, 2), "decode_matmuls": reps},
           "budget_sweep": rows, "cluster_cache": cache_rows, "prefetch_scheduler": sched_rows, "parity_sample": parity, "setup_s": round(setup_s, 1)}
    print(json.dumps(out))


def run_batched(args):
    """Batched configurations: configs[2] (c3: 10M x 768 fp16, nlist 4096 Zipf(1.1), nprobe 128, k 10, batch 32
    sharing about 40 % of the probed clusters) and configs[4] (c5: 30M x 1024 bf16, nlist 8192
    Zipf(1.2), nprobe 512, k 100, batch 256 from distinct components), all lists resident in HBM,
    searched list-major.  A step is one whole batch.  One JSON line."""
    import numpy as np
    import torch
    import paper_2502_20969_amd as P
    import workloads as W
    torch.cuda.set_device(0)
    c3 = args.workload == "c3"
    n = int((10_000_000 if c3 else 30_000_000) * args.scale)
    d, nlist, nprobe, k, B = (768, 4096, 128, 10, 32) if c3 else (1024, 8192, 512, 100, 256)
    if args.dim > 0:
        d = args.dim
    if args.batch > 0:
        B = args.batch
    if args.topk > 0:
        k = args.topk
    dtype, zipf = ("f16", 1.1) if c3 else ("bf16", 1.2)
    t0 = time.time()
    sizes = W.zipf_sizes(n, nlist, zipf, 20975 if c3 else 20977)
    ds = W.cluster_major_datastore(sizes, d, 0.3, 20976 if c3 else 20978, dtype=dtype, device="cuda", chunk=1 << 20)
    torch.cuda.synchronize()
    print(f"[{args.workload}] datastore of {n * d * 2 / 1e9:.1f} GB ready after {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
    n_sets = 8                                            # distinct batches cycled through the timed steps
    groups = args.groups if args.groups > 0 else (24 if c3 else B)      # 24 components: measured share 0.40
    qs = [W.shared_batch_queries(ds, B, groups, 20980 + i) for i in range(n_sets)]
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

    def run(nprobe_, steps, warmup):
        index.ivf_set_pipeline_depth(depth)
        for i in range(warmup):
            index.ivf_search_device(qs[i % n_sets], nprobe_, k, ids2[i % depth], dists2[i % depth])
        index.ivf_synchronize()
        t = time.perf_counter()
        for i in range(steps):
            index.ivf_search_device(qs[(warmup + i) % n_sets], nprobe_, k, ids2[i % depth], dists2[i % depth])
        index.ivf_synchronize()
        dt = time.perf_counter() - t
        # kernel durations: one batch at a time, so that no other kernel shares the GPU
        index.ivf_set_pipeline_depth(1)
        if not NO_EVENTS:
            index.ivf_profile_enable(True); index.ivf_profile_reset()
        for i in range(min(steps, n_sets)):
            index.ivf_search_device(qs[i % n_sets], nprobe_, k, ids, dists)
        p = index.ivf_profile_read(); index.ivf_profile_enable(False)
        calls = max(int(p.calls), 1)
        us_scan = p.ms_scan / calls * 1e3
        return {"nprobe": nprobe_, "qps": round(B * steps / dt, 1), "ms_per_batch": round(dt / steps * 1e3, 3),
                "us_scan": round(us_scan, 1), "us_coarse": round(p.ms_coarse / calls * 1e3, 1),
                "us_select": round(p.ms_select / calls * 1e3, 1),
                "scan_gb": round(p.scan_bytes / calls / 1e9, 3),
                "scan_gbs": round((p.scan_bytes / calls / 1e9) / (us_scan / 1e6), 1) if us_scan > 0 else 0.0}

    head = run(nprobe, args.steps if args.steps != 4096 else 16, 2)
    # measured sharing of the batch: 1 - |union of probed clusters| / (B * nprobe)
    pr = index.ivf_probe(qs[0].cpu().numpy(), nprobe)
    share = 1.0 - len(set(pr.reshape(-1).tolist())) / float(pr.size)
    sweep = []
    if not args.no_sweep:
        for np_ in ((16, 32, 64, 128, 256) if c3 else (64, 128, 256, 512)):
            sweep.append(run(np_, 8, 1))
    parity = None
    if not args.no_cpu:
        import oracle as O
        q0 = qs[0].cpu().numpy()
        index.ivf_search_device(qs[0], nprobe, k, ids, dists)
        index.ivf_synchronize()
        gi, gd = ids.cpu().numpy(), dists.cpu().numpy()
        rows_np = ds.rows.cpu().numpy() if c3 else ds.rows.cpu().view(torch.int16).numpy().view(np.uint16)
        off_np, cent_np = ds.offsets.numpy(), ds.centroids.cpu().numpy()
        bad, t1, done = 0, time.perf_counter(), 0
        for b in range(0, B, max(1, B // 4)):               # 4 sampled queries of the batch
            oi, osc = O.search(rows_np, O.F16 if c3 else O.BF16, off_np, None, cent_np, q0[b], nprobe, k, O.IP)
            bad += int(not np.array_equal(gi[b], oi)) + int(not np.allclose(gd[b], osc, rtol=2e-3))
            done += 1
        parity = {"queries": done, "mismatches": bad}
        cpu = {"value": round(done / (time.perf_counter() - t1), 3), "unit": "queries/s", "cores": O.threads(), "kind": "oracle",
               "sample": f"{done} queries of one batch, nprobe {nprobe}, k {k}"}
    out = {"metric": METRIC, "value": head["qps"], "unit": "queries/s", "n_gpus": 1,
           "steps": args.steps if args.steps != 4096 else 16, "warmup": 2, "ms_per_step": head["ms_per_batch"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
           "config": {"workload": f"configs[{2 if c3 else 4}] batched retrieval: {n} x {d} {dtype}, nlist {nlist} Zipf({zipf}), "
                                  f"nprobe {nprobe}, k {k}, batch {B} from {groups} mixture components, scale {args.scale}",
                      "measured_share": round(share, 3), "entry_point": "ivf_search_device (list-major)",
                      "batches_in_flight": depth},
           "roofline": {"bound": "hbm", "achieved": head["scan_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": round(head["scan_gbs"] / HBM_PEAK_GBS, 4),
                        "traffic": ((C3_SCAN_TRAFFIC_BYTES if c3 else C5_SCAN_TRAFFIC_BYTES)
                                    if (args.scale == 1.0 and args.dim == 0 and args.batch == 0 and args.topk == 0
                                        and args.groups == 0) else None),
                        "kernel": "batched_scan_kernel",
                        "us_per_launch": head["us_scan"], "bytes_per_launch": head["scan_gb"] * 1e9},
           "head": head, "nprobe_sweep": sweep, "parity_sample": parity, "setup_s": round(setup_s, 1)}
    if not args.no_cpu:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


def run_paper_shape(args):
    """A resident datastore of the size and shape the paper evaluates on (Sec. 5 set-up: 21 M x 768
    fp32 rows, 4096 clusters, inner product, top-3 retrieval), here with seeded synthetic rows and
    Zipf(1.1) list sizes: nprobe sweep 64..1024 at batch 1, and batches of 2, 4 and 8 independent
    queries per call at nprobe 256.  Parity on sampled queries: the oracle scans, on the host, copies
    of exactly the lists it selects.  One JSON line."""
    import numpy as np
    import torch
    import paper_2502_20969_amd as P
    import workloads as W
    torch.cuda.set_device(0)
    n = int(21_000_000 * args.scale)
    d, nlist, k, nq = 768, 4096, 3, 64
    t0 = time.time()
    sizes = W.zipf_sizes(n, nlist, 1.1, 20985)
    ds = W.cluster_major_datastore(sizes, d, 0.3, 20986, dtype="f32", device="cuda", chunk=1 << 20)
    pick = torch.randint(0, n, (4096,), generator=torch.Generator().manual_seed(20987)).cuda()
    _, q_out = W.query_pairs(ds.rows[pick], nq, 0.3, 20988)
    torch.cuda.synchronize()
    print(f"[n1] datastore of {n * d * 4 / 1e9:.1f} GB ready after {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    cent_np = ds.centroids.cpu().numpy()
    index = P.ivf_adopt_layout(ds.rows, "f32", ds.offsets, cent_np, metric=P.IVF_IP,
                               compute_stream=compute, copy_stream=copy)
    ids = torch.empty(nq, k, dtype=torch.int64, device="cuda")
    dists = torch.empty(nq, k, dtype=torch.float32, device="cuda")
    index.ivf_reserve(8, 1024, k)

    def run(nprobe, B, depth, steps):
        index.ivf_set_pipeline_depth(depth)
        index.ivf_reserve(B, 1024, k)
        def one(i):
            j = (i * B) % nq
            index.ivf_search_device(q_out[j:j + B], nprobe, k, ids[j:j + B], dists[j:j + B])
        for i in range(8):
            one(i)
        index.ivf_synchronize()
        t = time.perf_counter()
        for i in range(steps):
            one(8 + i)
        index.ivf_synchronize()
        dt = time.perf_counter() - t
        index.ivf_set_pipeline_depth(1)
        index.ivf_reserve(B, 1024, k)
        if not NO_EVENTS:
            index.ivf_profile_enable(True); index.ivf_profile_reset()
        for i in range(min(steps, 64)):
            one(i)
        index.ivf_synchronize()
        p = index.ivf_profile_read(); index.ivf_profile_enable(False)
        calls = max(int(p.calls), 1)
        us_scan = p.ms_scan / calls * 1e3
        gbs = (p.scan_bytes / calls / 1e9) / (us_scan / 1e6) if us_scan > 0 else 0.0
        return {"nprobe": nprobe, "batch": B, "searches_in_flight": depth, "qps": round(B * steps / dt, 1),
                "us_scan": round(us_scan, 1), "scan_mb": round(p.scan_bytes / calls / 1e6, 1),
                "scan_gbs": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4)}

    depth = args.depth if args.depth > 0 else 6
    steps = args.steps if args.steps != 4096 else 512
    head = run(256, 1, depth, steps)
    sweep = []
    if not args.no_sweep:
        for nprobe in (64, 128, 256, 512, 1024):
            sweep.append(run(nprobe, 1, depth, max(64, steps * 64 // nprobe)))
        sweep.append(run(256, 1, 1, steps))
        for B in (2, 4, 8):
            sweep.append(run(256, B, 1, max(32, steps // B)))
    parity, cpu = None, None
    if not args.no_cpu:
        import oracle as O
        nprobe = 256
        index.ivf_search_device(q_out, nprobe, k, ids, dists)
        index.ivf_synchronize()
        gi, gd = ids.cpu().numpy(), dists.cpu().numpy()
        q_np = q_out.cpu().numpy()
        off_np = ds.offsets.numpy()
        bad, done, t1, t_oracle = 0, 0, time.perf_counter(), 0.0
        for b in range(0, nq, nq // 4):
            sel = O.probe(cent_np, q_np[b], nprobe, O.IP)
            # a host datastore that holds only the selected lists, under their global row numbers
            coff = np.zeros(nlist + 1, dtype=np.int64)
            cnt = np.zeros(nlist, dtype=np.int64)
            cnt[sel] = off_np[sel + 1] - off_np[sel]
            coff[1:] = np.cumsum(cnt)
            rows = np.empty((int(coff[-1]), d), dtype=np.float32)
            gids = np.empty(int(coff[-1]), dtype=np.int64)
            for c in sel:
                lo, hi = int(off_np[c]), int(off_np[c + 1])
                rows[coff[c]:coff[c + 1]] = ds.rows[lo:hi].cpu().numpy()
                gids[coff[c]:coff[c + 1]] = np.arange(lo, hi)
            t2 = time.perf_counter()
            oi, osc = O.search(rows, O.F32, coff, gids, cent_np, q_np[b], nprobe, k, O.IP)
            t_oracle += time.perf_counter() - t2
            bad += int(not np.array_equal(gi[b], oi)) + int(not np.allclose(gd[b], osc, rtol=1e-4))
            done += 1
        parity = {"queries": done, "mismatches": bad}
        cpu = {"value": round(done / t_oracle, 3), "unit": "queries/s", "cores": O.threads(), "kind": "oracle",
               "sample": f"{done} queries, nprobe {nprobe}, k {k}, lists copied to the host beforehand"}
    out = {"metric": METRIC, "value": head["qps"], "unit": "queries/s", "n_gpus": 1, "steps": steps, "warmup": 8,
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
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4096)
    ap.add_argument("--warmup", type=int, default=512)
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
    ap.add_argument("--metric", default="ip", choices=["ip", "l2"], help="c2: distance function")
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c4", "c5", "n1"],
                    help="c2: single-query retrieval (the default bench line); c4: lookahead with host-resident lists; "
                         "c3 / c5: batched retrieval over fp16 / bf16 lists")
    ap.add_argument("--scale", type=float, default=1.0, help="c3, c4, c5: fraction of the named datastore to build")
    ap.add_argument("--dim", type=int, default=0, help="c3, c5: row dimension instead of the named one (a multiple of 64)")
    ap.add_argument("--batch", type=int, default=0, help="c3, c5: queries per batch instead of the named number")
    ap.add_argument("--topk", type=int, default=0, help="c3, c5: k instead of the named one")
    ap.add_argument("--groups", type=int, default=0, help="c3, c5: mixture components the batch's queries are drawn around")
    ap.add_argument("--pairs", type=int, default=16, help="c4: (q_in, q_out) pairs per budget")
    args = ap.parse_args()
    global NO_EVENTS
    NO_EVENTS = args.no_events
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if args.workload == "c4":
        return run_lookahead(args)
    if args.workload in ("c3", "c5"):
        return run_batched(args)
    if args.workload == "n1":
        return run_paper_shape(args)
    torch.cuda.set_device(0)
    index, stream, rows_host, assign_host, cent_host, q_in, q_out, info = build_config2("cuda", args.n, metric=args.metric)
    nq = q_out.shape[0]
    q_dev = q_out.contiguous()
    ids_dev = torch.empty(nq, args.k, dtype=torch.int64, device="cuda")
    dists_dev = torch.empty(nq, args.k, dtype=torch.float32, device="cuda")
    depth_trials = {}
    if args.depth == 0:
        for depth in (2, 4, 6, 8, 12, 16):
            index.ivf_set_pipeline_depth(depth)
            index.ivf_reserve(1, 1024, args.k)
            t = time_steps(index, stream, q_dev, ids_dev, dists_dev, args.nprobe, args.k, 1500, 100)
            depth_trials[depth] = round(1500 / t, 1)
        args.depth = max(depth_trials, key=depth_trials.get)
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

    # the same searches handed over as host buffers (ivf_search): every call starts from an idle
    # stream, the query is read from pinned host memory and the k results are stored there
    q_host = q_out.cpu().numpy()
    n_host = min(args.steps, 1024)
    for i in range(32):
        index.ivf_search(q_host[i % nq], args.nprobe, args.k)
    t_h = time.perf_counter()
    for i in range(n_host):
        index.ivf_search(q_host[i % nq], args.nprobe, args.k)
    dt_host = time.perf_counter() - t_h

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
                          "scan_mb": round(pr["scan_bytes_per_call"] / 1e6, 2),
                          # selected bytes over the wall time of the whole search, searches in flight as for `value`
                          "e2e_gbs": round(pr["scan_bytes_per_call"] * steps / t / 1e9, 1)})

    out = {
        "metric": METRIC, "value": round(args.steps / dt, 1), "unit": "queries/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"configs[1] single-query retrieval: {args.n} x 768 fp32, 1024-component mixture, "
                               f"nlist 1024 (k-means on a tenth of the rows), nprobe {args.nprobe}, k {args.k}, "
                               f"batch 1, {'inner product' if args.metric == 'ip' else 'squared L2'}, {nq} distinct queries cycled",
                   "entry_point": "ivf_search_device", "searches_in_flight": args.depth,
                   "depth_trials_qps": depth_trials, "seed": 20970},
        "one_at_a_time": {"value": round(args.steps / dt1, 1), "ms_per_step": dt1 / args.steps * 1e3},
        "host_buffers": {"value": round(n_host / dt_host, 1), "ms_per_step": dt_host / n_host * 1e3,
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
        base, (off, perm, lists, results) = cpu_baseline(rows_host, assign_host, cent_host, q_out, args.nprobe, args.k,
                                                         metric=args.metric)
        out["cpu_baseline"] = base
        # the timed outputs of those queries must equal the oracle's
        torch.cuda.synchronize()
        index.ivf_profile_enable(False)
        index.ivf_set_pipeline_depth(args.depth)
        for j in range(nq):
            index.ivf_search_device(q_dev[j], args.nprobe, args.k, ids_dev[j], dists_dev[j])
        index.ivf_synchronize()
        got = ids_dev.cpu().numpy()
        got_d = dists_dev.cpu().numpy().astype(np.float64)
        bad = sum(int(not np.array_equal(got[j], results[j][0])) for j in range(len(results)))
        rel = max(float(np.max(np.abs(got_d[j] - results[j][1]) / np.maximum(np.abs(results[j][1]), 1e-30)))
                  for j in range(len(results)))
        out["parity_sample"] = {"queries": len(results), "id_mismatches": bad, "near_tie_exemptions": 0 if bad == 0 else None,
                                "max_rel_distance_error": rel}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
