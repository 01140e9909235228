"""Parity at the named sizes of the benchmark configurations, in the launch configuration
bench.py times: configs[2] (10 M x 768 fp16, batch 32, list-major), configs[4] (30 M x 1024 bf16,
k 100, batch 256, list-major), configs[3] (lookahead over pinned host lists, at the largest size
the host pins) and the paper's resident shape (21 M x 768 fp32, k 3, batches of 1 and 8, both
distances).  Rows are generated on the GPU; for each sampled query the oracle selects its clusters
itself, exactly those lists are copied to the host, and the oracle's result over them is compared
element by element.  Three of the four datastores lie beyond 4 GiB byte offsets."""
import gc
import time

import numpy as np
import pytest
import torch

import oracle as O
import paper_2502_20969_amd as P
import workloads as W
from parity import compare_topk, oracle_search_selected

pytestmark = pytest.mark.gpu


def _free():
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    W.release_pinned_cache()


def _check_queries(gi, gd, rows_t, odt, off, cent, q_np, which, nprobe, k, metric, index=None):
    """Element-by-element comparison of the sampled queries; also the selected clusters."""
    exempt = 0
    for b in which:
        oi, osc, sel = oracle_search_selected(rows_t, odt, off, cent, q_np[b], nprobe, k, metric)
        exempt += compare_topk(gi[b], gd[b], oi, osc, k, odt, metric)
        if index is not None:
            assert np.array_equal(index.ivf_probe(q_np[b], nprobe)[0], sel), f"query {b}: selected clusters differ"
    return exempt


def _check_shape_properties(gi, gd, metric):
    assert np.all(gi >= 0)
    assert all(len(set(r)) == len(r) for r in gi)
    step = np.diff(gd.astype(np.float64), axis=1)
    assert np.all(step <= 0) if metric == O.IP else np.all(step >= 0)


def test_config2_mid_fp16_batch_32():
    t0 = time.time()
    ds, batches = W.config3_mid_fp16(device="cuda", n_sets=2)
    assert ds.n == 10_000_000 and ds.rows.element_size() * ds.rows.numel() > (4 << 30)
    off, cent = ds.offsets.numpy(), ds.centroids.cpu().numpy()
    index = P.ivf_adopt_layout(ds.rows, "f16", off, cent, metric=P.IVF_IP,
                               compute_stream=torch.cuda.Stream(), copy_stream=torch.cuda.Stream())
    nprobe, k, B = 128, 10, 32
    index.ivf_set_batch_mode(2)
    index.ivf_set_pipeline_depth(2)               # two batches in flight, as timed
    index.ivf_reserve(B, nprobe, k)
    ids = torch.full((2, B, k), -7, dtype=torch.int64, device="cuda")
    dists = torch.zeros(2, B, k, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    for rep in range(2):
        for j in range(2):
            index.ivf_search_device(batches[j], nprobe, k, ids[j], dists[j])
    index.ivf_synchronize()
    gi, gd = ids.cpu().numpy(), dists.cpu().numpy()
    exempt = 0
    for j in range(2):
        _check_shape_properties(gi[j], gd[j], O.IP)
        q_np = batches[j].cpu().numpy()
        exempt += _check_queries(gi[j], gd[j], ds.rows, O.F16, off, cent, q_np, range(j, B, 8), nprobe, k, O.IP,
                                 index if j == 0 else None)
    assert exempt == 0
    # measured sharing of the probed clusters: 1 - |union| / (B * nprobe); the config names about 0.4
    pr = index.ivf_probe(batches[0].cpu().numpy(), nprobe)
    share = 1.0 - len(set(pr.reshape(-1).tolist())) / float(pr.size)
    print(f"configs[2]: share {share:.3f}, {time.time() - t0:.1f} s")
    assert 0.3 < share < 0.5
    # the query-by-query path gives the same answers for the whole batch
    index.ivf_set_pipeline_depth(1)
    index.ivf_set_batch_mode(1)
    ids1 = torch.empty(B, k, dtype=torch.int64, device="cuda")
    dists1 = torch.empty(B, k, dtype=torch.float32, device="cuda")
    index.ivf_search_device(batches[0], nprobe, k, ids1, dists1)
    index.ivf_synchronize()
    assert torch.equal(ids1, ids[0]) and torch.equal(dists1, dists[0])
    index.close()
    del ds, batches, ids, dists
    _free()


def test_config4_large_bf16_k100_batch_256():
    t0 = time.time()
    ds, batches = W.config5_large_bf16(device="cuda", n_sets=2)
    assert ds.n == 30_000_000 and ds.d == 1024
    off, cent = ds.offsets.numpy(), ds.centroids.cpu().numpy()
    index = P.ivf_adopt_layout(ds.rows, "bf16", off, cent, metric=P.IVF_IP,
                               compute_stream=torch.cuda.Stream(), copy_stream=torch.cuda.Stream())
    nprobe, k, B = 512, 100, 256
    index.ivf_set_batch_mode(2)
    index.ivf_set_pipeline_depth(2)
    index.ivf_reserve(B, nprobe, k)
    ids = torch.full((2, B, k), -7, dtype=torch.int64, device="cuda")
    dists = torch.zeros(2, B, k, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    for j in range(2):
        index.ivf_search_device(batches[j], nprobe, k, ids[j], dists[j])
    index.ivf_synchronize()
    gi, gd = ids.cpu().numpy(), dists.cpu().numpy()
    exempt = 0
    for j in range(2):
        _check_shape_properties(gi[j], gd[j], O.IP)
        q_np = batches[j].cpu().numpy()
        exempt += _check_queries(gi[j], gd[j], ds.rows, O.BF16, off, cent, q_np, range(17 * j, B, 64), nprobe, k, O.IP,
                                 index if j == 0 else None)
    assert exempt == 0
    print(f"configs[4]: 8 queries of 2 batches equal to the oracle, {time.time() - t0:.1f} s")
    index.close()
    del ds, batches, ids, dists
    _free()


def test_config3_lookahead_host_lists():
    t0 = time.time()
    pinned, scale, note = W.pinned_rows(60_000_000, 768, "f16")
    nlist = max(64, int(16384 * scale))
    nprobe, k, pairs = 256, 10, 6
    ds, q_in, q_out = W.config4_lookahead(pinned, nlist, pairs)
    torch.cuda.synchronize()
    print(f"configs[3]: {pinned.shape[0]} rows pinned (scale {scale}; {note}), ready after {time.time() - t0:.1f} s")
    assert pinned.element_size() * pinned.numel() > (4 << 30)
    off, cent = ds.offsets.numpy(), ds.centroids.cpu().numpy()
    cap = int(8e9)
    index = P.ivf_adopt_layout(pinned, "f16", off, cent, metric=P.IVF_IP, placement=P.IVF_PLACE_HOST,
                               device_buffer_bytes=cap, compute_stream=torch.cuda.Stream(), copy_stream=torch.cuda.Stream())
    index.ivf_set_host_threads(16)
    qi, qo = q_in.numpy(), q_out.numpy()
    sizes = np.diff(off) * 768 * 2
    exempt = 0
    for budget in (0, int(1.28e9), 1 << 40):
        for b in range(pairs):
            res = O.Residency(nlist, cap)
            chosen, skipped, nbytes = O.prefetch(cent, off, O.F16, qi[b], nprobe, budget, res, O.IP)
            ps = index.ivf_prefetch(qi[b], nprobe, budget, flags=P.IVF_PREFETCH_RESET)
            assert ps.n_taken == len(chosen) and ps.n_skipped == skipped and ps.bytes == nbytes
            assert list(index.ivf_resident()) == list(res.clusters())
            gi, gd, ss = index.ivf_search(qo[b], nprobe, k, with_stats=True)      # copies still in flight
            ov, ms = O.split(cent, qo[b], nprobe, res.flags, O.IP)
            assert ss.n_overlap == len(ov) and ss.n_miss == len(ms)
            assert ss.bytes_gpu == sizes[ov].sum() and ss.bytes_host == sizes[ms].sum()
            oi, osc, sel = oracle_search_selected(pinned, O.F16, off, cent, qo[b], nprobe, k, O.IP)
            assert set(sel.tolist()) == set(ov.tolist()) | set(ms.tolist())
            exempt += compare_topk(gi[0], gd[0], oi, osc, k, O.F16, O.IP)
    assert exempt == 0
    index.close()
    del ds, pinned
    _free()


def test_paper_shape_fp32_k3_both_distances():
    t0 = time.time()
    ds, q_out = W.paper_shape_fp32(device="cuda")
    assert ds.n == 21_000_000 and ds.rows.element_size() * ds.rows.numel() > (60 << 30)
    off, cent = ds.offsets.numpy(), ds.centroids.cpu().numpy()
    nq, k, nprobe = q_out.shape[0], 3, 256
    q_np = q_out.cpu().numpy()
    for pm, om in ((P.IVF_IP, O.IP), (P.IVF_L2, O.L2)):
        index = P.ivf_adopt_layout(ds.rows, "f32", off, cent, metric=pm,
                                   compute_stream=torch.cuda.Stream(), copy_stream=torch.cuda.Stream())
        ids = torch.full((nq, k), -7, dtype=torch.int64, device="cuda")
        dists = torch.zeros(nq, k, dtype=torch.float32, device="cuda")
        # batch 1, six searches in flight (as timed); then the same queries in batches of 8
        index.ivf_set_pipeline_depth(6)
        index.ivf_reserve(8, 1024, k)
        torch.cuda.synchronize()
        for j in range(nq):
            index.ivf_search_device(q_out[j], nprobe, k, ids[j], dists[j])
        index.ivf_synchronize()
        gi, gd = ids.cpu().numpy(), dists.cpu().numpy()
        _check_shape_properties(gi, gd, om)
        assert _check_queries(gi, gd, ds.rows, O.F32, off, cent, q_np, range(0, nq, 8), nprobe, k, om, index) == 0
        index.ivf_set_pipeline_depth(1)
        ids8 = torch.full((nq, k), -7, dtype=torch.int64, device="cuda")
        dists8 = torch.zeros(nq, k, dtype=torch.float32, device="cuda")
        for j in range(0, nq, 8):
            index.ivf_search_device(q_out[j:j + 8], nprobe, k, ids8[j:j + 8], dists8[j:j + 8])
        index.ivf_synchronize()
        assert torch.equal(ids8, ids) and torch.equal(dists8, dists)
        # the other nprobe values of the sweep, one sampled query each
        for np_, b in ((64, 3), (1024, 5)):
            index.ivf_search_device(q_out[b], np_, k, ids8[b], dists8[b])
            index.ivf_synchronize()
            oi, osc, _ = oracle_search_selected(ds.rows, O.F32, off, cent, q_np[b], np_, k, om)
            assert compare_topk(ids8[b].cpu().numpy(), dists8[b].cpu().numpy(), oi, osc, k, O.F32, om) == 0
        index.close()
        print(f"paper shape, metric {om}: ok after {time.time() - t0:.1f} s")
    del ds
    _free()
