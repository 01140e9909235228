"""Seeded random configurations of the whole path against the oracle: shapes, storage types,
metrics, placements, id kinds, duplicates and empty lists drawn together, so that combinations no
hand-written case names are still exercised.  Every case is a fixed seed."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2502_20969_amd as P
import workloads as W
from parity import check_topk, stored

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def streams():
    assert torch.cuda.is_available()
    return torch.cuda.Stream(), torch.cuda.Stream()


@pytest.mark.parametrize("seed", range(60))
def test_random_search_case(streams, seed):
    rng = np.random.default_rng(9000 + seed)
    dtype = str(rng.choice(["f32", "f16", "bf16"]))
    metric = str(rng.choice(["ip", "l2"]))
    d = int(rng.choice([4, 7, 16, 24, 40, 64, 96, 100, 128, 200, 256, 384, 512, 768, 1024]))
    nlist = int(rng.choice([1, 2, 5, 17, 64, 100, 333, 1024, 1500, 3000]))
    n = int(rng.integers(max(1, nlist // 2), 25000))
    nprobe = int(rng.choice([1, 2, 3, 8, 31, 32, 63, 64, 65, 100, 400, 5000]))
    k = int(rng.choice([1, 2, 5, 10, 33, 56, 57, 64, 100, 112]))
    nq = int(rng.choice([1, 1, 2, 3, 5, 9, 17, 40]))
    placement = str(rng.choice(["device", "device", "host"]))
    idkind = str(rng.choice(["none", "perm", "sparse"]))
    dup = int(rng.choice([0, 0, n // 3, n]))
    pm, om = (P.IVF_IP, O.IP) if metric == "ip" else (P.IVF_L2, O.L2)
    centres = rng.standard_normal((nlist, d)).astype(np.float32)
    assign = rng.integers(0, nlist, n).astype(np.int32)
    if rng.random() < 0.3 and nlist > 2:
        assign[assign == 1] = 0                      # an empty list
    rows = centres[assign] + 0.5 * rng.standard_normal((n, d)).astype(np.float32)
    if dup:
        rows[rng.integers(0, n, dup)] = rows[rng.integers(0, n, dup)]
    ids = None if idkind == "none" else (rng.permutation(n).astype(np.int64) if idkind == "perm"
                                         else rng.permutation(n).astype(np.int64) * 7 + 3)
    st, odt = stored(rows, dtype)
    esz = 4 if dtype == "f32" else 2
    kw = {}
    if placement == "host":
        kw = dict(placement=P.IVF_PLACE_HOST, device_buffer_bytes=int(n * d * esz * rng.choice([0.0, 0.3, 1.0])) + 64)
    index = P.ivf_build_layout(st, dtype, centres, assign, ids=ids, metric=pm, compute_stream=streams[0],
                               copy_stream=streams[1], **kw)
    off, perm = O.build_layout(assign, nlist)
    lists = st[perm]
    lid = perm.astype(np.int64) if ids is None else ids[perm]
    q = (centres[rng.integers(0, nlist, nq)] + 0.5 * rng.standard_normal((nq, d))).astype(np.float32)
    if placement == "host":
        index.ivf_prefetch(q, nprobe, int(n * d * esz * rng.choice([0.1, 0.5, 2.0])), flags=P.IVF_PREFETCH_RESET)
    pr = index.ivf_probe(q, nprobe)
    for b in range(nq):
        assert list(pr[b]) == list(O.probe(centres, q[b], nprobe, om))
    gi, gd = index.ivf_search(q, nprobe, k)
    exempt = 0
    for b in range(nq):
        exempt += check_topk(gi[b], gd[b], lists, odt, off, lid, centres, q[b], nprobe, k, om)
    assert exempt == 0
    if placement == "device":
        q_dev = torch.from_numpy(q).cuda()
        ids_dev = torch.empty(nq, k, dtype=torch.int64, device="cuda")
        d_dev = torch.empty(nq, k, device="cuda")
        torch.cuda.synchronize()
        index.ivf_search_device(q_dev, nprobe, k, ids_dev, d_dev)
        index.ivf_synchronize()
        assert np.array_equal(ids_dev.cpu().numpy(), gi) and np.array_equal(d_dev.cpu().numpy(), gd)
    index.close()


@pytest.mark.parametrize("seed", range(64))
def test_random_batched_case(streams, seed):
    """List-major batched search: equal to the oracle and, bit for bit, to the query-by-query path.
    The first 24 seeds are 2-byte rows with the inner product; the later ones draw fp32 rows and
    squared L2 as well."""
    rng = np.random.default_rng(9500 + seed)
    dtype = str(rng.choice(["f16", "bf16"]))
    metric = "ip"
    if seed >= 24:
        rng2 = np.random.default_rng(9700 + seed)
        dtype = str(rng2.choice(["f32", "f32", "f16", "bf16"]))
        metric = str(rng2.choice(["ip", "l2"])) if dtype != "f32" else str(rng2.choice(["ip", "l2", "l2"]))
    pm, om = (P.IVF_IP, O.IP) if metric == "ip" else (P.IVF_L2, O.L2)
    d = int(rng.choice([64, 128, 192, 256, 768, 1024]))
    nlist = int(rng.choice([3, 16, 64, 200, 1000]))
    n = int(rng.integers(nlist, 40000))
    nprobe = int(rng.choice([1, 4, 16, 64, 100]))
    k = int(rng.choice([1, 10, 50, 100]))
    nq = int(rng.choice([2, 4, 7, 32, 33, 70]))
    zipf = float(rng.choice([0.0, 1.1, 1.5]))
    sizes = W.zipf_sizes(n, nlist, zipf, 9500 + seed, min_rows=int(rng.choice([0, 1])))
    ds = W.cluster_major_datastore(sizes, d, 0.4, 9600 + seed, dtype=dtype)
    rows = ds.rows.float().numpy()
    if rng.random() < 0.4:
        rows[rng.integers(0, n, n // 2)] = rows[rng.integers(0, n, n // 2)]
    st, odt = stored(rows, dtype)
    off, cent = ds.offsets.numpy(), ds.centroids.numpy()
    ids = None if rng.random() < 0.5 else rng.permutation(n).astype(np.int64) * 3 + 1
    t = torch.from_numpy(st.view(np.int16) if dtype == "bf16" else st).cuda()
    if dtype == "bf16":
        t = t.view(torch.bfloat16)
    index = P.ivf_adopt_layout(t, dtype, off, cent, ids=ids, metric=pm, compute_stream=streams[0],
                               copy_stream=streams[1])
    q = (cent[rng.integers(0, nlist, nq)] + 0.3 * rng.standard_normal((nq, d))).astype(np.float32)
    index.ivf_set_batch_mode(2)
    gi, gd, stats = index.ivf_search(q, nprobe, k, with_stats=True)
    union = set()
    for b in range(nq):
        union |= set(O.probe(cent, q[b], nprobe, om))
    assert stats.bytes_gpu == sum(int(off[c + 1] - off[c]) for c in union) * d * st.itemsize   # each list read once
    exempt = 0
    for b in range(nq):
        exempt += check_topk(gi[b], gd[b], st, odt, off, ids, cent, q[b], nprobe, k, om)
    assert exempt == 0
    index.ivf_set_batch_mode(1)
    hi, hd = index.ivf_search(q, nprobe, k)
    assert np.array_equal(gi, hi) and np.array_equal(gd, hd)
    index.close()


@pytest.mark.parametrize("seed", range(12))
def test_random_cache_rounds(streams, seed):
    """Prefetch, search and end-of-round over random cache parameters, against the oracle's cache round."""
    rng = np.random.default_rng(9700 + seed)
    dtype = str(rng.choice(["f32", "f16"]))
    d = int(rng.choice([32, 96, 256]))
    nlist = int(rng.choice([8, 40, 150]))
    n = int(rng.integers(nlist * 20, 30000))
    L, k = int(rng.choice([2, 6, 16])), 10
    fraction = float(rng.choice([0.0, 0.25, 0.5, 1.0]))
    decay = float(rng.choice([1.0, 2.0, 3.0]))
    h_inc = float(rng.choice([0.0, 0.5, 1.0]))
    sizes = W.zipf_sizes(n, nlist, 1.1, 9700 + seed)
    ds = W.cluster_major_datastore(sizes, d, 0.4, 9800 + seed, dtype=dtype)
    off, cent = ds.offsets.numpy(), ds.centroids.numpy()
    st, odt = stored(ds.rows.float().numpy(), dtype)
    bsz = np.diff(off) * d * (4 if dtype == "f32" else 2)
    cap = int(bsz.sum() * rng.choice([0.3, 0.6, 1.0]))
    index = P.ivf_adopt_layout(ds.rows.pin_memory(), dtype, off, cent, metric=P.IVF_IP, placement=P.IVF_PLACE_HOST,
                               device_buffer_bytes=cap, compute_stream=streams[0], copy_stream=streams[1])
    index.ivf_cache_configure(fraction, 1.0, decay, h_inc)
    res = O.Residency(nlist, cap)
    hot = np.full(nlist, -1.0, np.float32)
    used = np.zeros(nlist, np.uint8)
    for rnd in range(6):
        q = (cent[rng.integers(0, nlist)] + 0.2 * rng.standard_normal(d)).astype(np.float32)
        budget = int(bsz.sum() * rng.choice([0.05, 0.2, 0.5]))
        chosen, skipped, nbytes = O.prefetch(cent, off, odt, q, L, budget, res, O.IP)
        O.cache_admit(hot, res, 1.0)
        ps = index.ivf_prefetch(q, L, budget)
        assert (ps.n_taken, ps.n_skipped, ps.bytes) == (len(chosen), skipped, nbytes)
        gi, gd = index.ivf_search(q, L, k)
        ov, _ = O.split(cent, q, L, res.flags, O.IP)
        used[ov] = 1
        assert check_topk(gi[0], gd[0], st, odt, off, None, cent, q, L, k, O.IP) == 0
        ev = O.cache_round(hot, used, res, off, d, odt, decay, h_inc, fraction)
        cs = index.ivf_cache_end_round()
        assert cs.n_evicted == len(ev) and cs.bytes_kept == res.used.value
        assert np.array_equal(index.ivf_cache_hotness(), hot)
        assert list(index.ivf_resident()) == list(res.clusters())
        gi, gd = index.ivf_search(q, L, k)
        ov, _ = O.split(cent, q, L, res.flags, O.IP)
        used[ov] = 1
        assert check_topk(gi[0], gd[0], st, odt, off, None, cent, q, L, k, O.IP) == 0
    index.close()
