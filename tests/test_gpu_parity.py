"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle on the same seeded
inputs -- stage by stage (coarse scores, selected clusters, layout) and end to end."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2502_20969_amd as P
import workloads as W
from parity import check_topk, stored

pytestmark = pytest.mark.gpu

METRIC = {"ip": (P.IVF_IP, O.IP), "l2": (P.IVF_L2, O.L2)}


@pytest.fixture(scope="module")
def streams():
    assert torch.cuda.is_available()
    return torch.cuda.Stream(), torch.cuda.Stream()


def _random_problem(seed, n, d, nlist, dtype, empty=(), dup=0):
    """Clustered random rows with an arbitrary assignment and shuffled ids."""
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((nlist, d)).astype(np.float32)
    assign = rng.integers(0, nlist, n).astype(np.int32)
    for e in empty:
        assign[assign == e] = (e + 1) % nlist
    rows = centres[assign] + 0.5 * rng.standard_normal((n, d)).astype(np.float32)
    rows /= np.linalg.norm(rows, axis=1, keepdims=True)
    if dup:
        src = rng.integers(0, n, dup)
        dst = rng.integers(0, n, dup)
        rows[dst] = rows[src]                      # exact duplicates, possibly across lists
    ids = rng.permutation(n).astype(np.int64) * 3 + 1
    st, odt = stored(rows, dtype)
    return st, odt, centres, assign, ids, rng


def _oracle_layout(st, assign, ids, nlist):
    off, perm = O.build_layout(assign, nlist)
    return st[perm], off, ids[perm]


def _run_case(streams, seed, n, d, nlist, nprobe, k, dtype, metric, nq=5, empty=(), dup=0):
    pm, om = METRIC[metric]
    st, odt, cent, assign, ids, rng = _random_problem(seed, n, d, nlist, dtype, empty, dup)
    index = P.ivf_build_layout(st, dtype, cent, assign, ids=ids, metric=pm,
                               compute_stream=streams[0], copy_stream=streams[1])
    lists, off, lid = _oracle_layout(st, assign, ids, nlist)
    goff, gids = index.ivf_get_layout()
    assert np.array_equal(goff, off) and np.array_equal(gids, lid)
    q = (cent[rng.integers(0, nlist, nq)] + 0.5 * rng.standard_normal((nq, d))).astype(np.float32)
    q /= np.linalg.norm(q, axis=1, keepdims=True)
    # stage: coarse scores and selected clusters
    cs = index.ivf_coarse_scores(q)
    pr = index.ivf_probe(q, nprobe)
    L = min(nprobe, nlist)
    for b in range(nq):
        oc, osc = O.probe(cent, q[b], nlist, om, with_scores=True)
        np.testing.assert_allclose(cs[b][oc], osc, rtol=1e-12, atol=1e-11)
        assert list(pr[b]) == list(oc[:L]), f"query {b}: selected clusters differ"
    # end to end
    gi, gd = index.ivf_search(q, nprobe, k)
    exempt = 0
    for b in range(nq):
        exempt += check_topk(gi[b], gd[b], lists, odt, off, lid, cent, q[b], nprobe, k, om)
    index.close()
    return exempt


# ---- the tiny named workload ------------------------------------------------------------------
def test_config1_tiny(streams):
    ds, q_in, q_out = W.config1_tiny()
    cent = ds.centroids.numpy()
    index = P.ivf_build_layout(ds.rows, "f32", cent, ds.assign, metric=P.IVF_IP,
                               compute_stream=streams[0], copy_stream=streams[1])
    off, perm = O.build_layout(ds.assign.numpy(), 64)
    lists = ds.rows.numpy()[perm]
    goff, gids = index.ivf_get_layout()
    assert np.array_equal(goff, off) and np.array_equal(gids, perm)
    q = q_out.numpy()
    gi, gd = index.ivf_search(q, 8, 10)
    for b in range(16):
        assert list(index.ivf_probe(q[b], 8)[0]) == list(O.probe(cent, q[b], 8, O.IP))
        assert check_topk(gi[b], gd[b], lists, O.F32, off, perm, cent, q[b], 8, 10, O.IP) == 0
    # nprobe = nlist is exhaustive search: compare with a library matmul + argsort
    gi, gd = index.ivf_search(q, 64, 10)
    sc = ds.rows.numpy().astype(np.float64) @ q.astype(np.float64).T
    for b in range(16):
        want = np.lexsort((np.arange(ds.n), -sc[:, b]))[:10]
        assert list(gi[b]) == list(want)
    index.close()


# ---- every scan-kernel shape, dtype and metric ---------------------------------------------------
SHAPES = [  # d per dtype chosen to hit each (lanes per row, segments) variant and the fallback
    ("f32", 64), ("f32", 128), ("f32", 256), ("f32", 384), ("f32", 512), ("f32", 768),
    ("f32", 1024), ("f32", 2048), ("f32", 100), ("f32", 50), ("f32", 7),
    ("f16", 768), ("f16", 128), ("f16", 1024), ("f16", 36), ("f16", 4096),
    ("bf16", 1024), ("bf16", 768), ("bf16", 256), ("bf16", 20),
]


@pytest.mark.parametrize("dtype,d", SHAPES)
@pytest.mark.parametrize("metric", ["ip", "l2"])
def test_shapes(streams, dtype, d, metric):
    n = 6000 if d <= 1024 else 1500
    exempt = _run_case(streams, 100 + d, n, d, 24, 6, 10, dtype, metric, nq=4, empty=(3,))
    assert exempt == 0


def test_ragged_lists_many_tiles(streams):
    """Lists from 0 rows to thousands of rows: many tasks per list and ragged tails."""
    rng = np.random.default_rng(5)
    nlist, d = 40, 768
    sizes = np.concatenate([[0, 1, 2, 7, 8, 9, 15, 16, 17, 63, 64, 65], rng.integers(100, 3000, nlist - 12)])
    assign = np.repeat(np.arange(nlist), sizes).astype(np.int32)
    rng.shuffle(assign)
    n = assign.shape[0]
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    rows = (cent[assign] + 0.7 * rng.standard_normal((n, d))).astype(np.float32)
    index = P.ivf_build_layout(rows, "f32", cent, assign, metric=P.IVF_IP,
                               compute_stream=streams[0], copy_stream=streams[1])
    off, perm = O.build_layout(assign, nlist)
    lists = rows[perm]
    q = rng.standard_normal((6, d)).astype(np.float32)
    for nprobe in (1, 12, 40):
        gi, gd = index.ivf_search(q, nprobe, 10)
        for b in range(6):
            assert check_topk(gi[b], gd[b], lists, O.F32, off, perm, cent, q[b], nprobe, 10, O.IP) == 0
    index.close()


# ---- selection paths ------------------------------------------------------------------------------
@pytest.mark.parametrize("nlist,nprobe", [(1, 1), (2, 5), (2048, 64), (2049, 33), (5000, 300), (6000, 3000), (3000, 3000)])
def test_select_paths(streams, nlist, nprobe):
    """Full sort in LDS (nlist <= 2048), radix select + LDS sort, and the global-memory sort."""
    n = max(nlist * 2, 4000)
    assert _run_case(streams, 7 + nlist, n, 32, nlist, nprobe, 5, "f32", "ip", nq=3) == 0


def test_equal_centroid_scores_pick_lower_index(streams):
    """Duplicate centroids give bit-equal coarse scores; the boundary must take lower indices."""
    rng = np.random.default_rng(2)
    d = 16
    for nlist, reps in ((12, 4), (4000, 100)):
        base = rng.standard_normal((nlist // reps, d)).astype(np.float32)
        cent = np.tile(base, (reps, 1))
        n = nlist * 3
        assign = (np.arange(n) % nlist).astype(np.int32)
        rows = rng.standard_normal((n, d)).astype(np.float32)
        index = P.ivf_build_layout(rows, "f32", cent, assign, compute_stream=streams[0], copy_stream=streams[1])
        q = rng.standard_normal((3, d)).astype(np.float32)
        for nprobe in (1, reps // 2 + 1, reps + 2):
            pr = index.ivf_probe(q, nprobe)
            for b in range(3):
                assert list(pr[b]) == list(O.probe(cent, q[b], nprobe, O.IP))
        index.close()


# ---- ties, k limits, padding -------------------------------------------------------------------------
def test_exact_duplicates_ordered_by_id(streams):
    assert _run_case(streams, 31, 5000, 128, 16, 16, 20, "f32", "ip", nq=4, dup=2500) == 0
    assert _run_case(streams, 32, 5000, 768, 16, 5, 10, "f16", "l2", nq=4, dup=2500) == 0


def test_all_rows_identical(streams):
    n, d, nlist = 3000, 64, 8
    rows = np.tile(np.linspace(-1, 1, d, dtype=np.float32), (n, 1))
    rng = np.random.default_rng(4)
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    assign = rng.integers(0, nlist, n).astype(np.int32)
    ids = rng.permutation(n).astype(np.int64)
    index = P.ivf_build_layout(rows, "f32", cent, assign, ids=ids, compute_stream=streams[0], copy_stream=streams[1])
    q = rng.standard_normal((2, d)).astype(np.float32)
    gi, gd = index.ivf_search(q, 3, 25)
    off, perm = O.build_layout(assign, nlist)
    for b in range(2):
        oi, _ = O.search(rows[perm], O.F32, off, ids[perm], cent, q[b], 3, 25, O.IP)
        assert list(gi[b]) == list(oi)
    index.close()


@pytest.mark.parametrize("k", [1, 56, 57, 100, 112])
def test_k_range(streams, k):
    assert _run_case(streams, 40 + k, 8000, 256, 12, 4, k, "f32", "ip", nq=3) == 0


def test_padding_and_clamp(streams):
    rng = np.random.default_rng(8)
    n, d, nlist = 9, 32, 4
    rows = rng.standard_normal((n, d)).astype(np.float32)
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    assign = np.array([0, 0, 0, 1, 1, 1, 1, 3, 3], dtype=np.int32)
    for pm, om in METRIC.values():
        index = P.ivf_build_layout(rows, "f32", cent, assign, metric=pm, compute_stream=streams[0], copy_stream=streams[1])
        off, perm = O.build_layout(assign, nlist)
        q = rng.standard_normal((2, d)).astype(np.float32)
        for nprobe in (1, 2, 1000):
            gi, gd = index.ivf_search(q, nprobe, 12)
            for b in range(2):
                check_topk(gi[b], gd[b], rows[perm], O.F32, off, perm, cent, q[b], nprobe, 12, om, extra=0)
        index.close()


def test_error_codes_on_live_index(streams):
    rng = np.random.default_rng(1)
    rows = rng.standard_normal((100, 16)).astype(np.float32)
    cent = rng.standard_normal((4, 16)).astype(np.float32)
    index = P.ivf_build_layout(rows, "f32", cent, rng.integers(0, 4, 100).astype(np.int32),
                               compute_stream=streams[0], copy_stream=streams[1])
    q = rows[:1]
    for bad in (dict(nprobe=0, k=1), dict(nprobe=1, k=0)):
        with pytest.raises(P.IvfError) as e:
            index.ivf_search(q, bad["nprobe"], bad["k"])
        assert e.value.status == -1
    with pytest.raises(P.IvfError) as e:
        index.ivf_search(q, 1, P.IVF_MAX_K + 1)
    assert e.value.status == -5
    with pytest.raises(P.IvfError) as e:
        index.ivf_prefetch(q, 1, 100)
    assert e.value.status == -4
    index.close()


# ---- device-pointer entry point and adopted layouts ----------------------------------------------------
def test_search_device_and_adopt(streams):
    ds, _, q_out = W.config2_single_query(seed=3, n=40000, d=768, nlist=64, nq=12)
    off, perm = O.build_layout(ds.assign.numpy(), 64)
    lists = ds.rows.numpy()[perm]
    cent = ds.centroids.numpy()
    lists_dev = torch.from_numpy(lists).cuda()
    index = P.ivf_adopt_layout(lists_dev, "f32", off, cent, ids=perm, metric=P.IVF_IP,
                               compute_stream=streams[0], copy_stream=streams[1])
    q = q_out.numpy()
    hi, hd = index.ivf_search(q, 8, 10)
    q_dev = q_out.cuda()
    ids_dev = torch.empty(12, 10, dtype=torch.int64, device="cuda")
    d_dev = torch.empty(12, 10, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    # one query per call, as the single-query benchmark does
    for b in range(12):
        index.ivf_search_device(q_dev[b], 8, 10, ids_dev[b], d_dev[b])
    streams[0].synchronize()
    assert np.array_equal(ids_dev.cpu().numpy(), hi) and np.array_equal(d_dev.cpu().numpy(), hd)
    for b in range(12):
        assert check_topk(hi[b], hd[b], lists, O.F32, off, perm, cent, q[b], 8, 10, O.IP) == 0
    # several searches in flight on the library's own streams give the same results
    index.ivf_set_pipeline_depth(3)
    ids2 = torch.zeros_like(ids_dev)
    d2 = torch.zeros_like(d_dev)
    torch.cuda.synchronize()
    for rep in range(3):
        for b in range(12):
            index.ivf_search_device(q_dev[b], 8, 10, ids2[b], d2[b])
    index.ivf_synchronize()
    assert np.array_equal(ids2.cpu().numpy(), hi) and np.array_equal(d2.cpu().numpy(), hd)
    hi2, hd2 = index.ivf_search(q, 8, 10)        # host entry point while lanes exist
    assert np.array_equal(hi2, hi) and np.array_equal(hd2, hd)
    index.ivf_set_pipeline_depth(1)
    # profiling counters: rows covered equal the rows of the selected lists
    index.ivf_profile_enable(True)
    index.ivf_profile_reset()
    index.ivf_search_device(q_dev[0], 8, 10, ids_dev[0], d_dev[0])
    p = index.ivf_profile_read()
    want_rows = sum(int(off[c + 1] - off[c]) for c in O.probe(cent, q[0], 8, O.IP))
    assert p.calls == 1 and p.scan_rows == want_rows and p.scan_bytes == want_rows * 768 * 4
    assert p.ms_scan > 0
    index.ivf_profile_enable(False)
    index.close()


@pytest.mark.parametrize("dtype,d,n", [("f32", 32, 4500), ("f32", 64, 4500), ("f16", 128, 4500), ("f32", 96, 4500),
                                       ("f16", 256, 4500), ("f32", 768, 4500), ("bf16", 1024, 4500), ("f32", 100, 4500),
                                       ("f16", 36, 4500), ("f32", 768, 9500), ("f16", 512, 20000)])
def test_every_row_is_found_by_its_own_query(streams, dtype, d, n):
    """Coverage of the scan: with every list selected, the stored row itself is the nearest
    neighbour of its own values (normalised, distinct rows; inner product), whichever workgroup
    and wavefront its place in the row sequence falls to.  All rows are asked, in calls of 512
    queries (scan grids of 512 queries) and, for every 11th row, one query per call; lists are
    ragged and some are empty; the two largest cases fill the whole scan grid of a single query.
    Expected ids come from a float64 Gram matrix of the stored rows."""
    nlist = 9
    st, odt, cent, assign, ids, rng = _random_problem(1000 + d, n, d, nlist, dtype, empty=(2, 5))
    index = P.ivf_build_layout(st, dtype, cent, assign, ids=ids, metric=P.IVF_IP,
                               compute_stream=streams[0], copy_stream=streams[1])
    if dtype == "bf16":
        wide = torch.from_numpy(st.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    else:
        wide = st.astype(np.float64)
    self_ip = np.einsum("ij,ij->i", wide, wide)
    for lo in range(0, n, 1000):                      # the case is what it claims: every row wins its own query
        assert np.array_equal(np.argmax(wide[lo:lo + 1000] @ wide.T, axis=1), np.arange(lo, min(lo + 1000, n)))
    q = wide.astype(np.float32)                       # exact: stored values fit float32
    index.ivf_set_batch_mode(1)                       # query by query, also inside one call
    for lo in range(0, n, 512):
        gi, gd = index.ivf_search(q[lo:lo + 512], nlist, 1)
        assert np.array_equal(gi[:, 0], ids[lo:lo + 512]), f"rows {lo}..: {np.flatnonzero(gi[:, 0] != ids[lo:lo + 512])[:8] + lo}"
    for i in range(0, n, 11):
        gi, gd = index.ivf_search(q[i], nlist, 1)
        assert gi[0, 0] == ids[i], f"row {i}"
        np.testing.assert_allclose(gd[0, 0], self_ip[i], rtol=2e-3 if dtype != "f32" else 1e-4)
    index.close()
