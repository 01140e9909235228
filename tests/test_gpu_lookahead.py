"""GPU parity of lookahead retrieval (Sec. 4.1 steps 1-4, Sec. 4.3 'Prefetching target'): prefetch
plan, residency, overlap/miss split and the hybrid GPU + host search, against the oracle."""
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


def _problem(seed, n, d, nlist, dtype):
    sizes = W.zipf_sizes(n, nlist, 1.1, seed)
    ds = W.cluster_major_datastore(sizes, d, 0.4, seed + 1, dtype=dtype)
    q_in, q_out = W.query_pairs(ds.rows.float(), 6, 0.3, seed + 2)
    return ds, q_in.numpy(), q_out.numpy()


@pytest.mark.parametrize("dtype,metric", [("f16", "ip"), ("f32", "l2"), ("bf16", "ip")])
def test_prefetch_plan_and_hybrid_search(streams, dtype, metric):
    pm, om = {"ip": (P.IVF_IP, O.IP), "l2": (P.IVF_L2, O.L2)}[metric]
    n, d, nlist, L, k = 30000, 256, 48, 12, 10
    ds, q_in, q_out = _problem(50, n, d, nlist, dtype)
    off = ds.offsets.numpy()
    cent = ds.centroids.numpy()
    lists_pinned = ds.rows.pin_memory()
    st, odt = stored(ds.rows.float().numpy(), dtype)
    esz = 4 if dtype == "f32" else 2
    cap = int(n * d * esz // 3)
    index = P.ivf_adopt_layout(lists_pinned, dtype, off, cent, metric=pm, placement=P.IVF_PLACE_HOST,
                               device_buffer_bytes=cap, compute_stream=streams[0], copy_stream=streams[1])
    sizes = np.diff(off) * d * esz
    total_exempt = 0
    for b in range(q_in.shape[0]):
        for budget in (0, int(sizes[sizes > 0].min()), int(sizes.sum() // 10), 1 << 40):
            res = O.Residency(nlist, cap)
            chosen, skipped, nbytes = O.prefetch(cent, off, odt, q_in[b], L, budget, res, om)
            ps = index.ivf_prefetch(q_in[b], L, budget, flags=P.IVF_PREFETCH_RESET)
            assert ps.n_taken == len(chosen) and ps.n_skipped == skipped and ps.bytes == nbytes
            assert ps.buffer_used == res.used.value
            assert list(index.ivf_resident()) == list(res.clusters())
            # search right away: the copies are certainly still in flight
            gi, gd, ss = index.ivf_search(q_out[b], L, k, with_stats=True)
            ov, ms = O.split(cent, q_out[b], L, res.flags, om)
            assert ss.n_overlap == len(ov) and ss.n_miss == len(ms) and ss.n_probed == len(ov) + len(ms)
            _, _, hr = O.hybrid(st, odt, off, None, cent, q_out[b], L, k, res.flags, om)
            assert abs(ss.hit_rate - hr) < 1e-6
            assert ss.bytes_gpu == sizes[ov].sum() and ss.bytes_host == sizes[ms].sum()
            total_exempt += check_topk(gi[0], gd[0], st, odt, off, None, cent, q_out[b], L, k, om)
    assert total_exempt == 0
    # incremental prefetch (no reset): resident clusters are not copied again
    res = O.Residency(nlist, cap)
    index.ivf_prefetch(q_in[0], L, 1 << 40, flags=P.IVF_PREFETCH_RESET)
    O.prefetch(cent, off, odt, q_in[0], L, 1 << 40, res, om)
    ps = index.ivf_prefetch(q_out[0], L, 1 << 40)
    chosen, skipped, nbytes = O.prefetch(cent, off, odt, q_out[0], L, 1 << 40, res, om)
    assert ps.n_taken == len(chosen) and ps.bytes == nbytes and ps.n_skipped == skipped
    assert list(index.ivf_resident()) == list(res.clusters())
    ms = index.ivf_prefetch_wait()
    assert ms >= 0.0
    gi, gd = index.ivf_search(q_out[0], L, k)
    check_topk(gi[0], gd[0], st, odt, off, None, cent, q_out[0], L, k, om)
    index.close()


def test_built_host_index_with_ids_and_batches(streams):
    """ivf_build_layout with host placement, caller ids, a buffer smaller than one cluster
    (nothing can be prefetched: the whole search runs on the host) and a batch of queries."""
    rng = np.random.default_rng(12)
    n, d, nlist = 8000, 96, 10
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    assign = rng.integers(0, nlist, n).astype(np.int32)
    rows = (cent[assign] + 0.6 * rng.standard_normal((n, d))).astype(np.float32)
    ids = rng.permutation(n).astype(np.int64) + 5
    off, perm = O.build_layout(assign, nlist)
    q = rng.standard_normal((4, d)).astype(np.float32)
    for cap in (64, n * d * 4):
        index = P.ivf_build_layout(rows, "f32", cent, assign, ids=ids, placement=P.IVF_PLACE_HOST,
                                   device_buffer_bytes=cap, compute_stream=streams[0], copy_stream=streams[1])
        ps = index.ivf_prefetch(q, 5, 1 << 40, flags=P.IVF_PREFETCH_RESET)
        if cap == 64:
            assert ps.n_taken == 0 and len(index.ivf_resident()) == 0
        gi, gd, ss = index.ivf_search(q, 5, 10, with_stats=True)
        if cap == 64:
            assert ss.n_overlap == 0 and ss.hit_rate == 0.0
        else:
            assert ss.n_miss == 0 and ss.hit_rate == 1.0       # q_out == q_in, unbounded budget
        for b in range(4):
            assert check_topk(gi[b], gd[b], rows[perm], O.F32, off, ids[perm], cent, q[b], 5, 10, O.IP) == 0
        index.close()


def test_batched_prefetch_splits_the_budget(streams):
    """Sec. 4.2 'Batching design': one total budget, an equal share per query of the batch; a
    cluster an earlier query of the batch already brought in is not copied (or charged) again.
    Followed by a second round without reset (Sec. 4.3 'Prefetching for multi-round') and a
    batched hybrid search."""
    n, d, nlist, L, k, B = 30000, 256, 48, 12, 10, 4
    ds, q_in, q_out = _problem(61, n, d, nlist, "f16")
    off, cent = ds.offsets.numpy(), ds.centroids.numpy()
    st, odt = stored(ds.rows.float().numpy(), "f16")
    sizes = np.diff(off) * d * 2
    cap = int(n * d * 2 // 2)
    index = P.ivf_adopt_layout(ds.rows.pin_memory(), "f16", off, cent, metric=P.IVF_IP, placement=P.IVF_PLACE_HOST,
                               device_buffer_bytes=cap, compute_stream=streams[0], copy_stream=streams[1])
    for total in (int(sizes.sum() // 6), int(sizes.sum() // 3), 1 << 40):
        res = O.Residency(nlist, cap)
        taken, skipped, nbytes = 0, 0, 0
        for b in range(B):
            c, s, nb = O.prefetch(cent, off, odt, q_in[b], L, total // B, res, O.IP)
            taken += len(c); skipped += s; nbytes += nb
        ps = index.ivf_prefetch(q_in[:B], L, total, flags=P.IVF_PREFETCH_RESET)
        assert (ps.n_taken, ps.n_skipped, ps.bytes) == (taken, skipped, nbytes)
        assert list(index.ivf_resident()) == list(res.clusters())
        # second round, same batch after the rewrite: only clusters not yet resident are fetched
        taken2, nbytes2 = 0, 0
        for b in range(B):
            c, s, nb = O.prefetch(cent, off, odt, q_out[b], L, total // B, res, O.IP)
            taken2 += len(c); nbytes2 += nb
        ps2 = index.ivf_prefetch(q_out[:B], L, total)
        assert (ps2.n_taken, ps2.bytes) == (taken2, nbytes2)
        assert list(index.ivf_resident()) == list(res.clusters())
        gi, gd, ss = index.ivf_search(q_out[:B], L, k, with_stats=True)
        hit = 0.0
        for b in range(B):
            ov, ms = O.split(cent, q_out[b], L, res.flags, O.IP)
            hit += len(ov) / float(len(ov) + len(ms))
            assert check_topk(gi[b], gd[b], st, odt, off, None, cent, q_out[b], L, k, O.IP) == 0
        assert abs(ss.hit_rate - hit / B) < 1e-6
    index.close()


@pytest.mark.parametrize("fraction,decay,h_inc", [(0.5, 2.0, 1.0), (0.25, 3.0, 0.25)])
def test_cluster_cache_rounds(streams, fraction, decay, h_inc):
    """Sec. 4.2 'Cache design' and the appendix's hotness transition: prefetch (admission at
    h_init), search (use marks), end of round (decay, eviction down to the cache fraction,
    consolidation of the buffer) over several rounds, against the oracle's cache round.  Hotness
    is compared bit for bit, residency exactly, and every search after a consolidation must still
    return the oracle's neighbours, so the moved lists are intact."""
    n, d, nlist, L, k = 30000, 128, 40, 10, 10
    ds, q_in, q_out = _problem(71, n, d, nlist, "f16")
    rng = np.random.default_rng(3)
    off, cent = ds.offsets.numpy(), ds.centroids.numpy()
    st, odt = stored(ds.rows.float().numpy(), "f16")
    sizes = np.diff(off) * d * 2
    cap = int(sizes.sum() * 0.6)
    h_init = 1.0
    index = P.ivf_adopt_layout(ds.rows.pin_memory(), "f16", off, cent, metric=P.IVF_IP, placement=P.IVF_PLACE_HOST,
                               device_buffer_bytes=cap, compute_stream=streams[0], copy_stream=streams[1])
    index.ivf_cache_configure(fraction, h_init, decay, h_inc)
    res = O.Residency(nlist, cap)
    hot = np.full(nlist, -1.0, dtype=np.float32)
    used = np.zeros(nlist, dtype=np.uint8)
    moved_any, evicted_any = False, False
    for rnd in range(8):
        b = rnd % q_in.shape[0]
        # a different neighbourhood every other round, so that old clusters cool down
        qi = q_in[b] if rnd % 2 == 0 else (cent[rng.integers(0, nlist)] + 0.1 * rng.standard_normal(d)).astype(np.float32)
        qo = q_out[b] if rnd % 2 == 0 else qi
        budget = int(sizes.sum() // 4)
        chosen, skipped, nbytes = O.prefetch(cent, off, odt, qi, L, budget, res, O.IP)
        O.cache_admit(hot, res, h_init)
        ps = index.ivf_prefetch(qi, L, budget)
        assert (ps.n_taken, ps.n_skipped, ps.bytes) == (len(chosen), skipped, nbytes)
        gi, gd, ss = index.ivf_search(qo, L, k, with_stats=True)
        ov, ms = O.split(cent, qo, L, res.flags, O.IP)
        used[ov] = 1
        assert ss.n_overlap == len(ov) and ss.n_miss == len(ms)
        assert check_topk(gi[0], gd[0], st, odt, off, None, cent, qo, L, k, O.IP) == 0
        np.testing.assert_array_equal(index.ivf_cache_hotness(), hot)
        before = res.used.value
        ev = O.cache_round(hot, used, res, off, d, odt, decay, h_inc, fraction)
        cs = index.ivf_cache_end_round()
        assert cs.n_evicted == len(ev) and cs.bytes_cached == before and cs.bytes_kept == res.used.value
        assert cs.bytes_kept <= int(fraction * cap)
        np.testing.assert_array_equal(index.ivf_cache_hotness(), hot)
        assert list(index.ivf_resident()) == list(res.clusters())
        moved_any |= cs.bytes_moved > 0
        evicted_any |= cs.n_evicted > 0
        # the consolidated buffer still holds the right rows
        gi, gd, ss = index.ivf_search(qo, L, k, with_stats=True)
        ov2, _ = O.split(cent, qo, L, res.flags, O.IP)
        used[ov2] = 1
        assert ss.n_overlap == len(ov2)
        assert check_topk(gi[0], gd[0], st, odt, off, None, cent, qo, L, k, O.IP) == 0
    assert moved_any and evicted_any
    # a reset prefetch drops the cache
    index.ivf_prefetch(q_in[0], L, 0, flags=P.IVF_PREFETCH_RESET)
    assert (index.ivf_cache_hotness() < 0).all() and len(index.ivf_resident()) == 0
    index.close()


@pytest.mark.parametrize("dtype,d", [("f32", 768), ("f16", 100), ("bf16", 64), ("f32", 7)])
def test_identical_rows_split_between_host_and_gpu(streams, dtype, d):
    """The fp64 re-score has one order of operations on the device and on the host, so copies of a
    row score bit for bit the same whether their cluster was prefetched or not, and come out by id
    exactly as in the oracle: no near-tie exemption is needed."""
    rng = np.random.default_rng(17)
    n, nlist, L, k = 6000, 12, 8, 40
    base = rng.standard_normal((25, d)).astype(np.float32)          # every row is one of 25 vectors
    rows = base[rng.integers(0, 25, n)]
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    assign = rng.integers(0, nlist, n).astype(np.int32)
    ids = rng.permutation(n).astype(np.int64) * 5 + 2
    st, odt = stored(rows, dtype)
    off, perm = O.build_layout(assign, nlist)
    esz = 4 if dtype == "f32" else 2
    index = P.ivf_build_layout(st, dtype, cent, assign, ids=ids, placement=P.IVF_PLACE_HOST,
                               device_buffer_bytes=n * d * esz, compute_stream=streams[0], copy_stream=streams[1])
    q = rng.standard_normal((3, d)).astype(np.float32)
    for frac in (0.0, 0.35, 0.7, 2.0):
        index.ivf_prefetch(q, L, int(frac * n * d * esz), flags=P.IVF_PREFETCH_RESET)
        gi, gd, ss = index.ivf_search(q, L, k, with_stats=True)
        if 0.0 < frac < 1.0:
            assert ss.n_overlap > 0 and ss.n_miss > 0
        for b in range(3):
            oi, _ = O.search(st[perm], odt, off, ids[perm], cent, q[b], L, k, O.IP)
            assert list(gi[b]) == list(oi)
    index.close()


@pytest.mark.parametrize("dtype,d", [("f16", 128), ("f32", 96), ("bf16", 320)])
def test_hybrid_search_finds_every_row_by_its_own_query(streams, dtype, d):
    """Coverage of the hybrid search: with every list selected and about half of the lists
    resident, each stored row is the nearest neighbour of its own values (normalised, distinct
    rows) whether its list is scanned on the GPU or by the host threads.  All rows are asked, 64
    per call."""
    nlist = 14
    sizes = W.zipf_sizes(5000, nlist, 1.1, 21)
    sizes[4] += sizes[9]; sizes[9] = 0
    ds = W.cluster_major_datastore(sizes, d, 0.3, 22, dtype=dtype)
    off, cent = ds.offsets.numpy(), ds.centroids.numpy()
    wide = ds.rows.to(torch.float64).numpy()
    n = ds.n
    for lo in range(0, n, 1000):                      # the case is what it claims
        assert np.array_equal(np.argmax(wide[lo:lo + 1000] @ wide.T, axis=1), np.arange(lo, min(lo + 1000, n)))
    esz = 4 if dtype == "f32" else 2
    index = P.ivf_adopt_layout(ds.rows.pin_memory(), dtype, off, cent, metric=P.IVF_IP, placement=P.IVF_PLACE_HOST,
                               device_buffer_bytes=n * d * esz, compute_stream=streams[0], copy_stream=streams[1])
    q = wide.astype(np.float32)
    index.ivf_prefetch(q[0], nlist, n * d * esz // 2, flags=P.IVF_PREFETCH_RESET)      # whole lists up to half of the bytes
    res = set(index.ivf_resident())
    assert 0 < len(res) < nlist
    on_gpu = np.zeros(n, dtype=bool)
    for c in res:
        on_gpu[off[c]:off[c + 1]] = True
    assert on_gpu.any() and (~on_gpu).any()
    for lo in range(0, n, 64):
        gi, gd = index.ivf_search(q[lo:lo + 64], nlist, 1)
        want = np.arange(lo, min(lo + 64, n))
        assert np.array_equal(gi[:, 0], want), f"rows {want[gi[:, 0] != want][:8]} (on the GPU: {on_gpu[want[gi[:, 0] != want][:8]]})"
    index.close()
