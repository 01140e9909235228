"""Parity of kernel variants the shape sweep does not reach: the matrix-core coarse kernels, the
select kernel's exact redo when packed score prefixes tie, and the three ways id ranks arise."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2502_20969_amd as P
from parity import check_topk

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def streams():
    assert torch.cuda.is_available()
    return torch.cuda.Stream(), torch.cuda.Stream()


def _index(streams, cent, d, metric, seed=0):
    """A small index over `cent`: two rows per cluster."""
    rng = np.random.default_rng(seed)
    nlist = cent.shape[0]
    n = 2 * nlist
    assign = (np.arange(n) % nlist).astype(np.int32)
    rows = rng.standard_normal((n, d)).astype(np.float32)
    return P.ivf_build_layout(rows, "f32", cent, assign, metric=metric,
                              compute_stream=streams[0], copy_stream=streams[1])


@pytest.mark.parametrize("nq", [16, 47, 48, 130])
@pytest.mark.parametrize("metric", ["ip", "l2"])
@pytest.mark.parametrize("nlist,d", [(130, 36), (1000, 100), (257, 768)])
def test_coarse_scores_of_a_batch(streams, nq, metric, nlist, d):
    """16 or more queries go through the fp64 matrix-core kernels (two tile layouts); tiles are
    ragged in queries, centroids and the k dimension."""
    pm, om = (P.IVF_IP, O.IP) if metric == "ip" else (P.IVF_L2, O.L2)
    rng = np.random.default_rng(1000 * nq + nlist + d)
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    index = _index(streams, cent, d, pm)
    cs = index.ivf_coarse_scores(q)
    pr = index.ivf_probe(q, 20)
    for b in range(nq):
        oc, osc = O.probe(cent, q[b], nlist, om, with_scores=True)
        np.testing.assert_allclose(cs[b][oc], osc, rtol=1e-12, atol=1e-10)
        assert list(pr[b]) == list(oc[:20]), f"query {b}: selected clusters differ"
    index.close()


@pytest.mark.parametrize("nprobe", [1, 10, 63, 64])
def test_select_redoes_prefix_ties_exactly(streams, nprobe):
    """Centroids that differ from one another by a few ulps of one small component have fp64 scores
    that agree in far more than their leading 28 mantissa bits: the packed fast path cannot order
    them and the exact path must take over, also when the tie straddles the cut at 64."""
    rng = np.random.default_rng(5)
    d, near, far = 16, 150, 100
    base = rng.standard_normal(d).astype(np.float32)
    base[0] = np.float32(1e-3)
    cent = np.empty((near + far, d), dtype=np.float32)
    step = np.float32(base[0])
    for j in range(near):
        cent[j] = base
        cent[j, 0] = step
        step = np.nextafter(step, np.float32(1.0), dtype=np.float32)
    cent[near:] = 0.1 * rng.standard_normal((far, d)).astype(np.float32)
    order = rng.permutation(near + far)
    cent = np.ascontiguousarray(cent[order])
    index = _index(streams, cent, d, P.IVF_IP)
    q = np.stack([base + 0.01 * rng.standard_normal(d).astype(np.float32) for _ in range(4)]).astype(np.float32)
    q[:, 0] = np.abs(q[:, 0]) + 0.5          # the varied component counts, with a fixed sign
    pr = index.ivf_probe(q, nprobe)
    for b in range(4):
        oc, osc = O.probe(cent, q[b], nprobe, O.IP, with_scores=True)
        assert list(pr[b]) == list(oc)
        # the case is what it claims: neighbours in the oracle order agree to better than 2^-28
        full = O.probe(cent, q[b], near + far, O.IP, with_scores=True)[1]
        assert abs(full[1] - full[0]) < abs(full[0]) * 2.0 ** -30
    index.close()


@pytest.mark.parametrize("nlist", [1024, 4096])
@pytest.mark.parametrize("nprobe,layout", [(20, "spread"), (20, "few_groups"), (32, "few_groups"), (64, "spread"),
                                            (64, "few_groups"), (64, "most_in_63_groups"), (33, "most_in_63_groups")])
def test_select_cut_by_group_maxima_on_adversarial_layouts(streams, nlist, nprobe, layout):
    """The selection deals the scores to 64 or 128 groups by cluster index (index mod 64 / mod 128)
    and cuts at the nprobe-th largest group maximum; how many scores pass depends on how the large
    ones fall into the groups.  Large scores spread evenly: a few more than nprobe pass (one sort,
    or two sorts and a merge).  All large scores in 8 groups: hundreds pass (ranked by counting).
    Large scores in 63 groups and none elsewhere: the cut falls among the small ones and more pass
    than the pool holds (the exact general path takes over).  The result must be the oracle's
    every time."""
    rng = np.random.default_rng(77)
    d = 8
    small = 0.1 + 0.3 * rng.random(nlist)
    large = 1.0 + rng.permutation(nlist) * 1e-4           # distinct, far apart in the 40-bit prefixes
    idx = np.arange(nlist)
    if layout == "spread":
        is_large = rng.random(nlist) < 0.08
    elif layout == "few_groups":
        is_large = (idx % 128) < 8
    else:
        is_large = ((idx % 128) < 63) & (rng.random(nlist) < 0.75)
    score = np.where(is_large, large, small)
    cent = np.zeros((nlist, d), dtype=np.float32)
    cent[:, 0] = score.astype(np.float32)
    cent[:, 1:] = 0.01 * rng.standard_normal((nlist, d - 1)).astype(np.float32)
    index = _index(streams, cent, d, P.IVF_IP)
    q = np.zeros((3, d), dtype=np.float32)
    q[:, 0] = [1.0, 0.7, 2.5]
    q[:, 1:] = 0.01 * rng.standard_normal((3, d - 1)).astype(np.float32)
    pr = index.ivf_probe(q, nprobe)
    for b in range(3):
        assert list(pr[b]) == list(O.probe(cent, q[b], nprobe, O.IP))
    # and a whole search over the same index
    gi, gd = index.ivf_search(q, nprobe, 5)
    n = 2 * nlist
    rows_assign = (np.arange(n) % nlist).astype(np.int32)
    off, perm = O.build_layout(rows_assign, nlist)
    rows = np.random.default_rng(0).standard_normal((n, d)).astype(np.float32)
    for b in range(3):
        oi, osc = O.search(rows[perm], O.F32, off, perm.astype(np.int64), cent, q[b], nprobe, 5, O.IP)
        assert list(gi[b]) == list(oi)
    index.close()


@pytest.mark.parametrize("kind", ["increasing", "permutation", "sparse"])
def test_id_rank_tables(streams, kind):
    """Adopted layouts whose ids grow with the row (no rank table), are a permutation of the row
    numbers (the permutation is the table) or are arbitrary distinct values (sorted).  Half of the
    rows are exact duplicates, so equal scores must come out by smaller id."""
    rng = np.random.default_rng(9)
    n, d, nlist = 6000, 64, 12
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    assign = np.sort(rng.integers(0, nlist, n)).astype(np.int32)          # already cluster-major
    rows = (cent[assign] + 0.5 * rng.standard_normal((n, d))).astype(np.float32)
    src, dst = rng.integers(0, n, n // 2), rng.integers(0, n, n // 2)
    rows[dst] = rows[src]
    off = np.zeros(nlist + 1, dtype=np.int64)
    off[1:] = np.cumsum(np.bincount(assign, minlength=nlist))
    if kind == "increasing":
        ids = np.cumsum(rng.integers(1, 5, n)).astype(np.int64)
    elif kind == "permutation":
        ids = rng.permutation(n).astype(np.int64)
    else:
        ids = (rng.permutation(n).astype(np.int64) * 1_000_003 + 17) % (1 << 40)
        assert len(np.unique(ids)) == n
    lists_dev = torch.from_numpy(rows).cuda()
    index = P.ivf_adopt_layout(lists_dev, "f32", off, cent, ids=ids, metric=P.IVF_IP,
                               compute_stream=streams[0], copy_stream=streams[1])
    q = (cent[rng.integers(0, nlist, 6)] + 0.3 * rng.standard_normal((6, d))).astype(np.float32)
    gi, gd = index.ivf_search(q, 5, 30)
    for b in range(6):
        assert check_topk(gi[b], gd[b], rows, O.F32, off, ids, cent, q[b], 5, 30, O.IP) == 0
    index.close()


@pytest.mark.parametrize("B,d,micro", [(1, 8, 4), (7, 5, 3), (64, 33, 8), (256, 768, 32), (300, 100, 7),
                                       (1500, 16, 64), (130, 64, 1), (90, 12, 500)])
def test_prefetching_scheduler(streams, B, d, micro):
    """Greedy grouping of a global batch into micro-batches (Sec. 4.2 'Scheduling optimization for
    prefetching') against the oracle: the distances are added in the oracle's order, so the
    orders agree exactly, ties included (a quarter of the queries are exact duplicates)."""
    rng = np.random.default_rng(B * 31 + d)
    centres = rng.standard_normal((max(1, B // 6), d)).astype(np.float32)
    q = (centres[rng.integers(0, centres.shape[0], B)] + 0.3 * rng.standard_normal((B, d))).astype(np.float32)
    dup = rng.integers(0, B, B // 4)
    q[rng.integers(0, B, B // 4)] = q[dup]
    cent = rng.standard_normal((4, d)).astype(np.float32)
    index = _index(streams, cent, d, P.IVF_IP)
    order, ms = index.ivf_schedule(q, micro, with_time=True)
    assert list(order) == list(O.schedule(q, micro))
    assert ms >= 0.0
    index.close()


def test_scheduler_rejects_bad_arguments(streams):
    cent = np.zeros((4, 8), dtype=np.float32)
    index = _index(streams, cent, 8, P.IVF_IP)
    q = np.zeros((5000, 8), dtype=np.float32)
    with pytest.raises(P.binding.IvfError) as e:
        index.ivf_schedule(q, 8)
    assert e.value.status == -5
    with pytest.raises(P.binding.IvfError) as e:
        index.ivf_schedule(q[:10], 0)
    assert e.value.status == -1
    index.close()


def test_back_to_back_host_searches_return_their_own_results(streams):
    """A single-query ivf_search returns when the last kernel has published its results in pinned
    memory, while the stream may still be finishing: 400 calls in a row, alternating queries with
    different answers, must each return the answer of their own query (a stale or early read of the
    result buffer would return the previous one)."""
    rng = np.random.default_rng(77)
    n, d, nlist = 20000, 96, 40
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    assign = rng.integers(0, nlist, n).astype(np.int32)
    rows = (cent[assign] + 0.4 * rng.standard_normal((n, d))).astype(np.float32)
    index = P.ivf_build_layout(rows, "f32", cent, assign, metric=P.IVF_IP,
                               compute_stream=streams[0], copy_stream=streams[1])
    q = (cent[rng.integers(0, nlist, 8)] + 0.3 * rng.standard_normal((8, d))).astype(np.float32)
    off, perm = O.build_layout(assign, nlist)
    first = [index.ivf_search(q[b], 10, 7) for b in range(8)]
    assert len({tuple(f[0][0]) for f in first}) > 1           # the queries do differ in their answers
    for it in range(400):
        b = (it * 5) % 8
        gi, gd = index.ivf_search(q[b], 10, 7)
        assert np.array_equal(gi, first[b][0]) and np.array_equal(gd, first[b][1]), f"call {it}"
    for b in range(8):
        assert check_topk(first[b][0][0], first[b][1][0], rows[perm], O.F32, off, perm.astype(np.int64), cent, q[b],
                          10, 7, O.IP) == 0
    index.close()


@pytest.mark.parametrize("metric", ["ip", "l2"])
@pytest.mark.parametrize("nlist,d", [(1024, 64), (1039, 37), (4097, 100), (5000, 768), (20000, 32)])
def test_single_query_probe_of_large_indexes(streams, metric, nlist, d):
    """One query against 1024 or more centroids, several calls in a row: every selection path
    (register sort up to 64, the general sort, the selection pass before it, global sort memory
    for the full order), ragged last workgroups, rows that are not a multiple of 16 bytes, and
    centroids that tie exactly."""
    pm, om = (P.IVF_IP, O.IP) if metric == "ip" else (P.IVF_L2, O.L2)
    rng = np.random.default_rng(nlist + d)
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    cent[rng.integers(0, nlist, nlist // 8)] = cent[rng.integers(0, nlist, nlist // 8)]    # exact ties
    index = _index(streams, cent, d, pm)
    q = rng.standard_normal((6, d)).astype(np.float32)
    for nprobe in (1, 32, 64, 65, 200, nlist):
        for b in range(6):
            pr = index.ivf_probe(q[b], nprobe)
            assert list(pr[0]) == list(O.probe(cent, q[b], nprobe, om)), f"nprobe {nprobe}, query {b}"
    pr = index.ivf_probe(q[:3], 32)                  # three queries in one call: same answers
    for b in range(3):
        assert list(pr[b]) == list(O.probe(cent, q[b], 32, om))
    index.close()


def test_single_query_probe_redoes_prefix_ties(streams):
    """The prefix-tie case of the register sort with more than 1024 centroids, one query per call."""
    rng = np.random.default_rng(6)
    d, near, far = 16, 150, 1000
    base = rng.standard_normal(d).astype(np.float32)
    base[0] = np.float32(1e-3)
    cent = np.empty((near + far, d), dtype=np.float32)
    step = np.float32(base[0])
    for j in range(near):
        cent[j] = base
        cent[j, 0] = step
        step = np.nextafter(step, np.float32(1.0), dtype=np.float32)
    cent[near:] = 0.1 * rng.standard_normal((far, d)).astype(np.float32)
    cent = np.ascontiguousarray(cent[rng.permutation(near + far)])
    index = _index(streams, cent, d, P.IVF_IP)
    for nprobe in (1, 10, 63, 64):
        for b in range(4):
            q = (base + 0.01 * rng.standard_normal(d)).astype(np.float32)
            q[0] = abs(q[0]) + 0.5
            assert list(index.ivf_probe(q, nprobe)[0]) == list(O.probe(cent, q, nprobe, O.IP))
    index.close()
