"""Pins for the CPU oracle: every expected value here comes from the hand-worked
fixture, a closed form, a library routine (numpy matmul / argsort / dtype
conversion) or a set identity -- never from the oracle itself."""
import json
import os

import numpy as np
import pytest
import torch

import oracle as O

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "handworked_ivf.json")))


def _hand():
    cent = np.array(GOLD["centroids"], dtype=np.float32)
    rows, ids, off = [], [], [0]
    for c in range(4):
        L = GOLD["lists"][str(c)]
        rows += L["rows"]
        ids += L["ids"]
        off.append(len(rows))
    return cent, np.array(rows, dtype=np.float32), np.array(ids, dtype=np.int64), np.array(off, dtype=np.int64)


# ---- hand-worked example (App. B definitions) ---------------------------------

@pytest.mark.parametrize("metric,key", [(O.IP, "ip"), (O.L2, "l2")])
def test_handworked_scores_and_probe(metric, key):
    cent, rows, ids, off = _hand()
    x = np.array(GOLD["q_out"], dtype=np.float32)
    g = GOLD[key]
    got_c, got_s = O.probe(cent, x, 4, metric, with_scores=True)
    by_cluster = {int(c): s for c, s in zip(got_c, got_s)}
    for j, want in enumerate(g["coarse_scores_q_out"]):
        assert by_cluster[j] == want
    assert list(O.probe(cent, x, 2, metric)) == g["probe2_q_out"]
    for id_s, want in g["row_scores_q_out"].items():
        pos = int(np.nonzero(ids == int(id_s))[0][0])
        assert O.score(x, rows, O.F32, pos, metric) == want


def test_handworked_probe_order_all_four():
    cent, *_ = _hand()
    x = np.array(GOLD["q_out"], dtype=np.float32)
    assert list(O.probe(cent, x, 4, O.IP)) == GOLD["ip"]["probe4_q_out"]
    assert list(O.probe(cent, x, 99, O.IP)) == GOLD["ip"]["probe4_q_out"]  # clamped


@pytest.mark.parametrize("dtype", [O.F32, O.F16, O.BF16])
def test_handworked_search(dtype):
    cent, rows, ids, off = _hand()
    x = np.array(GOLD["q_out"], dtype=np.float32)
    if dtype == O.F16:
        stored = rows.astype(np.float16)
    elif dtype == O.BF16:
        stored = torch.from_numpy(rows).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    else:
        stored = rows
    for nprobe, name in [(2, "top3_nprobe2"), (4, "top3_nprobe4")]:
        i, s = O.search(stored, dtype, off, ids, cent, x, nprobe, 3, O.IP)
        assert list(i) == GOLD["ip"][name]["ids"]
        assert list(s) == GOLD["ip"][name]["scores"]
    i, s = O.search(stored, dtype, off, ids, cent, x, 2, 3, O.L2)
    assert list(i) == GOLD["l2"]["top3_nprobe2"]["ids"]        # exact tie id0/id3 -> lower id first
    assert list(s) == GOLD["l2"]["top3_nprobe2"]["scores"]


def test_handworked_lookahead():
    cent, rows, ids, off = _hand()
    g = GOLD["lookahead_ip_fp32"]
    q_in = np.array(GOLD["q_in"], dtype=np.float32)
    q_out = np.array(GOLD["q_out"], dtype=np.float32)
    assert [int((off[c + 1] - off[c]) * 2 * 4) for c in range(4)] == g["list_bytes"]
    assert list(O.probe(cent, q_in, 2, O.IP)) == GOLD["ip"]["probe2_q_in"]
    want_top = GOLD["ip"]["top3_nprobe2"]

    res = O.Residency(4, cap=1 << 30)
    chosen, skipped, nbytes = O.prefetch(cent, off, O.F32, q_in, 2, 1 << 40, res, O.IP)
    assert sorted(chosen) == g["budget_inf"]["resident"] and skipped == 0 and nbytes == 32
    ov, ms = O.split(cent, q_out, 2, res.flags, O.IP)
    assert list(ov) == g["budget_inf"]["overlap"] and list(ms) == g["budget_inf"]["miss"]
    i, s, hr = O.hybrid(rows, O.F32, off, ids, cent, q_out, 2, 3, res.flags, O.IP)
    assert list(i) == want_top["ids"] and list(s) == want_top["scores"] and hr == 0.5

    res = O.Residency(4, cap=1 << 30)
    chosen, skipped, nbytes = O.prefetch(cent, off, O.F32, q_in, 2, 20, res, O.IP)
    assert list(chosen) == g["budget_20"]["resident"]
    assert skipped == g["budget_20"]["skipped"] and nbytes == g["budget_20"]["bytes"]

    res = O.Residency(4, cap=1 << 30)
    chosen, skipped, nbytes = O.prefetch(cent, off, O.F32, q_in, 2, 0, res, O.IP)
    assert list(chosen) == [] and nbytes == 0
    ov, ms = O.split(cent, q_out, 2, res.flags, O.IP)
    assert list(ov) == [] and list(ms) == g["budget_0"]["miss"]
    i, s, hr = O.hybrid(rows, O.F32, off, ids, cent, q_out, 2, 3, res.flags, O.IP)
    assert list(i) == want_top["ids"] and list(s) == want_top["scores"] and hr == 0.0


def test_budget_skip_then_continue():
    """Sec. 4.3 'Prefetching target': an over-budget cluster is skipped whole and a later,
    smaller one is still taken.  Sizes chosen by hand: lists of 3, 1, 2 rows (d=1, fp32:
    12, 4, 8 bytes), q_in ranks them 0,1,2; budget 13 takes 0 (12 B), skips 1 (4 > 1) and 2."""
    cent = np.array([[3.0], [2.0], [1.0]], dtype=np.float32)
    off = np.array([0, 3, 4, 6], dtype=np.int64)
    x = np.array([1.0], dtype=np.float32)
    res = O.Residency(3, cap=1 << 20)
    chosen, skipped, nbytes = O.prefetch(cent, off, O.F32, x, 3, 13, res, O.IP)
    assert list(chosen) == [0] and skipped == 2 and nbytes == 12
    # budget 11: cluster 0 (12 B) does not fit, 1 (4 B) and then 2 (8 B > 7) ...
    res = O.Residency(3, cap=1 << 20)
    chosen, skipped, nbytes = O.prefetch(cent, off, O.F32, x, 3, 11, res, O.IP)
    assert list(chosen) == [1] and skipped == 2 and nbytes == 4
    # budget 12 with a device buffer cap of 8 bytes: 0 blocked by the cap, 1 fits, 2 blocked
    res = O.Residency(3, cap=8)
    chosen, skipped, nbytes = O.prefetch(cent, off, O.F32, x, 3, 12, res, O.IP)
    assert list(chosen) == [1] and skipped == 2 and res.used.value == 4
    # never looks beyond the first L ranked clusters
    res = O.Residency(3, cap=1 << 20)
    chosen, _, _ = O.prefetch(cent, off, O.F32, x, 1, 11, res, O.IP)
    assert list(chosen) == []
    # incremental call: a resident cluster costs nothing and is not taken again
    res = O.Residency(3, cap=1 << 20)
    O.prefetch(cent, off, O.F32, x, 1, 100, res, O.IP)
    chosen, skipped, nbytes = O.prefetch(cent, off, O.F32, x, 3, 12, res, O.IP)
    assert list(chosen) == [1, 2] and skipped == 0 and nbytes == 12 and res.used.value == 24


# ---- widening of fp16 / bf16 against library conversions ------------------------

def test_widen_all_f16_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([O.widen(int(b), O.F16) for b in bits])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def test_widen_all_bf16_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).double().numpy()
    got = np.array([O.widen(int(b), O.BF16) for b in bits])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])


# ---- closed forms ---------------------------------------------------------------

def test_score_closed_forms():
    d = 7
    rows = np.zeros((3, d), dtype=np.float32)
    rows[0, 2] = 4.0
    rows[1, 5] = -2.0
    rows[2, :] = np.arange(1, d + 1)
    x = np.zeros(d, dtype=np.float32)
    x[2] = 0.5
    x[5] = 3.0
    assert O.score(x, rows, O.F32, 0, O.IP) == 2.0
    assert O.score(x, rows, O.F32, 1, O.IP) == -6.0
    assert O.score(x, rows, O.F32, 2, O.IP) == 0.5 * 3 + 3.0 * 6
    assert O.score(x, rows, O.F32, 0, O.L2) == 3.5 ** 2 + 9.0
    assert O.score(x, rows, O.F32, 1, O.L2) == 0.25 + 25.0
    # ||x-y||^2 = ||x||^2 + ||y||^2 - 2<x,y>, all integers here so exact
    xi = np.arange(d, dtype=np.float32) - 3
    want = float((xi.astype(np.int64) ** 2).sum() + (np.arange(1, d + 1) ** 2).sum()
                 - 2 * (xi.astype(np.int64) * np.arange(1, d + 1)).sum())
    assert O.score(xi, rows, O.F32, 2, O.L2) == want


# ---- brute force through numpy --------------------------------------------------

def _random_index(rng, n, d, nlist, dtype=O.F32, empty=()):
    rows = rng.standard_normal((n, d)).astype(np.float32)
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    allowed = np.array([c for c in range(nlist) if c not in empty])
    assign = allowed[rng.integers(0, len(allowed), n)].astype(np.int32)
    order = np.argsort(assign, kind="stable")
    off = np.zeros(nlist + 1, dtype=np.int64)
    np.add.at(off, assign + 1, 1)
    off = np.cumsum(off)
    lists = rows[order]
    ids = order.astype(np.int64)
    if dtype == O.F16:
        stored = lists.astype(np.float16)
        wide = stored.astype(np.float64)
    elif dtype == O.BF16:
        t = torch.from_numpy(lists).to(torch.bfloat16)
        stored = t.view(torch.int16).numpy().view(np.uint16)
        wide = t.double().numpy()
    else:
        stored, wide = lists, lists.astype(np.float64)
    return cent, stored, wide, ids, off, assign


def _brute(wide, ids, x, k, metric, mask=None):
    x64 = x.astype(np.float64)
    if metric == O.IP:
        s = wide @ x64
        key = -s
    else:
        s = ((wide - x64[None, :]) ** 2).sum(1)
        key = s
    cand = np.arange(len(ids)) if mask is None else np.nonzero(mask)[0]
    order = cand[np.lexsort((ids[cand], key[cand]))][:k]
    return ids[order], s[order]


@pytest.mark.parametrize("metric", [O.IP, O.L2])
@pytest.mark.parametrize("dtype", [O.F32, O.F16, O.BF16])
def test_exhaustive_equals_brute_force(metric, dtype):
    rng = np.random.default_rng(7 + metric + 10 * dtype)
    cent, stored, wide, ids, off, _ = _random_index(rng, 600, 19, 9, dtype)
    for _ in range(5):
        x = rng.standard_normal(19).astype(np.float32)
        wi, ws = _brute(wide, ids, x, 12, metric)
        gi, gs = O.search(stored, dtype, off, ids, cent, x, 9, 12, metric)
        assert list(gi) == list(wi)
        np.testing.assert_allclose(gs, ws, rtol=1e-12, atol=1e-13)
        gi2, _ = O.search(stored, dtype, off, ids, cent, x, 1000, 12, metric)  # clamp
        assert list(gi2) == list(wi)


@pytest.mark.parametrize("metric", [O.IP, O.L2])
def test_ivf_equals_brute_force_over_probed_lists(metric):
    """nprobe < nlist: brute force restricted to the rows whose cluster is among the
    numpy-ranked nearest centroids."""
    rng = np.random.default_rng(11 + metric)
    cent, stored, wide, ids, off, assign = _random_index(rng, 800, 24, 16, empty=(3, 7))
    cl_of_pos = np.repeat(np.arange(16), np.diff(off))
    for _ in range(5):
        x = rng.standard_normal(24).astype(np.float32)
        c64 = cent.astype(np.float64)
        cs = c64 @ x.astype(np.float64) if metric == O.IP else ((c64 - x[None, :].astype(np.float64)) ** 2).sum(1)
        ranked = np.lexsort((np.arange(16), -cs if metric == O.IP else cs))
        for L in (1, 4, 16):
            assert list(O.probe(cent, x, L, metric)) == list(ranked[:L])
            mask = np.isin(cl_of_pos, ranked[:L])
            wi, ws = _brute(wide, ids, x, 10, metric, mask)
            gi, gs = O.search(stored, O.F32, off, ids, cent, x, L, 10, metric)
            assert list(gi[:len(wi)]) == list(wi)
            np.testing.assert_allclose(gs[:len(wi)], ws, rtol=1e-12, atol=1e-13)
            assert all(i == -1 for i in gi[len(wi):])


def test_single_list_is_plain_knn_and_padding():
    rng = np.random.default_rng(3)
    cent, stored, wide, ids, off, _ = _random_index(rng, 5, 8, 1)
    x = rng.standard_normal(8).astype(np.float32)
    wi, ws = _brute(wide, ids, x, 5, O.IP)
    gi, gs = O.search(stored, O.F32, off, ids, cent, x, 1, 8, O.IP)
    assert list(gi[:5]) == list(wi) and list(gi[5:]) == [-1, -1, -1]
    assert np.all(np.isneginf(gs[5:]))
    gi, gs = O.search(stored, O.F32, off, ids, cent, x, 1, 8, O.L2)
    assert np.all(np.isposinf(gs[5:]))
    # ids=None: the row position is the id
    gi, _ = O.search(stored, O.F32, off, None, cent, x, 1, 5, O.IP)
    assert list(ids[gi]) == list(wi)


def test_prefix_and_monotonicity():
    rng = np.random.default_rng(5)
    cent, stored, wide, ids, off, _ = _random_index(rng, 1000, 16, 12)
    x = rng.standard_normal(16).astype(np.float32)
    full = O.probe(cent, x, 12, O.IP)
    for L in range(1, 12):
        assert list(O.probe(cent, x, L, O.IP)) == list(full[:L])
    i20, s20 = O.search(stored, O.F32, off, ids, cent, x, 5, 20, O.IP)
    for k in (1, 3, 10):
        ik, sk = O.search(stored, O.F32, off, ids, cent, x, 5, k, O.IP)
        assert list(ik) == list(i20[:k]) and list(sk) == list(s20[:k])
    prev = None
    for L in range(1, 13):
        _, s = O.search(stored, O.F32, off, ids, cent, x, L, 10, O.IP)
        if prev is not None:
            assert np.all(s >= prev)      # i-th best never gets worse with more clusters
        prev = s


def test_exact_ties_resolved_by_lower_id():
    """Four copies of one vector spread over two lists with shuffled ids."""
    cent = np.array([[1, 0], [0, 1]], dtype=np.float32)
    rows = np.array([[1, 1], [1, 1], [0, 1], [1, 1], [1, 1]], dtype=np.float32)
    ids = np.array([9, 4, 1, 7, 2], dtype=np.int64)
    off = np.array([0, 2, 5], dtype=np.int64)
    x = np.array([1.0, 1.0], dtype=np.float32)
    i, s = O.search(rows, O.F32, off, ids, cent, x, 2, 3, O.IP)
    assert list(i) == [2, 4, 7] and list(s) == [2.0, 2.0, 2.0]
    # equal centroid scores -> lower cluster index first
    assert list(O.probe(cent, x, 2, O.IP)) == [0, 1]


# ---- lookahead identities -------------------------------------------------------

@pytest.mark.parametrize("metric", [O.IP, O.L2])
def test_split_and_hybrid_identities(metric):
    rng = np.random.default_rng(21 + metric)
    n, d, nlist, L, k = 1500, 12, 20, 6, 7
    cent, stored, wide, ids, off, _ = _random_index(rng, n, d, nlist, O.F16)
    sizes = np.diff(off) * d * 2
    for trial in range(8):
        q_in = rng.standard_normal(d).astype(np.float32)
        q_out = (q_in + 0.3 * rng.standard_normal(d)).astype(np.float32)
        for budget in (0, int(sizes.min()), int(sizes.sum() // 8), 1 << 40):
            res = O.Residency(nlist, cap=1 << 40)
            chosen, skipped, nbytes = O.prefetch(cent, off, O.F16, q_in, L, budget, res, metric)
            ranked_in = list(O.probe(cent, q_in, L, metric))
            assert set(chosen) <= set(ranked_in)
            assert nbytes == sizes[chosen].sum() <= budget
            assert len(chosen) + skipped == L
            # replay: each skipped cluster was larger than what was left when considered
            rem = budget
            for c in ranked_in:
                if c in chosen:
                    rem -= sizes[c]
                else:
                    assert sizes[c] > rem
            if budget == 1 << 40:
                assert list(chosen) == ranked_in
            ov, ms = O.split(cent, q_out, L, res.flags, metric)
            c_out = list(O.probe(cent, q_out, L, metric))
            assert sorted(list(ov) + list(ms)) == sorted(c_out)
            assert not (set(ov) & set(ms))
            assert set(ov) <= set(res.clusters()) and not (set(ms) & set(res.clusters()))
            hi, hs, hr = O.hybrid(stored, O.F16, off, ids, cent, q_out, L, k, res.flags, metric)
            pi, ps = O.search(stored, O.F16, off, ids, cent, q_out, L, k, metric)
            assert list(hi) == list(pi) and list(hs) == list(ps)
            assert hr == len(ov) / len(c_out)
        # q_out == q_in and an unbounded budget: every cluster is a hit (Table 1, Self-RAG row)
        res = O.Residency(nlist, cap=1 << 40)
        O.prefetch(cent, off, O.F16, q_in, L, 1 << 40, res, metric)
        _, _, hr = O.hybrid(stored, O.F16, off, ids, cent, q_in, L, k, res.flags, metric)
        assert hr == 1.0


# ---- layout ---------------------------------------------------------------------

def test_layout_bijection_monotone_stable_and_invariance():
    rng = np.random.default_rng(9)
    n, d, nlist = 700, 10, 13
    rows = rng.standard_normal((n, d)).astype(np.float32)
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    assign = rng.integers(0, nlist, n).astype(np.int32)
    assign[assign == 5] = 6                      # an empty list
    off, perm = O.build_layout(assign, nlist)
    assert off[0] == 0 and off[-1] == n and np.all(np.diff(off) >= 0)
    assert np.array_equal(np.diff(off), np.bincount(assign, minlength=nlist))
    assert sorted(perm) == list(range(n))
    for c in range(nlist):
        seg = perm[off[c]:off[c + 1]]
        assert np.all(assign[seg] == c) and np.all(np.diff(seg) > 0)   # stable
    with pytest.raises(ValueError):
        O.build_layout(np.array([0, nlist], dtype=np.int32), nlist)
    x = rng.standard_normal(d).astype(np.float32)
    base = O.search(rows[perm], O.F32, off, perm, cent, x, 4, 9, O.IP)
    # shuffle the input rows (ids travel with them) and relabel the clusters
    shuf = rng.permutation(n)
    relabel = rng.permutation(nlist)
    assign2 = relabel[assign[shuf]].astype(np.int32)
    off2, perm2 = O.build_layout(assign2, nlist)
    cent2 = np.empty_like(cent)
    cent2[relabel] = cent
    got = O.search(rows[shuf][perm2], O.F32, off2, shuf[perm2], cent2, x, 4, 9, O.IP)
    assert list(got[0]) == list(base[0]) and list(got[1]) == list(base[1])


def test_workload_generators_are_seeded():
    import workloads as W
    a, qi, qo = W.config2_single_query(seed=5, n=3000, d=32, nlist=16, nq=4)
    b, qi2, qo2 = W.config2_single_query(seed=5, n=3000, d=32, nlist=16, nq=4)
    assert torch.equal(a.rows, b.rows) and torch.equal(a.assign, b.assign) and torch.equal(qo, qo2)
    np.testing.assert_allclose(a.rows.norm(dim=1).numpy(), 1.0, rtol=1e-5)
    np.testing.assert_allclose(qo.norm(dim=1).numpy(), 1.0, rtol=1e-5)
    sizes = W.zipf_sizes(10000, 64, 1.1, seed=3)
    assert int(sizes.sum()) == 10000 and int(sizes.min()) >= 1
    ds = W.cluster_major_datastore(sizes, 16, 0.3, seed=4, dtype="f16")
    assert ds.rows.shape == (10000, 16) and ds.offsets[-1] == 10000
    c0 = ds.rows[ds.offsets[5]:ds.offsets[6]].float().mean(0)
    np.testing.assert_allclose(ds.centroids[5].numpy(), c0.numpy(), rtol=1e-4, atol=1e-6)


# ---- cluster cache with decaying hotness (Sec. 4.2 "Cache design"; appendix, hotness transition) ----
def _cache_state(row_counts, d, cap, resident):
    nlist = len(row_counts)
    off = np.zeros(nlist + 1, dtype=np.int64)
    off[1:] = np.cumsum(row_counts)
    res = O.Residency(nlist, cap)
    res.flags[list(resident)] = 1
    res.used.value = int(sum(row_counts[c] for c in resident) * d * 4)
    hot = np.full(nlist, -1.0, dtype=np.float32)
    return off, res, hot, np.zeros(nlist, dtype=np.uint8)


def test_handworked_cache_round():
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "handworked_cache.json")))
    off, res, hot, used = _cache_state(g["row_counts"], g["d"], g["cap_bytes"], g["resident"])
    O.cache_admit(hot, res, g["h_init"])
    assert [c for c in range(len(hot)) if hot[c] == g["h_init"]] == g["resident"]
    used[g["used"]] = 1
    ev = O.cache_round(hot, used, res, off, g["d"], O.F32, g["decay"], g["h_inc"], g["fraction"])
    assert list(ev) == g["evicted"] and res.used.value == g["bytes_after"]
    assert list(hot) == g["hot_after"] and not used.any()
    assert list(res.clusters()) == [c for c in g["resident"] if c not in g["evicted"]]


def test_hotness_closed_forms():
    """Never used: h_r = h_init / d^r.  Used every round: h_r = h_init / d^r + h_inc (1 - d^-r) / (1 - 1/d)
    (a geometric series); with d = 2, h_init = h_inc = 1 that is 2 - 2^-r, exact in single precision."""
    off, res, hot, used = _cache_state([4, 4], 4, 1 << 20, [0, 1])
    O.cache_admit(hot, res, 1.0)
    for r in range(1, 21):
        used[1] = 1
        assert len(O.cache_round(hot, used, res, off, 4, O.F32, 2.0, 1.0, 0.5)) == 0
        assert hot[0] == np.float32(2.0 ** -r) and hot[1] == np.float32(2.0 - 2.0 ** -r)
    off, res, hot, used = _cache_state([4, 4], 4, 1 << 20, [0, 1])
    O.cache_admit(hot, res, 0.7)
    dcy, inc = 3.0, 0.25
    for r in range(1, 15):
        used[1] = 1
        O.cache_round(hot, used, res, off, 4, O.F32, dcy, inc, 0.5)
        assert abs(hot[0] - 0.7 / dcy ** r) <= 1e-6 * 0.7 / dcy ** r + 1e-12
        want = 0.7 / dcy ** r + inc * (1.0 - dcy ** -r) / (1.0 - 1.0 / dcy)
        assert abs(hot[1] - want) <= 2e-6 * want


def test_cache_eviction_invariants():
    """Random states: the evicted clusters are exactly the coldest ones, as few as bring the cache
    under its share; nothing leaves a cache that is under it; absent clusters stay absent."""
    rng = np.random.default_rng(77)
    for trial in range(200):
        nlist = int(rng.integers(1, 40))
        counts = rng.integers(0, 50, nlist)
        d = 8
        resident = [c for c in range(nlist) if rng.random() < 0.6]
        cap = int(max(1, counts.sum()) * d * 4 * rng.uniform(0.5, 2.0))
        off, res, hot, used = _cache_state(counts, d, cap, resident)
        if res.used.value > cap:
            continue
        for c in resident:
            hot[c] = np.float32(rng.choice([0.25, 0.5, 1.0, 1.5, 3.0]))        # many ties
        used[rng.random(nlist) < 0.3] = 1
        used_before = used.copy()
        hot_before, bytes_before = hot.copy(), res.used.value
        fraction = float(rng.choice([0.0, 0.25, 0.5, 1.0]))
        ev = O.cache_round(hot, used, res, off, d, O.F32, 2.0, 1.0, fraction)
        limit = int(fraction * cap)
        sizes = counts * d * 4
        upd = {c: np.float32(np.float32(hot_before[c] / np.float32(2.0)) + (np.float32(1.0) if used_before[c] else np.float32(0.0)))
               for c in resident}
        assert not used.any()
        assert all(hot[c] == -1.0 for c in range(nlist) if c not in resident)
        kept = [c for c in resident if c not in set(ev)]
        assert sorted(kept) == list(res.clusters())
        assert all(hot[c] == upd[c] for c in kept) and all(hot[c] == -1.0 for c in ev)
        assert res.used.value == bytes_before - int(sizes[list(ev)].sum())
        if bytes_before <= limit:
            assert len(ev) == 0
        else:
            assert res.used.value <= limit or not kept
            # one eviction fewer would not have been enough
            assert res.used.value + int(sizes[ev[-1]]) > limit
            # every evicted cluster is at most as hot as every kept one; equal hotness: larger index left
            for e in ev:
                for c in kept:
                    assert upd[e] < upd[c] or (upd[e] == upd[c] and e > c)
            # and they left coldest first
            for a, b in zip(ev[:-1], ev[1:]):
                assert upd[a] < upd[b] or (upd[a] == upd[b] and a > b)


# ---- prefetching scheduler (Sec. 4.2 "Scheduling optimization for prefetching") ----------------------
def test_schedule_handworked_line():
    """Points on a line at 0, 10, 1, 11, 2, 12 (as one-hot-scaled vectors along the first axis), micro-batches
    of 3: the seed 0 takes its two nearest (1, then 2), the next seed is index 1 (at 10) and takes 11, 12."""
    pos = np.array([0.0, 10.0, 1.0, 11.0, 2.0, 12.0], dtype=np.float32)
    q = np.zeros((6, 4), dtype=np.float32)
    q[:, 0] = pos
    assert list(O.schedule(q, 3)) == [0, 2, 4, 1, 3, 5]
    assert list(O.schedule(q, 1)) == [0, 1, 2, 3, 4, 5]
    assert list(O.schedule(q, 2)) == [0, 2, 1, 3, 4, 5]          # 0 with 1; then 10 with 11; then 2 with 12
    # equal distances: the lower index first (seed at 0; 1 and -1 are equally far)
    q2 = np.zeros((3, 2), dtype=np.float32)
    q2[:, 0] = [0.0, 1.0, -1.0]
    assert list(O.schedule(q2, 3)) == [0, 1, 2]
    q2[:, 0] = [0.0, -1.0, 1.0]
    assert list(O.schedule(q2, 3)) == [0, 1, 2]


def test_schedule_whole_batch_is_an_argsort_and_invariants():
    rng = np.random.default_rng(21)
    for B, d, m in ((17, 5, 17), (40, 8, 100), (64, 16, 8), (33, 7, 4), (50, 3, 1)):
        q = rng.standard_normal((B, d)).astype(np.float32)
        order = O.schedule(q, m)
        assert sorted(order) == list(range(B))
        dist = ((q[:, None, :].astype(np.float64) - q[None, :, :].astype(np.float64)) ** 2).sum(-1)
        if m >= B:
            # one micro-batch: the seed, then everyone else by distance to it (numpy's stable argsort)
            assert order[0] == 0 and list(order[1:]) == list(np.argsort(dist[0][1:], kind="stable") + 1)
        left = set(range(B))
        for g0 in range(0, B, m):
            grp = list(order[g0:g0 + m])
            seed = grp[0]
            assert seed == min(left)                       # the lowest remaining index seeds the group
            left.remove(seed)
            for a, b in zip(grp[1:-1], grp[2:]):
                assert dist[seed, a] <= dist[seed, b]      # nearest first
            for x in grp[1:]:
                left.remove(x)
            if grp[1:] and left:
                assert dist[seed, grp[-1]] <= min(dist[seed, y] for y in left)   # nobody nearer was left out


def test_schedule_recovers_separated_groups():
    """Queries drawn tightly around well-separated centres, as many per centre as the micro-batch
    holds: every micro-batch is one centre's queries."""
    rng = np.random.default_rng(22)
    centres, m, d = 6, 5, 12
    c = 10.0 * rng.standard_normal((centres, d))
    label = rng.permutation(np.repeat(np.arange(centres), m))
    q = (c[label] + 0.01 * rng.standard_normal((centres * m, d))).astype(np.float32)
    order = O.schedule(q, m)
    for g0 in range(0, centres * m, m):
        assert len(set(label[order[g0:g0 + m]])) == 1


# ---- prefetch amount (App. C "Finding Prefetching Amount") ------------------------------------

def test_prefetch_amount_is_the_generation_window_on_a_pcie_class_link():
    """App. C, case 1: with a miss rate that falls linearly until everything is fetched and a link
    whose transfer time per byte exceeds what a fetched byte saves the CPU, the best amount is what
    the link moves during generation, B * t_LLM, and the time is t_LLM plus the CPU's share."""
    B, t_llm, nprobe, t_cc = 50e9, 0.020, 256, 20e-6
    b_full = 4e9                                           # the miss rate reaches 0 here
    bs = np.array([0.0, b_full])
    rs = np.array([1.0, 0.0])
    assert nprobe * t_cc / b_full < 1.0 / B               # a byte costs more to move than it saves
    b, t = O.prefetch_amount(B, t_llm, nprobe, t_cc, bs, rs, step=1e6)
    assert b == B * t_llm
    assert t == pytest.approx(t_llm + (1.0 - B * t_llm / b_full) * nprobe * t_cc, rel=1e-12)


def test_prefetch_amount_goes_beyond_the_window_when_cpu_search_is_slow():
    """App. C, case 2 with a linear miss rate: when a fetched byte saves more CPU time than it costs
    to move (nprobe * t_cc / b_full > 1 / B), every further byte pays and the best amount is
    everything (the derivative never reaches zero before the miss rate does)."""
    B, t_llm, nprobe, t_cc = 50e9, 0.005, 256, 2e-3
    b_full = 2e9
    assert nprobe * t_cc / b_full > 1.0 / B and b_full > B * t_llm
    b, t = O.prefetch_amount(B, t_llm, nprobe, t_cc, np.array([0.0, b_full]), np.array([1.0, 0.0]), step=1e6)
    assert b == b_full and t == pytest.approx(b_full / B, rel=1e-12)


def test_prefetch_amount_stationary_point_of_a_convex_miss_curve():
    """App. C, case 2: for r_miss(b) = exp(-b / s), sampled finely, the derivative condition
    1 / B + r'(b) nprobe t_cc = 0 gives b* = s ln(B nprobe t_cc / s) when that lies beyond
    B * t_LLM; otherwise the answer is B * t_LLM."""
    B, nprobe, t_cc, s = 50e9, 256, 1e-3, 1e9
    bs = np.arange(0.0, 12e9 + 1, 1e6)
    rs = np.exp(-bs / s)
    b_star = s * np.log(B * nprobe * t_cc / s)
    assert b_star > 1e9
    b, t = O.prefetch_amount(B, 0.010, nprobe, t_cc, bs, rs, step=1e6)          # window 0.5 GB < b*
    assert abs(b - b_star) <= 2e6
    assert t == pytest.approx(b_star / B + np.exp(-b_star / s) * nprobe * t_cc, rel=1e-6)
    b, t = O.prefetch_amount(B, 0.100, nprobe, t_cc, bs, rs, step=1e6)          # window 5 GB > b*
    assert b == B * 0.100


def test_prefetch_amount_brute_force_on_random_convex_curves():
    """The grid search against numpy's own argmin of the same objective on random convex,
    non-increasing curves, and: the result never lies below the generation window."""
    rng = np.random.default_rng(12)
    for _ in range(50):
        n = int(rng.integers(2, 12))
        bs = np.concatenate([[0.0], np.cumsum(rng.integers(1, 40, n - 1)) * 1e8])
        slopes = -np.sort(rng.random(n - 1))[::-1]                        # rising towards 0: convex
        rs = np.concatenate([[0.0], np.cumsum(slopes * np.diff(bs))])
        rs = (rs - rs.min()) / max(rs.max() - rs.min(), 1e-30)           # from 1 down to 0
        B = float(rng.choice([16e9, 50e9, 400e9]))
        t_llm, nprobe, t_cc = float(rng.uniform(0.001, 0.05)), int(rng.integers(1, 512)), float(rng.uniform(1e-6, 1e-3))
        step = 1e7
        b, t = O.prefetch_amount(B, t_llm, nprobe, t_cc, bs, rs, step)
        grid = np.append(np.arange(0.0, max(B * t_llm, bs[-1]) + 0.5, step), B * t_llm)
        obj = np.where(grid <= B * t_llm, t_llm, grid / B) + np.interp(grid, bs, rs) * nprobe * t_cc
        assert t == pytest.approx(obj.min(), rel=1e-12, abs=1e-15)
        assert b >= B * t_llm - 1e-3
