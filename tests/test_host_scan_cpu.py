"""The host part of the hybrid search (Sec. 4.1 step 3) against the oracle, without a GPU: the
candidates `ivf_host_scan` hands to the merge step contain the oracle's k nearest rows of the
scanned clusters, with the same float64 scores."""
import numpy as np
import pytest

import oracle as O
import paper_2502_20969_amd as P
from parity import NEAR_TIE, stored


def _problem(seed, n, d, nlist, dtype, dup=0):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((nlist, d)).astype(np.float32)
    assign = np.sort(rng.integers(0, nlist, n)).astype(np.int32)          # cluster-major
    assign[assign == 3 % nlist] = (3 % nlist + 1) % nlist if nlist > 1 else 0   # an empty list
    assign = np.sort(assign)
    rows = (centres[assign] + 0.5 * rng.standard_normal((n, d))).astype(np.float32)
    rows /= np.linalg.norm(rows, axis=1, keepdims=True)
    if dup:
        rows[rng.integers(0, n, dup)] = rows[rng.integers(0, n, dup)]
    off = np.zeros(nlist + 1, dtype=np.int64)
    off[1:] = np.cumsum(np.bincount(assign, minlength=nlist))
    st, odt = stored(rows, dtype)
    return st, odt, off, centres, rng


@pytest.mark.parametrize("metric", ["ip", "l2"])
@pytest.mark.parametrize("dtype,d", [("f32", 128), ("f16", 96), ("bf16", 64), ("f32", 100), ("f16", 7), ("f32", 768)])
@pytest.mark.parametrize("threads", [1, 5])
def test_host_scan_candidates_contain_the_oracles_top_k(dtype, d, metric, threads):
    pm, om = (P.IVF_IP, O.IP) if metric == "ip" else (P.IVF_L2, O.L2)
    n, nlist = 3000, 12
    st, odt, off, cent, rng = _problem(d * 7 + threads, n, d, nlist, dtype, dup=n // 4)
    ids = (rng.permutation(n).astype(np.int64) * 7 + 5)
    for trial, (k, ncl) in enumerate([(1, 1), (10, 4), (10, nlist), (100, 7), (5, 0)]):
        q = rng.standard_normal(d).astype(np.float32)
        clusters = rng.permutation(nlist)[:ncl].astype(np.int32)
        use_ids = ids if trial % 2 == 0 else None
        gi, gs = P.ivf_host_scan(st, dtype, off, q, clusters, k, ids=use_ids, metric=pm, threads=threads)
        assert len(gi) <= k + max(8, k // 8)
        assert len(set(gi.tolist())) == len(gi)                       # no row twice
        oi, osc = O.search_clusters(st, odt, off, use_ids, q, clusters, k, om)
        valid = oi >= 0
        score_of = dict(zip(gi.tolist(), gs.tolist()))
        # the candidates, ordered as the merge step orders them, start with the oracle's answer
        sign = -1.0 if metric == "ip" else 1.0
        order = sorted(range(len(gi)), key=lambda i: (sign * gs[i], gi[i]))
        mine = [int(gi[i]) for i in order][:int(valid.sum())]
        for pos, (want, got) in enumerate(zip(oi[valid].tolist(), mine)):
            if want != got:                                            # only a near-tie may differ
                assert got in score_of and abs(score_of[got] - osc[pos]) <= NEAR_TIE * max(abs(osc[pos]), 1e-300), \
                    f"trial {trial} pos {pos}: {got} vs {want}"
            else:
                np.testing.assert_allclose(score_of[got], osc[pos], rtol=1e-12, atol=1e-12)
        assert int(valid.sum()) == min(k, int(sum(off[c + 1] - off[c] for c in clusters)))


def test_host_scan_rejects_bad_arguments():
    rows = np.zeros((4, 8), dtype=np.float32)
    off = np.array([0, 4], dtype=np.int64)
    q = np.zeros(8, dtype=np.float32)
    with pytest.raises(P.binding.IvfError) as e:
        P.ivf_host_scan(rows, "f32", off, q, np.array([0], dtype=np.int32), 0)
    assert e.value.status == -1
    with pytest.raises(P.binding.IvfError) as e:
        P.ivf_host_scan(rows, "f32", off, q, np.array([0], dtype=np.int32), 10, threads=0)
    assert e.value.status == -1
    with pytest.raises(P.binding.IvfError) as e:
        P.ivf_host_scan(rows, "f32", off, q, np.array([0], dtype=np.int32), P.IVF_MAX_K + 1)
    assert e.value.status == -5


def test_host_scan_of_the_hand_worked_miss_list():
    """Hand-worked fixture (tests/golden/handworked_ivf.json): with an unlimited budget q_out's
    cluster 1 is the miss; its rows are ids 2 and 3 with inner products 0.25 and 0.3125, squared
    distances 0.8125 and 0.3125 (exact binary fractions)."""
    import json
    import os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "handworked_ivf.json")))
    rows, ids, off = [], [], [0]
    for c in range(4):
        rows += g["lists"][str(c)]["rows"]
        ids += g["lists"][str(c)]["ids"]
        off.append(len(rows))
    rows = np.array(rows, dtype=np.float32)
    miss = np.array(g["lookahead_ip_fp32"]["budget_inf"]["miss"], dtype=np.int32)
    for metric, key in ((P.IVF_IP, "ip"), (P.IVF_L2, "l2")):
        gi, gs = P.ivf_host_scan(rows, "f32", np.array(off, dtype=np.int64), np.array(g["q_out"], dtype=np.float32),
                                 miss, 3, ids=np.array(ids, dtype=np.int64), metric=metric, threads=2)
        got = dict(zip(gi.tolist(), gs.tolist()))
        want = {i: g[key]["row_scores_q_out"][str(i)] for i in (2, 3)}
        assert got == want
