"""The budget walk of ivf_prefetch (Sec. 4.3 'Prefetching target'; several queries per call:
Sec. 4.2 'Batching'; later rounds: Sec. 4.3 'Prefetching for multi-round') against the oracle,
without a GPU.  ivf_prefetch runs this same code after ranking the clusters on the GPU."""
import json
import os

import numpy as np
import pytest

import oracle as O
import paper_2502_20969_amd as P


def _index(seed, nlist, d):
    rng = np.random.default_rng(seed)
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    sizes = rng.integers(0, 400, nlist)
    sizes[rng.integers(0, nlist, 3)] = 0                       # empty clusters are legal
    off = np.zeros(nlist + 1, dtype=np.int64)
    off[1:] = np.cumsum(sizes)
    return cent, off, rng


@pytest.mark.parametrize("dtype,esz", [(O.F32, 4), (O.F16, 2)])
@pytest.mark.parametrize("nq", [1, 3, 8])
def test_plan_equals_the_oracle_over_rounds(dtype, esz, nq):
    nlist, d, L = 60, 24, 14
    cent, off, rng = _index(nq * 10 + esz, nlist, d)
    rb = d * esz
    total = int(off[-1]) * rb
    for cap in (total // 5, total * 2):
        res = O.Residency(nlist, cap)
        res_off = np.full(nlist, -1, dtype=np.int64)
        used = 0
        for rnd, budget in enumerate([0, rb * 50, total // 8, total // 3, 1 << 40]):
            q = rng.standard_normal((nq, d)).astype(np.float32)
            ranked = np.stack([O.probe(cent, q[b], L, O.IP) for b in range(nq)]).astype(np.int32)
            want, want_skipped, want_bytes = [], 0, 0
            for b in range(nq):                                # equal shares, queries in order, one residency
                ch, sk, nb = O.prefetch(cent, off, dtype, q[b], L, budget // nq, res, O.IP)
                want += list(ch); want_skipped += sk; want_bytes += nb
            before = res_off.copy()
            taken, st, used = P.ivf_prefetch_plan(ranked, off, rb, budget, cap, res_off, used)
            assert list(taken) == want, f"cap {cap} round {rnd}"
            assert st.n_taken == len(want) and st.n_skipped == want_skipped and st.bytes == want_bytes
            assert st.n_ranked == nq * L and st.n_resident == nq * L - len(want) - want_skipped
            assert used == res.used.value == st.buffer_used and used <= cap
            assert list(np.flatnonzero(res_off >= 0)) == list(res.clusters())
            assert np.array_equal(res_off[before >= 0], before[before >= 0])      # nothing moves
            # clusters sit back to back in the order taken
            mark = (used - want_bytes) // rb
            for c in taken:
                assert res_off[c] == mark
                mark += off[c + 1] - off[c]


def test_plan_of_the_hand_worked_example():
    """The lookahead part of the hand-worked fixture (tests/golden/handworked_ivf.json, worked from
    Sec. 4.1 step 1 and Sec. 4.3 'Prefetching target'): four lists of 16, 16, 8, 16 bytes, q_in ranks
    lists 0 and 3 first."""
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "handworked_ivf.json")))
    look = g["lookahead_ip_fp32"]
    rows = [len(g["lists"][str(c)]["ids"]) for c in range(4)]
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int64)
    rb = g["d"] * 4
    assert [int(r) * rb for r in rows] == look["list_bytes"]
    ranked = np.array([g["ip"]["probe2_q_in"]], dtype=np.int32)
    for budget, key in ((1 << 40, "budget_inf"), (20, "budget_20"), (0, "budget_0")):
        res_off = np.full(4, -1, dtype=np.int64)
        taken, st, used = P.ivf_prefetch_plan(ranked, off, rb, budget, 1 << 20, res_off, 0)
        assert sorted(taken.tolist()) == look[key]["resident"]
        assert list(np.flatnonzero(res_off >= 0)) == look[key]["resident"]
        if "skipped" in look[key]:
            assert st.n_skipped == look[key]["skipped"] and st.bytes == look[key]["bytes"]


def test_plan_rejects_bad_arguments():
    off = np.array([0, 2, 4], dtype=np.int64)
    res_off = np.full(2, -1, dtype=np.int64)
    with pytest.raises(P.binding.IvfError) as e:
        P.ivf_prefetch_plan(np.array([[0, 2]], dtype=np.int32), off, 8, 100, 1000, res_off, 0)
    assert e.value.status == -1
    with pytest.raises(P.binding.IvfError) as e:
        P.ivf_prefetch_plan(np.array([[0, 1]], dtype=np.int32), off, 8, 100, 10, res_off, 11)
    assert e.value.status == -1
