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


# ---- how much to prefetch (App. C "Finding Prefetching Amount") ------------------------------

def test_prefetch_amount_equals_the_oracle_on_random_curves():
    """ivf_prefetch_amount looks only at bandwidth * t_llm and the measured points beyond it; the
    oracle tries every amount on a grid that contains those points.  Both must name the same amount
    and the same time, on convex curves (the paper's assumption) and on curves that are merely
    non-increasing."""
    rng = np.random.default_rng(44)
    cases = {1: 0, 2: 0}
    for trial in range(300):
        n = int(rng.integers(1, 14))
        bs = np.concatenate([[float(rng.integers(0, 3)) * 1e8], np.zeros(n - 1)])
        bs[1:] = bs[0] + np.cumsum(rng.integers(1, 40, n - 1)) * 1e8
        if trial % 2 == 0:
            slopes = -np.sort(rng.random(n - 1))[::-1]                    # convex
        else:
            slopes = -rng.random(n - 1) * (rng.random(n - 1) < 0.7)       # any non-increasing curve, with flat pieces
        rs = np.concatenate([[0.0], np.cumsum(slopes * np.diff(bs))]) if n > 1 else np.zeros(1)
        span = rs.max() - rs.min()
        rs = (rs - rs.min()) / span * rng.uniform(0.3, 1.0) if span > 0 else np.full(n, rng.uniform(0, 1))
        B = float(rng.choice([16e9, 52e9, 64e9, 400e9]))
        t_llm = float(rng.choice([0.0, rng.uniform(0.001, 0.05)]))
        nprobe, t_cc = int(rng.integers(1, 512)), float(rng.choice([0.0, rng.uniform(1e-6, 3e-3)]))
        amount, seconds, which = P.ivf_prefetch_amount(B, t_llm, nprobe, t_cc, bs, rs)
        ob, ot = O.prefetch_amount(B, t_llm, nprobe, t_cc, bs, rs, step=1e7)
        assert amount == ob, (trial, amount, ob)
        assert seconds == pytest.approx(ot, rel=1e-12, abs=1e-18)
        assert which == (1 if amount == B * t_llm else 2)
        cases[which] += 1
    assert cases[1] > 30 and cases[2] > 30              # both cases of App. C were met


def test_prefetch_amount_of_a_measured_sweep():
    """Numbers of the kind the lookahead benchmark measures: 52 GB/s, 18 ms of generation, nprobe 256,
    5 us of host time per missed cluster: a byte costs more to move than it saves, so the answer is
    the generation window, 0.936 GB, with the miss rate read off the line between the measured points."""
    bs = np.array([0.0, 0.25e9, 0.5e9, 0.9e9, 1.28e9, 2.0e9])
    rs = np.array([1.0, 0.83, 0.67, 0.47, 0.32, 0.27])
    amount, seconds, which = P.ivf_prefetch_amount(52e9, 0.018, 256, 5e-6, bs, rs)
    assert which == 1 and amount == 52e9 * 0.018
    r = 0.47 + (0.32 - 0.47) * (0.936e9 - 0.9e9) / (1.28e9 - 0.9e9)
    assert seconds == pytest.approx(0.018 + r * 256 * 5e-6, rel=1e-12)
    # a host that needs 1 ms per missed cluster changes the answer: every measured point pays until the curve flattens
    amount, seconds, which = P.ivf_prefetch_amount(52e9, 0.018, 256, 1e-3, bs, rs)
    assert which == 2 and amount == 1.28e9
    assert seconds == pytest.approx(1.28e9 / 52e9 + 0.32 * 256 * 1e-3, rel=1e-12)


def test_prefetch_amount_rejects_bad_arguments():
    bs, rs = np.array([0.0, 1e9]), np.array([1.0, 0.5])
    for args in ((0.0, 0.01, 8, 1e-5, bs, rs), (1e9, -1.0, 8, 1e-5, bs, rs), (1e9, 0.01, 0, 1e-5, bs, rs),
                 (1e9, 0.01, 8, -1e-5, bs, rs), (1e9, 0.01, 8, 1e-5, bs[::-1].copy(), rs),
                 (1e9, 0.01, 8, 1e-5, bs, rs[::-1].copy()), (1e9, 0.01, 8, 1e-5, bs, np.array([1.5, 0.5])),
                 (float("nan"), 0.01, 8, 1e-5, bs, rs)):
        with pytest.raises(P.binding.IvfError) as e:
            P.ivf_prefetch_amount(*args)
        assert e.value.status == -1
