"""The host part of a cache round (Sec. 4.2 'Cache design': eviction down to the cache fraction,
then consolidation of the buffer) against the oracle and against a byte-level simulation of the
moves, without a GPU.  ivf_cache_end_round runs this same code after the hotness update."""
import numpy as np
import pytest

import oracle as O
import paper_2502_20969_amd as P


def _state(seed, nlist, rb, fill):
    """Random sizes, a random subset cached at scattered (non-overlapping, gappy) buffer places."""
    rng = np.random.default_rng(seed)
    sizes = rng.integers(0, 50, nlist)
    sizes[rng.integers(0, nlist, 2)] = 0
    off = np.zeros(nlist + 1, dtype=np.int64)
    off[1:] = np.cumsum(sizes)
    cached = rng.permutation(nlist)[:int(nlist * fill)]
    order = rng.permutation(cached)                    # buffer order is not cluster order
    res_off = np.full(nlist, -1, dtype=np.int64)
    at = 0
    for c in order:
        at += int(rng.integers(0, 30))                 # a gap left by an earlier eviction
        res_off[c] = at
        at += int(sizes[c])
    hot = np.full(nlist, -1.0, dtype=np.float32)
    hot[cached] = rng.choice(np.array([0.25, 0.5, 1.0, 1.5, 2.0], dtype=np.float32), len(cached))   # many ties
    return off, sizes, res_off, hot, at * rb, rng


@pytest.mark.parametrize("fraction", [0.0, 0.3, 0.5, 1.0])
@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_plan_evicts_like_the_oracle_and_moves_every_byte_right(seed, fraction):
    nlist, rb = 70, 16
    off, sizes, res_off, hot, end_bytes, rng = _state(seed, nlist, rb, 0.6)
    cap = int(end_bytes * 1.2)
    used = int(sizes[res_off >= 0].sum()) * rb
    # the buffer as it is: every cached cluster's bytes are its cluster number (mod 251) + position
    buf = np.full(cap, 255, dtype=np.uint8)
    content = {}
    for c in np.flatnonzero(res_off >= 0):
        n = int(sizes[c]) * rb
        content[c] = ((np.arange(n) * 7 + c * 13) % 251).astype(np.uint8)
        buf[res_off[c] * rb:res_off[c] * rb + n] = content[c]
    # oracle: the order in which clusters would leave if all had to (decay 1, no increment, nothing
    # used: the hotness stays as it is)
    ores = O.Residency(nlist, cap)
    ores.flags[res_off >= 0] = 1
    ores.used.value = used
    leave_order = O.cache_round(hot.copy(), np.zeros(nlist, dtype=np.uint8), ores, off, rb // 4, O.F32, 1.0, 0.0, 0.0)
    order_before = [c for c in np.argsort(res_off, kind="stable") if res_off[c] >= 0]
    before_res = res_off.copy()
    # this buffer has gaps, so the bytes in use (its fill mark) exceed the cached bytes: the
    # coldest clusters leave, in the oracle's order, until the mark minus what left fits the limit
    evicted, moves, new_used = P.ivf_cache_plan(hot, off, rb, res_off, end_bytes, cap, fraction)
    m = min(len(evicted), len(leave_order))      # (the oracle stops at zero bytes; an empty cluster may stay there)
    assert list(evicted[:m]) == list(leave_order[:m])
    limit = int(fraction * cap)
    left = [int(sizes[c]) * rb for c in evicted]
    assert end_bytes - sum(left) <= limit or len(evicted) == int((before_res >= 0).sum())
    assert len(evicted) == 0 or end_bytes - sum(left[:-1]) > limit
    survivors = [c for c in order_before if res_off[c] >= 0]
    assert set(order_before) - set(survivors) == set(evicted.tolist())
    assert all(hot[c] == -1.0 for c in evicted)
    # survivors: packed from 0 in their old order
    at = 0
    for c in survivors:
        assert res_off[c] * rb == at
        at += int(sizes[c]) * rb
    assert new_used == at
    # carry out the moves on the bytes: staging when asked for, plain copy otherwise (a plain copy
    # of overlapping ranges is done front to back here, as a device copy may do it)
    for c, via, src, dst, n in moves:
        assert n == int(sizes[c]) * rb and dst < src
        assert via == (1 if src - dst < n else 0)
        if via:
            tmp = buf[src:src + n].copy()
            buf[dst:dst + n] = tmp
        else:
            for i in range(0, n, 64):                  # chunked forward copy; ranges do not overlap
                buf[dst + i:dst + min(i + 64, n)] = buf[src + i:src + min(i + 64, n)]
    for c in survivors:
        n = int(sizes[c]) * rb
        assert np.array_equal(buf[res_off[c] * rb:res_off[c] * rb + n], content[c]), f"cluster {c} was damaged"


@pytest.mark.parametrize("fraction", [0.2, 0.5, 0.8])
def test_plan_on_a_packed_buffer_equals_the_oracle(fraction):
    """A buffer without gaps (what prefetching alone produces): bytes in use = cached bytes, so the
    eviction must be the oracle's, in its order, ties included."""
    nlist, rb = 90, 8
    rng = np.random.default_rng(int(fraction * 10))
    sizes = rng.integers(0, 40, nlist)
    off = np.zeros(nlist + 1, dtype=np.int64)
    off[1:] = np.cumsum(sizes)
    cached = rng.permutation(nlist)[:60]
    res_off = np.full(nlist, -1, dtype=np.int64)
    at = 0
    for c in cached:
        res_off[c] = at
        at += int(sizes[c])
    used = at * rb
    cap = used + 100
    hot = np.full(nlist, -1.0, dtype=np.float32)
    hot[cached] = rng.choice(np.array([0.5, 1.0, 1.5], dtype=np.float32), len(cached))
    ores = O.Residency(nlist, cap)
    ores.flags[res_off >= 0] = 1
    ores.used.value = used
    ohot = hot.copy()
    want = O.cache_round(ohot, np.zeros(nlist, dtype=np.uint8), ores, off, rb // 4, O.F32, 1.0, 0.0, fraction)
    evicted, moves, new_used = P.ivf_cache_plan(hot, off, rb, res_off, used, cap, fraction)
    assert list(evicted) == list(want) and len(want) > 0
    assert np.array_equal(hot, ohot)
    assert new_used == ores.used.value
    assert list(np.flatnonzero(res_off >= 0)) == list(ores.clusters())


def test_plan_rejects_bad_arguments():
    off = np.array([0, 2, 4], dtype=np.int64)
    with pytest.raises(P.binding.IvfError) as e:
        P.ivf_cache_plan(np.zeros(2, dtype=np.float32), off, 8, np.full(2, -1, dtype=np.int64), 0, 100, 1.5)
    assert e.value.status == -1
