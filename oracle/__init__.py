"""ctypes front end of the CPU oracle (oracle/ivf_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg, never by the product package.  The arithmetic all
lives in the C file; this module only marshals numpy arrays.
"""
import ctypes as C
import os

import numpy as np

from .build import LIB, build

IP, L2 = 0, 1
F32, F16, BF16 = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        L = C.CDLL(LIB)
        L.orc_widen.restype = C.c_double
        L.orc_widen.argtypes = [C.c_uint16, C.c_int]
        L.orc_score.restype = C.c_double
        L.orc_score.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int32, C.c_int]
        L.orc_threads.restype = C.c_int
        vp, i32, i64, u64, ci = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_int
        sigs = {
            "orc_build_layout": [vp, i64, i32, vp, vp],
            "orc_probe": [vp, i32, i32, ci, vp, i32, vp, vp],
            "orc_search": [vp, ci, vp, vp, vp, i32, i32, ci, vp, i32, i32, vp, vp],
            "orc_search_clusters": [vp, ci, vp, vp, i32, ci, vp, vp, i32, i32, vp, vp],
            "orc_prefetch": [vp, i32, i32, ci, vp, ci, vp, i32, u64, u64, vp, vp, vp, vp, vp],
            "orc_split": [vp, i32, i32, ci, vp, i32, vp, vp, vp, vp, vp],
            "orc_hybrid": [vp, ci, vp, vp, vp, i32, i32, ci, vp, i32, i32, vp, vp, vp, vp],
            "orc_schedule": [vp, i32, i32, i32, vp],
            "orc_cache_round": [vp, vp, vp, vp, i32, i32, ci, C.c_float, C.c_float, C.c_double, u64, vp, vp],
        }
        L.orc_prefetch_amount.restype = C.c_double
        L.orc_prefetch_amount.argtypes = [C.c_double, C.c_double, i32, C.c_double, vp, vp, i32, C.c_double, vp]
        L.orc_cache_admit.restype = None
        L.orc_cache_admit.argtypes = [vp, vp, i32, C.c_float]
        for name, args in sigs.items():
            getattr(L, name).restype = C.c_int32
            getattr(L, name).argtypes = args
        _lib = L
    return _lib


def _p(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _rows(lists, dtype):
    """Row storage as the oracle reads it: float32, or raw 16-bit patterns."""
    if dtype == F32:
        return np.ascontiguousarray(lists, dtype=np.float32)
    a = np.ascontiguousarray(lists)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, "fp16/bf16 rows are passed as float16 or raw uint16 patterns"
    return a


def widen(bits, dtype):
    return lib().orc_widen(int(bits), int(dtype))


def threads():
    return lib().orc_threads()


def score(x, rows, dtype, row, metric):
    rows = _rows(rows, dtype)
    x = _f32(x)
    return lib().orc_score(_p(x), _p(rows), dtype, int(row), x.shape[0], metric)


def build_layout(assign, nlist):
    assign = np.ascontiguousarray(assign, dtype=np.int32)
    n = assign.shape[0]
    off = np.zeros(nlist + 1, dtype=np.int64)
    perm = np.zeros(n, dtype=np.int64)
    rc = lib().orc_build_layout(_p(assign), C.c_int64(n), C.c_int32(nlist), _p(off), _p(perm))
    if rc != 0:
        raise ValueError("assignment outside [0, nlist)")
    return off, perm


def probe(centroids, x, L, metric, with_scores=False):
    centroids = _f32(centroids)
    x = _f32(x)
    nlist, d = centroids.shape
    Lc = min(L, nlist)
    out = np.zeros(max(Lc, 1), dtype=np.int32)
    sc = np.zeros(max(Lc, 1), dtype=np.float64)
    got = lib().orc_probe(_p(centroids), nlist, d, metric, _p(x), L, _p(out), _p(sc))
    assert got == Lc
    return (out[:got], sc[:got]) if with_scores else out[:got]


def search_clusters(lists, dtype, off, ids, x, clusters, k, metric):
    rows = _rows(lists, dtype)
    off = np.ascontiguousarray(off, dtype=np.int64)
    ids = None if ids is None else np.ascontiguousarray(ids, dtype=np.int64)
    x = _f32(x)
    clusters = np.ascontiguousarray(clusters, dtype=np.int32)
    oi = np.zeros(k, dtype=np.int64)
    os_ = np.zeros(k, dtype=np.float64)
    rc = lib().orc_search_clusters(_p(rows), dtype, _p(off), _p(ids), x.shape[0], metric, _p(x),
                                   _p(clusters), clusters.shape[0], k, _p(oi), _p(os_))
    assert rc == 0
    return oi, os_


def search(lists, dtype, off, ids, centroids, x, L, k, metric):
    rows = _rows(lists, dtype)
    off = np.ascontiguousarray(off, dtype=np.int64)
    ids = None if ids is None else np.ascontiguousarray(ids, dtype=np.int64)
    centroids = _f32(centroids)
    x = _f32(x)
    nlist, d = centroids.shape
    oi = np.zeros(k, dtype=np.int64)
    os_ = np.zeros(k, dtype=np.float64)
    rc = lib().orc_search(_p(rows), dtype, _p(off), _p(ids), _p(centroids), nlist, d, metric,
                          _p(x), L, k, _p(oi), _p(os_))
    assert rc == 0
    return oi, os_


class Residency:
    """Which clusters sit in the device buffer, and how many bytes they take."""

    def __init__(self, nlist, cap):
        self.flags = np.zeros(nlist, dtype=np.uint8)
        self.used = C.c_uint64(0)
        self.cap = int(cap)

    def reset(self):
        self.flags[:] = 0
        self.used = C.c_uint64(0)

    def clusters(self):
        return np.nonzero(self.flags)[0].astype(np.int32)


def prefetch(centroids, off, dtype, x_in, L, budget, res, metric):
    """Returns (chosen clusters in the order taken, n_skipped, bytes_taken)."""
    centroids = _f32(centroids)
    off = np.ascontiguousarray(off, dtype=np.int64)
    x_in = _f32(x_in)
    nlist, d = centroids.shape
    chosen = np.zeros(max(min(L, nlist), 1), dtype=np.int32)
    skipped = C.c_int32(0)
    nbytes = C.c_uint64(0)
    got = lib().orc_prefetch(_p(centroids), nlist, d, metric, _p(off), dtype, _p(x_in), L,
                             C.c_uint64(int(budget)), C.c_uint64(res.cap), _p(res.flags),
                             C.byref(res.used), _p(chosen), C.byref(skipped), C.byref(nbytes))
    assert got >= 0
    return chosen[:got], skipped.value, nbytes.value


def cache_admit(hot, res, h_init):
    """Newly resident clusters (hot < 0) start at h_init.  hot: float32[nlist], updated in place."""
    assert hot.dtype == np.float32 and hot.flags.c_contiguous
    lib().orc_cache_admit(_p(hot), _p(res.flags), len(hot), C.c_float(h_init))


def cache_round(hot, used_flags, res, off, d, dtype, decay, h_inc, fraction):
    """One hotness round and the eviction that ends a batch; updates hot, used_flags (cleared),
    res.flags and res.used in place.  Returns the evicted clusters in the order they left."""
    assert hot.dtype == np.float32 and used_flags.dtype == np.uint8
    off = np.ascontiguousarray(off, dtype=np.int64)
    nlist = len(hot)
    evicted = np.zeros(max(nlist, 1), dtype=np.int32)
    n = lib().orc_cache_round(_p(hot), _p(used_flags), _p(res.flags), _p(off), nlist, d, dtype,
                              C.c_float(decay), C.c_float(h_inc), C.c_double(fraction), C.c_uint64(res.cap),
                              C.byref(res.used), _p(evicted))
    assert n >= 0
    return evicted[:n]


def prefetch_amount(bandwidth, t_llm, nprobe, t_cc, budgets, miss_rates, step):
    """App. C: the prefetch amount (bytes) that minimises t_1 + t_2, tried on a grid of `step` bytes,
    and that time.  budgets / miss_rates: the measured miss-rate curve."""
    bs = np.ascontiguousarray(budgets, dtype=np.float64)
    rs = np.ascontiguousarray(miss_rates, dtype=np.float64)
    assert bs.ndim == 1 and bs.shape == rs.shape and bs.shape[0] >= 1 and np.all(np.diff(bs) > 0)
    t = C.c_double(0.0)
    b = lib().orc_prefetch_amount(float(bandwidth), float(t_llm), int(nprobe), float(t_cc), _p(bs), _p(rs),
                                  bs.shape[0], float(step), C.byref(t))
    return b, t.value


def schedule(q, micro):
    """Greedy grouping of the queries q [B, d] into micro-batches of `micro`; returns the order."""
    q = _f32(q)
    B, d = q.shape
    order = np.zeros(B, dtype=np.int32)
    assert lib().orc_schedule(_p(q), B, d, int(micro), _p(order)) == B
    return order


def split(centroids, x_out, L, res_flags, metric):
    centroids = _f32(centroids)
    x_out = _f32(x_out)
    nlist, d = centroids.shape
    res_flags = np.ascontiguousarray(res_flags, dtype=np.uint8)
    cap = max(min(L, nlist), 1)
    ov = np.zeros(cap, dtype=np.int32)
    ms = np.zeros(cap, dtype=np.int32)
    no, nm = C.c_int32(0), C.c_int32(0)
    got = lib().orc_split(_p(centroids), nlist, d, metric, _p(x_out), L, _p(res_flags),
                          _p(ov), C.byref(no), _p(ms), C.byref(nm))
    assert got == no.value + nm.value
    return ov[:no.value], ms[:nm.value]


def hybrid(lists, dtype, off, ids, centroids, x_out, L, k, res_flags, metric):
    """Returns (ids, scores, hit_rate)."""
    rows = _rows(lists, dtype)
    off = np.ascontiguousarray(off, dtype=np.int64)
    ids = None if ids is None else np.ascontiguousarray(ids, dtype=np.int64)
    centroids = _f32(centroids)
    x_out = _f32(x_out)
    nlist, d = centroids.shape
    res_flags = np.ascontiguousarray(res_flags, dtype=np.uint8)
    oi = np.zeros(k, dtype=np.int64)
    os_ = np.zeros(k, dtype=np.float64)
    hr = C.c_double(0.0)
    rc = lib().orc_hybrid(_p(rows), dtype, _p(off), _p(ids), _p(centroids), nlist, d, metric,
                          _p(x_out), L, k, _p(res_flags), _p(oi), _p(os_), C.byref(hr))
    assert rc == 0
    return oi, os_, hr.value
