"""ctypes binding of libivf.so: same names as include/ivf.h, argument marshalling only.

Host arguments are numpy arrays (or CPU torch tensors); device arguments are torch CUDA
tensors.  Nothing here computes: every step of the search runs in the HIP library, and the
module raises at import of the library if it has not been built.
"""
import collections
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libivf.so")

IVF_IP, IVF_L2 = 0, 1
IVF_F32, IVF_F16, IVF_BF16 = 0, 1, 2
IVF_PLACE_DEVICE, IVF_PLACE_HOST = 0, 1
IVF_PREFETCH_RESET = 1
IVF_MAX_K = 112
DTYPE_CODE = {"f32": IVF_F32, "f16": IVF_F16, "bf16": IVF_BF16}

EXPORTS = [
    "ivf_build_layout", "ivf_adopt_layout", "ivf_free", "ivf_prefetch", "ivf_prefetch_wait",
    "ivf_search", "ivf_search_device", "ivf_search_device_noalloc", "ivf_reserve", "ivf_coarse_scores", "ivf_probe",
    "ivf_resident", "ivf_batched_scores", "ivf_get_layout", "ivf_profile_enable", "ivf_profile_read",
    "ivf_profile_reset", "ivf_set_host_threads", "ivf_set_pipeline_depth", "ivf_synchronize",
    "ivf_set_batch_mode", "ivf_cache_configure", "ivf_cache_end_round", "ivf_cache_hotness",
    "ivf_schedule", "ivf_host_scan", "ivf_host_scan_capacity", "ivf_prefetch_amount", "ivf_prefetch_plan", "ivf_cache_plan", "ivf_strerror", "ivf_last_error",
]


class CacheStats(C.Structure):
    _fields_ = [("n_cached", C.c_int32), ("n_evicted", C.c_int32), ("bytes_cached", C.c_uint64),
                ("bytes_kept", C.c_uint64), ("bytes_moved", C.c_uint64), ("ms_update", C.c_float),
                ("ms_compact", C.c_float), ("n_launches", C.c_int32)]


class PrefetchStats(C.Structure):
    _fields_ = [("n_ranked", C.c_int32), ("n_taken", C.c_int32), ("n_skipped", C.c_int32),
                ("n_resident", C.c_int32), ("bytes", C.c_uint64), ("buffer_used", C.c_uint64)]


class SearchStats(C.Structure):
    _fields_ = [("n_probed", C.c_int32), ("n_overlap", C.c_int32), ("n_miss", C.c_int32),
                ("hit_rate", C.c_float), ("bytes_gpu", C.c_uint64), ("bytes_host", C.c_uint64),
                ("ms_total", C.c_float), ("ms_probe", C.c_float), ("ms_host_scan", C.c_float),
                ("n_exact_gpu", C.c_int32), ("n_exact_host", C.c_int32)]


class Profile(C.Structure):
    _fields_ = [("calls", C.c_uint64), ("ms_coarse", C.c_double), ("ms_select", C.c_double),
                ("ms_scan", C.c_double), ("ms_merge", C.c_double), ("scan_bytes", C.c_uint64),
                ("scan_rows", C.c_uint64)]


class IvfError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"libivf status {status}: {text}")
        self.status = status


_lib = None


def load():
    """Loads libivf.so; fails loudly when it is missing (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz, u32, ci = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_uint32, C.c_int
    L.ivf_build_layout.argtypes = [vp, i64, i32, ci, vp, i32, vp, vp, ci, ci, sz, vp, vp, C.POINTER(vp)]
    L.ivf_adopt_layout.argtypes = [vp, vp, vp, i64, i32, ci, vp, i32, ci, ci, sz, vp, vp, C.POINTER(vp)]
    L.ivf_free.argtypes = [vp]
    L.ivf_free.restype = None
    L.ivf_prefetch.argtypes = [vp, vp, i32, i32, sz, u32, C.POINTER(PrefetchStats)]
    L.ivf_prefetch_wait.argtypes = [vp, C.POINTER(C.c_float)]
    L.ivf_search.argtypes = [vp, vp, i32, i32, i32, vp, vp, C.POINTER(SearchStats)]
    L.ivf_search_device.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    L.ivf_search_device_noalloc.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    L.ivf_reserve.argtypes = [vp, i32, i32, i32]
    L.ivf_coarse_scores.argtypes = [vp, vp, i32, vp]
    L.ivf_probe.argtypes = [vp, vp, i32, i32, vp]
    L.ivf_resident.argtypes = [vp, vp, C.POINTER(i32)]
    L.ivf_batched_scores.argtypes = [vp, vp, i32, i32, vp, vp]
    L.ivf_get_layout.argtypes = [vp, vp, vp]
    L.ivf_profile_enable.argtypes = [vp, ci]
    L.ivf_profile_read.argtypes = [vp, C.POINTER(Profile)]
    L.ivf_profile_reset.argtypes = [vp]
    L.ivf_set_host_threads.argtypes = [vp, i32]
    L.ivf_set_pipeline_depth.argtypes = [vp, i32]
    L.ivf_synchronize.argtypes = [vp]
    L.ivf_set_batch_mode.argtypes = [vp, i32]
    L.ivf_cache_configure.argtypes = [vp, C.c_float, C.c_float, C.c_float, C.c_float]
    L.ivf_cache_end_round.argtypes = [vp, C.POINTER(CacheStats)]
    L.ivf_cache_hotness.argtypes = [vp, vp]
    L.ivf_schedule.argtypes = [vp, vp, i32, i32, vp, C.POINTER(C.c_float)]
    L.ivf_strerror.argtypes = [ci]
    L.ivf_strerror.restype = C.c_char_p
    L.ivf_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("ivf_free", "ivf_strerror", "ivf_last_error"):
            getattr(L, name).restype = ci
    _lib = L
    return L


_torch_mod = None


def _torch():
    global _torch_mod
    if _torch_mod is None:
        import torch
        _torch_mod = torch
    return _torch_mod


def _check(status):
    if status != 0:
        L = load()
        raise IvfError(status, f"{L.ivf_strerror(status).decode()} ({L.ivf_last_error().decode()})")


def _host(a, dtype):
    """numpy view of a host array in the dtype the ABI wants (no arithmetic, copies only if needed)."""
    if a is None:
        return None
    if hasattr(a, "detach"):          # torch CPU tensor
        assert a.device.type == "cpu", "expected a host array"
        import torch
        if a.dtype == torch.bfloat16:
            a = a.contiguous().view(torch.int16)
        a = a.detach().contiguous().numpy()
    if dtype is None:
        return np.ascontiguousarray(a)
    return np.ascontiguousarray(a, dtype=dtype)


def _ptr(a):
    if a is None:
        return None
    if hasattr(a, "data_ptr"):
        return C.c_void_p(a.data_ptr())
    return C.c_void_p(a.ctypes.data)


def _stream(s):
    return None if s is None else C.c_void_p(s.cuda_stream)


def _rows_host(vectors, dtype):
    code = DTYPE_CODE[dtype]
    if code == IVF_F32:
        return _host(vectors, np.float32)
    a = _host(vectors, None)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype == np.int16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"]
    return a


class Index:
    """Owner of one ivf_index handle."""

    def __init__(self, handle, d, nlist, n, keep=()):
        self._h = handle
        self.d, self.nlist, self.n = d, nlist, n
        self._keep = keep      # arrays the index adopted and that must outlive it
        # device tensors of searches the library may still touch (a pipelined or list-major call is
        # finished when its stream is next needed or in ivf_synchronize): one entry per stream at most
        self._inflight = collections.deque(maxlen=32)
        self._search_device = load().ivf_search_device
        t = _torch()
        self._f32, self._i64 = t.float32, t.int64

    def _device_triple(self, q_dev, k, ids_dev, dists_dev):
        """Checks the three device tensors of a device-side search (this runs once per search: kept short);
        returns the number of queries."""
        if q_dev.dtype is not self._f32 or ids_dev.dtype is not self._i64 or dists_dev.dtype is not self._f32:
            raise TypeError("queries and distances must be float32, ids int64")
        if not (q_dev.is_cuda and ids_dev.is_cuda and dists_dev.is_cuda):
            raise ValueError("expected CUDA tensors")
        if not (q_dev.is_contiguous() and ids_dev.is_contiguous() and dists_dev.is_contiguous()):
            raise ValueError("expected contiguous tensors")
        nq = q_dev.numel() // self.d
        if ids_dev.numel() < nq * k or dists_dev.numel() < nq * k:
            raise ValueError("ids / dists hold fewer than nq * k entries")
        return nq

    def close(self):
        if self._h is not None:
            load().ivf_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- lookahead -------------------------------------------------------------------------
    def ivf_prefetch(self, q_in, nprobe, budget_bytes, flags=0):
        q = _host(q_in, np.float32).reshape(-1, self.d)
        st = PrefetchStats()
        _check(load().ivf_prefetch(self._h, _ptr(q), q.shape[0], nprobe, int(budget_bytes), flags, C.byref(st)))
        return st

    def ivf_prefetch_wait(self):
        ms = C.c_float(0)
        _check(load().ivf_prefetch_wait(self._h, C.byref(ms)))
        return ms.value

    # -- search ------------------------------------------------------------------------------
    def ivf_search(self, q_out, nprobe, k, with_stats=False):
        q = _host(q_out, np.float32).reshape(-1, self.d)
        nq = q.shape[0]
        ids = np.empty((nq, k), dtype=np.int64)
        dists = np.empty((nq, k), dtype=np.float32)
        st = SearchStats()
        _check(load().ivf_search(self._h, _ptr(q), nq, nprobe, k, _ptr(ids), _ptr(dists), C.byref(st)
                                 if with_stats else None))
        return (ids, dists, st) if with_stats else (ids, dists)

    def ivf_search_device(self, q_dev, nprobe, k, ids_dev, dists_dev):
        """q_dev [nq, d] float32, ids_dev [nq, k] int64, dists_dev [nq, k] float32: CUDA tensors.
        The three tensors are kept referenced until ivf_synchronize (the library may read the queries
        and rewrite the outputs until then)."""
        nq = self._device_triple(q_dev, k, ids_dev, dists_dev)
        self._inflight.append((q_dev, ids_dev, dists_dev))
        status = self._search_device(self._h, q_dev.data_ptr(), nq, nprobe, k, ids_dev.data_ptr(), dists_dev.data_ptr())
        if status != 0:
            _check(status)

    def ivf_search_device_noalloc(self, q_dev, nprobe, k, ids_dev, dists_dev):
        """ivf_search_device on the library's fixed scratch area: allocates nothing."""
        nq = self._device_triple(q_dev, k, ids_dev, dists_dev)
        _check(load().ivf_search_device_noalloc(self._h, _ptr(q_dev), nq, nprobe, k, _ptr(ids_dev), _ptr(dists_dev)))

    def ivf_reserve(self, nq, nprobe, k):
        _check(load().ivf_reserve(self._h, nq, nprobe, k))

    # -- stages ------------------------------------------------------------------------------
    def ivf_coarse_scores(self, q):
        q = _host(q, np.float32).reshape(-1, self.d)
        out = np.empty((q.shape[0], self.nlist), dtype=np.float64)
        _check(load().ivf_coarse_scores(self._h, _ptr(q), q.shape[0], _ptr(out)))
        return out

    def ivf_probe(self, q, nprobe):
        q = _host(q, np.float32).reshape(-1, self.d)
        out = np.empty((q.shape[0], min(nprobe, self.nlist)), dtype=np.int32)
        _check(load().ivf_probe(self._h, _ptr(q), q.shape[0], nprobe, _ptr(out)))
        return out

    def ivf_batched_scores(self, q, cluster, rows_in_cluster):
        """MFMA filter scores [nq, rows] of one cluster and the error bound eps [nq] the scan assumes."""
        q = _host(q, np.float32).reshape(-1, self.d)
        scores = np.empty((q.shape[0], rows_in_cluster), dtype=np.float32)
        eps = np.empty(q.shape[0], dtype=np.float32)
        _check(load().ivf_batched_scores(self._h, _ptr(q), q.shape[0], int(cluster), _ptr(scores), _ptr(eps)))
        return scores, eps

    def ivf_resident(self):
        n = C.c_int32(self.nlist)
        out = np.empty(self.nlist, dtype=np.int32)
        _check(load().ivf_resident(self._h, _ptr(out), C.byref(n)))
        return out[:n.value].copy()

    def ivf_get_layout(self):
        off = np.empty(self.nlist + 1, dtype=np.int64)
        ids = np.empty(self.n, dtype=np.int64)
        _check(load().ivf_get_layout(self._h, _ptr(off), _ptr(ids)))
        return off, ids

    # -- prefetching scheduler ---------------------------------------------------------------
    def ivf_schedule(self, q, micro, with_time=False):
        q = _host(q, np.float32).reshape(-1, self.d)
        order = np.empty(q.shape[0], dtype=np.int32)
        ms = C.c_float(0)
        _check(load().ivf_schedule(self._h, _ptr(q), q.shape[0], int(micro), _ptr(order), C.byref(ms)))
        return (order, ms.value) if with_time else order

    # -- cluster cache -----------------------------------------------------------------------
    def ivf_cache_configure(self, fraction=0.5, h_init=1.0, decay=2.0, h_inc=1.0):
        _check(load().ivf_cache_configure(self._h, C.c_float(fraction), C.c_float(h_init), C.c_float(decay),
                                          C.c_float(h_inc)))

    def ivf_cache_end_round(self):
        st = CacheStats()
        _check(load().ivf_cache_end_round(self._h, C.byref(st)))
        return st

    def ivf_cache_hotness(self):
        out = np.empty(self.nlist, dtype=np.float32)
        _check(load().ivf_cache_hotness(self._h, _ptr(out)))
        return out

    # -- profiling ---------------------------------------------------------------------------
    def ivf_profile_enable(self, on=True):
        _check(load().ivf_profile_enable(self._h, 1 if on else 0))

    def ivf_profile_read(self):
        p = Profile()
        _check(load().ivf_profile_read(self._h, C.byref(p)))
        return p

    def ivf_profile_reset(self):
        _check(load().ivf_profile_reset(self._h))

    def ivf_set_host_threads(self, n):
        _check(load().ivf_set_host_threads(self._h, n))

    def ivf_set_pipeline_depth(self, depth):
        _check(load().ivf_set_pipeline_depth(self._h, depth))

    def ivf_synchronize(self):
        _check(load().ivf_synchronize(self._h))
        self._inflight.clear()

    def ivf_set_batch_mode(self, mode):
        _check(load().ivf_set_batch_mode(self._h, mode))


def ivf_build_layout(vectors, dtype, centroids, assign, ids=None, metric=IVF_IP,
                     placement=IVF_PLACE_DEVICE, device_buffer_bytes=0, compute_stream=None,
                     copy_stream=None):
    rows = _rows_host(vectors, dtype)
    cent = _host(centroids, np.float32)
    asg = _host(assign, np.int32)
    idv = _host(ids, np.int64)
    n, d = rows.shape
    nlist = cent.shape[0]
    assert cent.shape[1] == d and asg.shape[0] == n
    h = C.c_void_p()
    _check(load().ivf_build_layout(_ptr(rows), n, d, DTYPE_CODE[dtype], _ptr(cent), nlist, _ptr(asg),
                                   _ptr(idv), metric, placement, int(device_buffer_bytes),
                                   _stream(compute_stream), _stream(copy_stream), C.byref(h)))
    return Index(h, d, nlist, n)


def ivf_adopt_layout(lists, dtype, offsets, centroids, ids=None, metric=IVF_IP,
                     placement=IVF_PLACE_DEVICE, device_buffer_bytes=0, compute_stream=None,
                     copy_stream=None):
    """lists: torch tensor [n, d], on the GPU (device placement) or pinned on the host."""
    assert lists.is_contiguous()
    if placement == IVF_PLACE_DEVICE:
        assert lists.is_cuda
    else:
        assert (not lists.is_cuda) and lists.is_pinned()
    n, d = lists.shape
    cent = _host(centroids, np.float32)
    off = _host(offsets, np.int64)
    idv = _host(ids, np.int64)
    nlist = cent.shape[0]
    h = C.c_void_p()
    _check(load().ivf_adopt_layout(_ptr(lists), _ptr(off), _ptr(idv), n, d, DTYPE_CODE[dtype], _ptr(cent),
                                   nlist, metric, placement, int(device_buffer_bytes),
                                   _stream(compute_stream), _stream(copy_stream), C.byref(h)))
    return Index(h, d, nlist, n, keep=(lists,))


def ivf_host_scan(lists, dtype, offsets, q, clusters, k, ids=None, metric=IVF_IP, threads=4):
    """Host scan of the listed clusters for one query: (ids, float64 scores) of the candidates the
    merge step would receive, unordered.  lists: host array [n, d] in the stored type."""
    rows = _rows_host(lists, dtype)
    off = _host(offsets, np.int64)
    idv = _host(ids, np.int64)
    qv = _host(q, np.float32).reshape(-1)
    cl = _host(clusters, np.int32).reshape(-1)
    d = rows.shape[1]
    assert qv.shape[0] == d
    L = load()
    cap = max(1, int(L.ivf_host_scan_capacity(int(k))))      # 0 for a k the library will refuse below
    out_ids = np.empty(cap, dtype=np.int64)
    out_scores = np.empty(cap, dtype=np.float64)
    n_out = C.c_int32(0)
    _check(L.ivf_host_scan(_ptr(rows), _ptr(off), _ptr(idv), d, DTYPE_CODE[dtype], metric, _ptr(qv), _ptr(cl),
                           cl.shape[0], k, threads, _ptr(out_ids), _ptr(out_scores), C.byref(n_out)))
    return out_ids[:n_out.value], out_scores[:n_out.value]


def ivf_prefetch_amount(bandwidth, t_llm, nprobe, t_cc, budgets, miss_rates):
    """The prefetch budget of App. C for a measured miss-rate curve: (bytes, seconds of t_1 + t_2, case)."""
    bs = _host(budgets, np.float64).reshape(-1)
    rs = _host(miss_rates, np.float64).reshape(-1)
    assert bs.shape == rs.shape
    L = load()
    L.ivf_prefetch_amount.argtypes = [C.c_double, C.c_double, C.c_int32, C.c_double, C.c_void_p, C.c_void_p, C.c_int32,
                                      C.c_void_p, C.c_void_p, C.c_void_p]
    amount, seconds, which = C.c_double(0.0), C.c_double(0.0), C.c_int32(0)
    _check(L.ivf_prefetch_amount(float(bandwidth), float(t_llm), int(nprobe), float(t_cc), _ptr(bs), _ptr(rs), bs.shape[0],
                                 C.byref(amount), C.byref(seconds), C.byref(which)))
    return amount.value, seconds.value, which.value


def ivf_prefetch_plan(ranked, offsets, row_bytes, budget_bytes, buffer_bytes, resident_off, buffer_used):
    """The budget walk of ivf_prefetch over already ranked clusters (ranked: [nq, nprobe] int32).
    resident_off (int64[nlist], -1 = absent) is updated in place.  Returns (clusters to copy in
    order, PrefetchStats, buffer bytes in use afterwards)."""
    rk = _host(ranked, np.int32)
    rk = rk.reshape(1, -1) if rk.ndim == 1 else rk
    off = _host(offsets, np.int64)
    assert resident_off.dtype == np.int64 and resident_off.flags["C_CONTIGUOUS"]
    nlist = off.shape[0] - 1
    assert resident_off.shape[0] == nlist
    taken = np.empty(rk.size, dtype=np.int32)
    n_taken = C.c_int32(0)
    used = C.c_size_t(int(buffer_used))
    st = PrefetchStats()
    L = load()
    L.ivf_prefetch_plan.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_size_t, C.c_size_t,
                                    C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    _check(L.ivf_prefetch_plan(_ptr(rk), rk.shape[0], rk.shape[1], _ptr(off), nlist, int(row_bytes), int(budget_bytes),
                               int(buffer_bytes), _ptr(resident_off), C.byref(used), _ptr(taken), C.byref(n_taken),
                               C.byref(st)))
    return taken[:n_taken.value], st, used.value


class CacheMove(C.Structure):
    _fields_ = [("cluster", C.c_int32), ("via_staging", C.c_int32), ("from_byte", C.c_uint64),
                ("to_byte", C.c_uint64), ("bytes", C.c_uint64)]


def ivf_cache_plan(hotness, offsets, row_bytes, resident_off, buffer_used, buffer_bytes, fraction):
    """Eviction and consolidation plan of a cache round.  hotness (float32[nlist]) and resident_off
    (int64[nlist]) are updated in place.  Returns (evicted clusters in order, list of moves as
    (cluster, via_staging, from_byte, to_byte, bytes), buffer bytes in use afterwards)."""
    assert hotness.dtype == np.float32 and hotness.flags["C_CONTIGUOUS"]
    assert resident_off.dtype == np.int64 and resident_off.flags["C_CONTIGUOUS"]
    off = _host(offsets, np.int64)
    nlist = off.shape[0] - 1
    assert hotness.shape[0] == nlist and resident_off.shape[0] == nlist
    evicted = np.empty(nlist, dtype=np.int32)
    moves = (CacheMove * nlist)()
    n_ev, n_mv = C.c_int32(0), C.c_int32(0)
    used = C.c_size_t(int(buffer_used))
    L = load()
    L.ivf_cache_plan.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_size_t, C.c_void_p, C.c_void_p, C.c_size_t,
                                 C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    _check(L.ivf_cache_plan(_ptr(hotness), _ptr(off), nlist, int(row_bytes), _ptr(resident_off), C.byref(used),
                            int(buffer_bytes), float(fraction), _ptr(evicted), C.byref(n_ev), moves, C.byref(n_mv)))
    mv = [(m.cluster, m.via_staging, m.from_byte, m.to_byte, m.bytes) for m in moves[:n_mv.value]]
    return evicted[:n_ev.value], mv, used.value
