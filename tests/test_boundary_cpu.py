"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import numpy as np

import paper_2502_20969_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "ivf.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ivf_[a-z_]+)\s*\(", header))
    assert declared == set(P.EXPORTS), declared ^ set(P.EXPORTS)
    L = P.load()
    for name in declared:
        assert hasattr(L, name), name


def test_status_strings():
    L = P.load()
    assert L.ivf_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert L.ivf_strerror(code) not in (b"ok", b"unknown status")
    assert L.ivf_strerror(-99) == b"unknown status"


def test_bad_arguments_are_rejected_on_the_host():
    L = P.load()
    h = C.c_void_p()
    cent = np.zeros((2, 4), dtype=np.float32)
    rows = np.zeros((3, 4), dtype=np.float32)
    asg = np.zeros(3, dtype=np.int32)
    vp = lambda a: C.c_void_p(a.ctypes.data)
    # NULL centroids, bad dtype, bad metric, bad placement, d < 1, d too large
    assert L.ivf_build_layout(vp(rows), 3, 4, 0, None, 2, vp(asg), None, 0, 0, 0, None, None, C.byref(h)) == -1
    assert L.ivf_build_layout(vp(rows), 3, 4, 7, vp(cent), 2, vp(asg), None, 0, 0, 0, None, None, C.byref(h)) == -1
    assert L.ivf_build_layout(vp(rows), 3, 4, 0, vp(cent), 2, vp(asg), None, 5, 0, 0, None, None, C.byref(h)) == -1
    assert L.ivf_build_layout(vp(rows), 3, 4, 0, vp(cent), 2, vp(asg), None, 0, 9, 0, None, None, C.byref(h)) == -1
    assert L.ivf_build_layout(vp(rows), 3, 0, 0, vp(cent), 2, vp(asg), None, 0, 0, 0, None, None, C.byref(h)) == -1
    assert L.ivf_build_layout(vp(rows), 3, 5000, 0, vp(cent), 2, vp(asg), None, 0, 0, 0, None, None, C.byref(h)) == -5
    assert b"5000" in L.ivf_last_error()
    # assignment out of range is found before any device work
    bad = np.array([0, 2, 1], dtype=np.int32)
    assert L.ivf_build_layout(vp(rows), 3, 4, 0, vp(cent), 2, vp(bad), None, 0, 0, 0, None, None, C.byref(h)) == -1
    off = np.array([0, 2, 2], dtype=np.int64)     # does not end at n = 3
    assert L.ivf_adopt_layout(vp(rows), vp(off), None, 3, 4, 0, vp(cent), 2, 0, 0, 0, None, None, C.byref(h)) == -1
    # NULL index
    assert L.ivf_search(None, vp(rows), 1, 1, 1, vp(rows), vp(rows), None) == -1
    assert L.ivf_prefetch(None, vp(rows), 1, 1, 0, 0, None) == -1
    L.ivf_free(None)


def test_entry_point_build_calls_both_builders(monkeypatch):
    """__graft_entry__.build() must reach the HIP build and the oracle build (the oracle package also
    exports a function called build, which once shadowed the module of that name)."""
    import sys
    import __graft_entry__ as entry
    import oracle.build  # noqa: F401
    import paper_2502_20969_amd.build  # noqa: F401
    calls = []
    monkeypatch.setattr(sys.modules["paper_2502_20969_amd.build"], "build", lambda: calls.append("hip"))
    monkeypatch.setattr(sys.modules["oracle.build"], "build", lambda: calls.append("oracle"))
    entry.build()
    assert calls == ["hip", "oracle"]
