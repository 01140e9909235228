"""The entry point that allocates nothing (ivf_search_device_noalloc), called through the C-ABI:
its outputs equal those of ivf_search_device bit for bit, on two calls in a row, the second with a
smaller input; a search whose workspace does not fit the fixed scratch area is refused."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2502_20969_amd as P
from parity import check_topk, stored

pytestmark = pytest.mark.gpu


def _problem(seed, n, d, nlist, dtype):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((nlist, d)).astype(np.float32)
    assign = rng.integers(0, nlist, n).astype(np.int32)
    rows = centres[assign] + 0.5 * rng.standard_normal((n, d)).astype(np.float32)
    rows /= np.linalg.norm(rows, axis=1, keepdims=True)
    ids = rng.permutation(n).astype(np.int64) * 2 + 5
    st, odt = stored(rows, dtype)
    return st, odt, centres, assign, ids, rng


@pytest.mark.parametrize("dtype,metric", [("f32", "ip"), ("f16", "l2")])
def test_noalloc_equals_search_device_twice(dtype, metric):
    assert torch.cuda.is_available()
    pm, om = (P.IVF_IP, O.IP) if metric == "ip" else (P.IVF_L2, O.L2)
    n, d, nlist = 60000, 256, 96
    st, odt, cent, assign, ids, rng = _problem(77, n, d, nlist, dtype)
    stream = torch.cuda.Stream()
    index = P.ivf_build_layout(st, dtype, cent, assign, ids=ids, metric=pm,
                               compute_stream=stream, copy_stream=torch.cuda.Stream())
    off, perm = O.build_layout(assign, nlist)
    lists, lid = st[perm], ids[perm]
    q_all = (cent[rng.integers(0, nlist, 7)] + 0.5 * rng.standard_normal((7, d))).astype(np.float32)
    q_all /= np.linalg.norm(q_all, axis=1, keepdims=True)
    # first call: 7 queries, nprobe 24, k 20; second call: smaller in every size
    for nq, nprobe, k in ((7, 24, 20), (3, 5, 4)):
        q = torch.from_numpy(q_all[:nq]).cuda()
        ref_i = torch.full((nq, k), -9, dtype=torch.int64, device="cuda")
        ref_d = torch.zeros(nq, k, dtype=torch.float32, device="cuda")
        index.ivf_set_batch_mode(1)
        index.ivf_search_device(q, nprobe, k, ref_i, ref_d)
        index.ivf_synchronize()
        got_i = torch.full((nq, k), -9, dtype=torch.int64, device="cuda")
        got_d = torch.zeros(nq, k, dtype=torch.float32, device="cuda")
        index.ivf_search_device_noalloc(q, nprobe, k, got_i, got_d)
        torch.cuda.synchronize()
        assert torch.equal(got_i, ref_i)
        assert torch.equal(got_d.view(torch.int32), ref_d.view(torch.int32))
        gi, gd = got_i.cpu().numpy(), got_d.cpu().numpy()
        for b in range(nq):
            assert check_topk(gi[b], gd[b], lists, odt, off, lid, cent, q_all[b], nprobe, k, om) == 0
    index.close()


def test_noalloc_refuses_what_does_not_fit():
    n, d, nlist = 20000, 64, 64
    st, odt, cent, assign, ids, rng = _problem(78, n, d, nlist, "f32")
    index = P.ivf_build_layout(st, "f32", cent, assign, metric=P.IVF_IP,
                               compute_stream=torch.cuda.Stream(), copy_stream=torch.cuda.Stream())
    nq, k = 4096, 100                    # 4096 queries x 4 wavefront lists x 128 candidates x 8 bytes = 16 MiB
    q = torch.zeros(nq, d, device="cuda")
    ids_dev = torch.empty(nq, k, dtype=torch.int64, device="cuda")
    dists_dev = torch.empty(nq, k, dtype=torch.float32, device="cuda")
    with pytest.raises(P.IvfError) as e:
        index.ivf_search_device_noalloc(q, 64, k, ids_dev, dists_dev)
    assert e.value.status == -5 and "scratch" in str(e.value)
    # a host-placed index is refused too
    index.close()
