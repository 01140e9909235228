"""Full-size parity: the single-query workload at its real size (1,000,000 x 768 fp32, nlist 1024),
in the launch configuration bench.py times (ivf_search_device, several searches in flight),
checked on sampled queries the oracle computes one by one, plus the exhaustive-search identity."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2502_20969_amd as P
import workloads as W
from parity import check_topk

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c2():
    assert torch.cuda.is_available()
    ds, q_in, q_out = W.config2_single_query(device="cuda")
    rows = ds.rows.cpu().numpy()
    assign = ds.assign.cpu().numpy()
    cent = ds.centroids.cpu().numpy()
    index = P.ivf_build_layout(rows, "f32", cent, assign, metric=P.IVF_IP,
                               compute_stream=torch.cuda.Stream(), copy_stream=torch.cuda.Stream())
    off, perm = O.build_layout(assign, 1024)
    goff, gids = index.ivf_get_layout()
    assert np.array_equal(goff, off) and np.array_equal(gids, perm)
    lists = rows[perm]
    del rows
    yield index, lists, off, perm, cent, q_in, q_out
    index.close()


def test_bench_configuration_matches_oracle(c2):
    index, lists, off, perm, cent, q_in, q_out = c2
    nq = q_out.shape[0]
    ids = torch.full((nq, 10), -7, dtype=torch.int64, device="cuda")
    dists = torch.zeros(nq, 10, dtype=torch.float32, device="cuda")
    index.ivf_set_pipeline_depth(4)
    index.ivf_reserve(1, 1024, 10)
    torch.cuda.synchronize()
    for rep in range(2):
        for j in range(nq):
            index.ivf_search_device(q_out[j], 32, 10, ids[j], dists[j])
    index.ivf_synchronize()
    gi, gd = ids.cpu().numpy(), dists.cpu().numpy()
    q = q_out.cpu().numpy()
    exempt = 0
    for j in range(0, nq, 16):          # 16 sampled queries
        exempt += check_topk(gi[j], gd[j], lists, O.F32, off, perm, cent, q[j], 32, 10, O.IP)
    assert exempt == 0
    # properties that hold for every query at any size
    assert np.all(gi >= 0) and np.all(np.diff(gd, axis=1) <= 0)
    assert all(len(set(r)) == 10 for r in gi)
    index.ivf_set_pipeline_depth(1)
    # the measured q_in / q_out cluster overlap of this workload (reported, and sanity-bounded)
    pin = index.ivf_probe(q_in.cpu().numpy()[:64], 32)
    pout = index.ivf_probe(q[:64], 32)
    overlap = np.mean([len(set(a) & set(b)) / 32 for a, b in zip(pin, pout)])
    print(f"mean |C_in & C_out| / |C_out| at nprobe 32: {overlap:.3f}")
    assert 0.2 < overlap <= 1.0


def test_every_nprobe_of_the_sweep(c2):
    index, lists, off, perm, cent, q_in, q_out = c2
    q = q_out.cpu().numpy()[:2]
    for nprobe in (1, 4, 64, 256, 1024):
        gi, gd = index.ivf_search(q, nprobe, 10)
        for b in range(2):
            assert check_topk(gi[b], gd[b], lists, O.F32, off, perm, cent, q[b], nprobe, 10, O.IP) == 0
    # nprobe = nlist is exhaustive search: compare with a library matmul + argsort
    gi, gd = index.ivf_search(q, 1024, 10)
    sc = lists.astype(np.float64) @ q.astype(np.float64).T
    for b in range(2):
        want = perm[np.lexsort((perm, -sc[:, b]))[:10]]
        assert list(gi[b]) == list(want)
