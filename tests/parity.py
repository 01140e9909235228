"""Comparison rules shared by the GPU parity tests (bar set by the benchmark spec):
ids bit-exact except on near-ties whose relative score gap is below 1e-6, distances within
1e-4 relative (fp32 rows) or 2e-3 (fp16 / bf16 rows)."""
import numpy as np

import oracle as O

NEAR_TIE = 1e-6
RTOL = {O.F32: 1e-4, O.F16: 2e-3, O.BF16: 2e-3}


def stored(rows_f32, dtype):
    """(array as stored for both sides, oracle dtype code) from float32 rows."""
    import torch
    if dtype == "f32":
        return np.ascontiguousarray(rows_f32, dtype=np.float32), O.F32
    if dtype == "f16":
        return rows_f32.astype(np.float16), O.F16
    t = torch.from_numpy(np.ascontiguousarray(rows_f32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16), O.BF16


def compare_topk(gpu_ids, gpu_dists, oi, osc, k, odt, metric):
    """Compares one query's GPU result (k entries) with the oracle's first k + extra results
    (oi, osc).  Returns the number of near-tie exemptions used."""
    score_of = {int(i): s for i, s in zip(oi, osc) if i >= 0}
    exempt = 0
    for pos in range(k):
        want, got = int(oi[pos]), int(gpu_ids[pos])
        if want == -1:
            assert got == -1, f"pos {pos}: expected padding, got id {got}"
            assert np.isinf(gpu_dists[pos]) and (gpu_dists[pos] < 0) == (metric == O.IP)
            continue
        if got != want:
            assert got in score_of, f"pos {pos}: id {got} is not among the oracle's top {len(oi)}"
            a, b = score_of[got], osc[pos]
            assert abs(a - b) <= NEAR_TIE * max(abs(a), abs(b)), \
                f"pos {pos}: id {got} (score {a}) vs oracle id {want} (score {b}) is not a near-tie"
            exempt += 1
        ref = score_of[got]
        assert abs(gpu_dists[pos] - ref) <= RTOL[odt] * max(abs(ref), 1e-30) + 1e-30, \
            f"pos {pos}: distance {gpu_dists[pos]} vs oracle {ref}"
    return exempt


def check_topk(gpu_ids, gpu_dists, lists, odt, off, ids, cent, x, nprobe, k, metric, extra=8):
    """Compares one query's GPU result with the oracle.  Returns the number of near-tie
    exemptions used.  The oracle is asked for k + extra results so that a GPU id that is not in
    its top k can be looked up."""
    oi, osc = O.search(lists, odt, off, ids, cent, x, nprobe, k + extra, metric)
    return compare_topk(gpu_ids, gpu_dists, oi, osc, k, odt, metric)


def oracle_search_selected(rows_t, odt, off, cent, x, nprobe, k, metric, extra=8):
    """Oracle search of one query over a datastore too large to copy to the host whole: the
    oracle selects its clusters from the centroids, exactly those lists are copied from `rows_t`
    (a torch tensor [n, d], on the GPU or on the host, cluster-major with offsets `off`) into a
    host datastore in which every other list is empty and rows keep their global row number as id,
    and the oracle then searches that datastore (it selects the same clusters again).
    Returns (ids, scores) of the k + extra nearest and the selected clusters."""
    import torch
    nlist = cent.shape[0]
    sel = O.probe(cent, x, nprobe, metric)
    cnt = np.zeros(nlist, dtype=np.int64)
    cnt[sel] = off[sel + 1] - off[sel]
    coff = np.zeros(nlist + 1, dtype=np.int64)
    coff[1:] = np.cumsum(cnt)
    order = np.sort(sel)
    parts = [rows_t[int(off[c]):int(off[c + 1])] for c in order]
    block = torch.cat(parts).cpu() if parts else rows_t[:0].cpu()
    if block.dtype == torch.bfloat16:
        block = block.view(torch.int16)
    rows = block.numpy()
    if rows.dtype == np.int16:
        rows = rows.view(np.uint16)
    gids = np.concatenate([np.arange(off[c], off[c + 1], dtype=np.int64) for c in order]) if parts else np.zeros(0, np.int64)
    assert rows.shape[0] == coff[-1] == gids.shape[0]
    oi, osc = O.search(rows, odt, coff, gids, cent, x, nprobe, k + extra, metric)
    return oi, osc, sel
