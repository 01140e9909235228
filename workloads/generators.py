"""Input generators (see package docstring).  Inputs only; no search arithmetic."""
from dataclasses import dataclass
from typing import Optional

import torch

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _normalize(x: torch.Tensor) -> torch.Tensor:
    return x / x.norm(dim=-1, keepdim=True).clamp_min(1e-30)


@dataclass
class Datastore:
    """A synthetic vector datastore.

    rows       [n, d] in `dtype`; input order when `assign` is set, cluster-major
               (list c = rows offsets[c]:offsets[c+1]) when `offsets` is set
    centroids  [nlist, d] float32
    """
    rows: torch.Tensor
    centroids: torch.Tensor
    dtype: str
    assign: Optional[torch.Tensor] = None
    offsets: Optional[torch.Tensor] = None
    centres: Optional[torch.Tensor] = None      # mixture centres the rows were drawn around
    component: Optional[torch.Tensor] = None    # mixture component of each row (kmeans route)

    @property
    def n(self):
        return self.rows.shape[0]

    @property
    def d(self):
        return self.rows.shape[1]

    @property
    def nlist(self):
        return self.centroids.shape[0]


def mixture_rows(n, d, n_comp, sigma, seed, device="cpu", chunk=1 << 18):
    """n unit-norm rows: normalize(centre_c + sigma * N(0, I)), c uniform over n_comp
    centres drawn from N(0, I).  Returns (rows fp32, component int64, centres fp32)."""
    g = _gen(seed, device)
    centres = torch.randn(n_comp, d, generator=g, device=device)
    comp = torch.randint(0, n_comp, (n,), generator=g, device=device)
    rows = torch.empty(n, d, device=device)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        noise = torch.randn(e - s, d, generator=g, device=device)
        rows[s:e] = _normalize(centres[comp[s:e]] + sigma * noise)
    return rows, comp, centres


def _nearest(rows, centroids, chunk=1 << 16):
    """Index of the L2-nearest centroid of each row (input preparation only)."""
    out = torch.empty(rows.shape[0], dtype=torch.int64, device=rows.device)
    c2 = (centroids * centroids).sum(1)
    for s in range(0, rows.shape[0], chunk):
        r = rows[s:s + chunk].float()
        dist = c2[None, :] - 2.0 * (r @ centroids.T)
        out[s:s + chunk] = dist.argmin(1)
    return out


def kmeans_datastore(n, d, n_comp, sigma, nlist, iters, seed, sample=None, dtype="f32",
                     device="cpu"):
    """Mixture rows, centroids from `iters` Lloyd iterations (on a seeded sample of
    `sample` rows when given; initial centroids = nlist seeded random sample rows),
    and each row's nearest-centroid assignment."""
    rows, comp, centres = mixture_rows(n, d, n_comp, sigma, seed, device)
    g = _gen(seed + 1, device)
    if sample is not None and sample < n:
        pick = torch.randperm(n, generator=g, device=device)[:sample]
        train = rows[pick]
    else:
        train = rows
    init = torch.randperm(train.shape[0], generator=g, device=device)[:nlist]
    cent = train[init].clone()
    for _ in range(iters):
        a = _nearest(train, cent)
        sums = torch.zeros_like(cent).index_add_(0, a, train)
        cnt = torch.zeros(nlist, device=device).index_add_(0, a, torch.ones_like(a, dtype=torch.float32))
        keep = cnt > 0
        cent[keep] = sums[keep] / cnt[keep, None]
    assign = _nearest(rows, cent).to(torch.int32)
    rows = rows.to(TORCH_DTYPE[dtype])
    return Datastore(rows=rows, centroids=cent.contiguous(), dtype=dtype, assign=assign,
                     centres=centres, component=comp)


def zipf_sizes(n, nlist, exponent, seed, min_rows=1):
    """nlist list sizes summing to n with size of rank r proportional to r^-exponent,
    rank order randomly permuted over the clusters.  exponent 0 gives near-uniform sizes."""
    g = _gen(seed, "cpu")
    w = torch.arange(1, nlist + 1, dtype=torch.float64) ** (-float(exponent))
    sizes = torch.floor(w / w.sum() * (n - min_rows * nlist)).to(torch.int64) + min_rows
    sizes[0] += n - int(sizes.sum())
    return sizes[torch.randperm(nlist, generator=g)]


def cluster_major_datastore(sizes, d, sigma, seed, dtype="f16", device="cpu", out=None,
                            chunk=1 << 18):
    """Rows generated directly in cluster-major order: list c has sizes[c] rows
    normalize(centre_c + sigma * N(0, I)), rounded to `dtype`; the centroid of list c is
    the mean of its stored rows (zero for an empty list).  `out` may be a preallocated
    (for example pinned-host) [n, d] tensor that receives the rows chunk by chunk."""
    sizes = sizes.to(torch.int64).cpu()
    nlist = sizes.shape[0]
    n = int(sizes.sum())
    offsets = torch.zeros(nlist + 1, dtype=torch.int64)
    offsets[1:] = torch.cumsum(sizes, 0)
    g = _gen(seed, device)
    centres = torch.randn(nlist, d, generator=g, device=device)
    tdt = TORCH_DTYPE[dtype]
    rows = out if out is not None else torch.empty(n, d, dtype=tdt, device=device)
    assert rows.shape == (n, d) and rows.dtype == tdt
    sums = torch.zeros(nlist, d, dtype=torch.float32, device=device)
    off_dev = offsets.to(device)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        pos = torch.arange(s, e, device=device)
        cl = torch.searchsorted(off_dev, pos, right=True) - 1
        noise = torch.randn(e - s, d, generator=g, device=device)
        block = _normalize(centres[cl] + sigma * noise).to(tdt)
        sums.index_add_(0, cl, block.float())
        rows[s:e].copy_(block)
    cent = sums / sizes.to(device).clamp_min(1).float()[:, None]
    return Datastore(rows=rows, centroids=cent.contiguous(), dtype=dtype, offsets=offsets,
                     centres=centres)


def query_pairs(anchor_rows, nq, alpha, seed, anchor_noise=0.1):
    """(q_in, q_out), both [nq, d] float32 unit vectors on the anchors' device.

    q_in  = normalize(anchor + anchor_noise * g),  anchor = a seeded random row,
    q_out = normalize(q_in + alpha * g'),          g, g' ~ N(0, I/d)  (unit expected norm).
    """
    device = anchor_rows.device
    d = anchor_rows.shape[1]
    g = _gen(seed, device)
    pick = torch.randint(0, anchor_rows.shape[0], (nq,), generator=g, device=device)
    base = anchor_rows[pick].float()
    scale = d ** -0.5
    q_in = _normalize(base + anchor_noise * scale * torch.randn(nq, d, generator=g, device=device))
    q_out = _normalize(q_in + alpha * scale * torch.randn(nq, d, generator=g, device=device))
    return q_in.contiguous(), q_out.contiguous()


def perturbed(q, alpha, seed):
    """normalize(q + alpha * g), g ~ N(0, I/d): the rewritten form of each query in q [nq, d]."""
    g = _gen(seed, q.device)
    d = q.shape[1]
    return _normalize(q + alpha * (d ** -0.5) * torch.randn(q.shape, generator=g, device=q.device)).contiguous()


# ---- the named workloads ------------------------------------------------------

def config1_tiny(seed=20969, device="cpu", dtype="f32"):
    """20,000 x 128 rows from a 64-component mixture (sigma 0.3), nlist 64 from 10 Lloyd
    iterations, 16 query pairs with alpha 0.2.  Searched with inner product, nprobe 8, k 10."""
    ds = kmeans_datastore(20000, 128, 64, 0.3, 64, 10, seed, dtype=dtype, device=device)
    q_in, q_out = query_pairs(ds.rows, 16, 0.2, seed + 2)
    return ds, q_in, q_out


def config2_single_query(seed=20970, device="cpu", n=1_000_000, d=768, nlist=1024, nq=256,
                         dtype="f32"):
    """1,000,000 x 768 fp32 rows from a 1024-component mixture, nlist 1024 from k-means on a
    100k sample, nq query pairs with alpha 0.3.  Searched with nprobe 32, k 10, batch 1.
    `n`, `d`, `nlist` can be scaled down for tests; the sample stays one tenth of n."""
    ds = kmeans_datastore(n, d, nlist, 0.3, nlist, 10, seed, sample=max(nlist, n // 10),
                          dtype=dtype, device=device)
    q_in, q_out = query_pairs(ds.rows, nq, 0.3, seed + 2)
    return ds, q_in, q_out


def shared_batch_queries(ds, nq, n_groups, seed, noise=0.5):
    """nq unit-norm float32 queries drawn around `n_groups` of the datastore's mixture centres, so
    that the queries of one group probe largely the same clusters (a batch that shares lists).
    n_groups = nq gives queries from distinct components."""
    device = ds.centres.device
    g = _gen(seed, device)
    d = ds.centres.shape[1]
    pick = torch.randperm(ds.centres.shape[0], generator=g, device=device)[:n_groups]
    which = torch.arange(nq, device=device) % n_groups
    base = _normalize(ds.centres[pick][which])
    q = _normalize(base + noise * (d ** -0.5) * torch.randn(nq, d, generator=g, device=device))
    return q.contiguous()


def config3_mid_fp16(device="cuda", scale=1.0, groups=24, n_sets=8, batch=32, d=768):
    """configs[2]: 10,000,000 x 768 fp16 rows generated cluster-major, nlist 4096 with Zipf(1.1)
    sizes; batches of 32 queries drawn around `groups` mixture centres (24: measured sharing of the
    probed clusters 0.40 at nprobe 128).  Searched with inner product, nprobe 128, k 10.
    Returns (datastore, list of n_sets query batches)."""
    n = int(10_000_000 * scale)
    sizes = zipf_sizes(n, 4096, 1.1, 20975)
    ds = cluster_major_datastore(sizes, d, 0.3, 20976, dtype="f16", device=device, chunk=1 << 20)
    return ds, [shared_batch_queries(ds, batch, groups, 20980 + i) for i in range(n_sets)]


def config5_large_bf16(device="cuda", scale=1.0, n_sets=8, batch=256, d=1024, groups=None):
    """configs[4]: 30,000,000 x 1024 bf16 rows generated cluster-major, nlist 8192 with Zipf(1.2)
    sizes; batches of 256 queries from 256 distinct mixture components.  Searched with inner
    product, nprobe 512, k 100.  Returns (datastore, list of n_sets query batches)."""
    n = int(30_000_000 * scale)
    sizes = zipf_sizes(n, 8192, 1.2, 20977)
    ds = cluster_major_datastore(sizes, d, 0.3, 20978, dtype="bf16", device=device, chunk=1 << 20)
    return ds, [shared_batch_queries(ds, batch, groups or batch, 20980 + i) for i in range(n_sets)]


def config4_lookahead(pinned_out, nlist, pairs, device="cuda"):
    """configs[3]: fp16 rows generated on `device` chunk by chunk into `pinned_out` (a pinned host
    tensor [n, 768]; 60,000,000 rows at full size), nlist near-uniform lists (16384 at full size),
    `pairs` query pairs with alpha 0.3.  Searched with inner product, nprobe 256 at full size, k 10.
    Returns (datastore, q_in, q_out); the queries are host tensors."""
    n, d = pinned_out.shape
    sizes = zipf_sizes(n, nlist, 0.1, 20972)
    ds = cluster_major_datastore(sizes, d, 0.3, 20973, dtype="f16", device=device, out=pinned_out, chunk=1 << 20)
    q_in, q_out = query_pairs(pinned_out, pairs, 0.3, 20974)
    return ds, q_in, q_out


def paper_shape_fp32(device="cuda", scale=1.0, nq=64):
    """The shape the paper evaluates on (Sec. 5 set-up): 21,000,000 x 768 fp32 rows, 4096 clusters,
    here generated cluster-major with Zipf(1.1) sizes; nq queries = perturbed stored rows.
    Searched with nprobe 64 .. 1024, k 3, batches of 1 to 8.  Returns (datastore, q_out)."""
    n = int(21_000_000 * scale)
    sizes = zipf_sizes(n, 4096, 1.1, 20985)
    ds = cluster_major_datastore(sizes, 768, 0.3, 20986, dtype="f32", device=device, chunk=1 << 20)
    pick = torch.randint(0, n, (4096,), generator=torch.Generator().manual_seed(20987)).to(device)
    _, q_out = query_pairs(ds.rows[pick], nq, 0.3, 20988)
    return ds, q_out


def pinned_rows(n_full, d, dtype, scales=(1.0, 0.6875, 0.5, 0.25, 0.125, 0.0625)):
    """A pinned host tensor [n, d] for a host-placed datastore of n_full rows; when the host
    refuses to pin that much, the next smaller scale is tried.  Returns (tensor, scale, note) with
    n = n_full * scale and note = the refusal message of the first failed attempt."""
    note = None
    for scale in scales:
        n = int(n_full * scale)
        try:
            return torch.empty((n, d), dtype=TORCH_DTYPE[dtype], pin_memory=True), scale, note
        except RuntimeError as e:
            if note is None:
                note = str(e).splitlines()[0]
    raise RuntimeError(f"could not pin even {scales[-1]} of {n_full} x {d} {dtype}: {note}")


def release_pinned_cache():
    """Gives freed pinned host blocks back to the system (torch keeps them cached otherwise, and the
    amount of pinned memory a process may hold is limited)."""
    fn = getattr(torch._C, "_host_emptyCache", None)
    if fn is not None:
        fn()
