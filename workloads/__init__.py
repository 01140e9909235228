"""Seeded synthetic inputs shaped like the paper's datastores.

This package makes INPUTS only: mixture-of-Gaussians embeddings, a k-means
used to obtain centroids and an assignment for those inputs, Zipf list sizes,
and q_in / q_out query pairs.  It holds none of the search method's arithmetic
(no probing, no list scan, no top-k, no prefetch planning) and is the only code
shared by the CPU oracle's tests and the HIP path's tests.

All tensors come from torch generators seeded from one integer, on the CPU or
on a GPU (`device=`).  The same call with the same seed and device gives the
same values.
"""
from .generators import (  # noqa: F401
    Datastore,
    cluster_major_datastore,
    kmeans_datastore,
    mixture_rows,
    perturbed,
    query_pairs,
    shared_batch_queries,
    zipf_sizes,
    config1_tiny,
    config2_single_query,
    config3_mid_fp16,
    config4_lookahead,
    config5_large_bf16,
    paper_shape_fp32,
    pinned_rows,
    release_pinned_cache,
)
