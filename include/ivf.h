/*
 * libivf -- IVF-Flat nearest-neighbour search with lookahead prefetch for one
 * MI355X (gfx950).  C ABI: plain pointers and sizes, no C++ or torch types.
 *
 * The operations are those of TeleRAG (arxiv 2502.20969):
 *   - IVF search (App. B): coarse scoring of the query against all centroids,
 *     selection of the nprobe nearest clusters, a scan of the rows of those
 *     clusters, and the k nearest rows.
 *   - Lookahead retrieval (Sec. 4.1 steps 1-4, Sec. 4.3 "Prefetching target"):
 *     clusters ranked by q_in are copied host->device under a byte budget while
 *     other work runs; q_out is then searched over the resident clusters
 *     (C_overlap) on the GPU and over the others (C_miss) on the host, and the
 *     two partial results are merged.
 *
 * Conventions
 *   - Every function returns 0 (IVF_OK) or a negative ivf_status; nothing
 *     throws or aborts across this boundary.  ivf_strerror() names a status;
 *     ivf_last_error() gives a longer message for the calling thread.
 *   - "host" pointers are ordinary process memory unless "pinned" is said;
 *     "device" pointers are HIP device memory on the current device.
 *   - An index is used by one host thread at a time.  The library never frees
 *     or keeps caller memory unless a function says the index adopts it.
 *   - Metric (App. B, the distance d): IVF_IP ranks by inner product, larger is
 *     nearer, reported distances are the raw inner products (descending).
 *     IVF_L2 ranks by squared Euclidean distance, smaller is nearer, reported
 *     distances are the squared distances (ascending).  The coarse and the fine
 *     stage use the same metric.
 *   - Order: equal scores are ordered by smaller cluster index (coarse stage)
 *     or smaller vector id (fine stage), so results are deterministic.
 *   - nprobe larger than nlist is clamped to nlist.  When fewer than k rows
 *     were scanned the tail is padded with id -1 and distance -INF (IP) or
 *     +INF (L2).
 *   - Arithmetic: coarse scores are accumulated in fp64.  The list scan
 *     accumulates in fp32 over rows stored as fp32 / fp16 / bf16 with the fp32
 *     query; the k' = k + max(8, k / 8) best rows are then re-scored in fp64 and
 *     ordered by that score, and the fp64 value rounded to fp32 is what is
 *     returned.  The k nearest are exact with respect to the fp64 scores: when
 *     the k-th fp64 score found is not above the last fp32 score kept by more
 *     than a bound of the scan's rounding, a row that was dropped could belong
 *     to the result, and the query gets an exact second pass (every selected
 *     row scored in fp64) on the device, and likewise on the host for the host
 *     part of a hybrid search.
 */
#ifndef IVF_H
#define IVF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ivf_index ivf_index; /* opaque */

enum ivf_status {
    IVF_OK = 0,
    IVF_EINVAL = -1, /* bad argument: NULL, size < 1, unknown enum, assignment out of range */
    IVF_ENOMEM = -2, /* host or device allocation failed; the index is unchanged */
    IVF_EHIP = -3,   /* a HIP call failed; ivf_last_error() holds its text */
    IVF_ESTATE = -4, /* call not valid for this index (e.g. prefetch on a device-resident index) */
    IVF_ELIMIT = -5  /* a size is above what this build supports (k, d, n) */
};

enum ivf_metric { IVF_IP = 0, IVF_L2 = 1 };
enum ivf_dtype { IVF_F32 = 0, IVF_F16 = 1, IVF_BF16 = 2 }; /* storage type of list rows */
enum ivf_placement {
    IVF_PLACE_DEVICE = 0, /* every list resident in HBM */
    IVF_PLACE_HOST = 1    /* lists in pinned host memory + a device prefetch buffer
                             (Sec. "Implementation Details": pinned region, fixed GPU buffer) */
};

#define IVF_PREFETCH_RESET 1u /* drop all residency before planning (each request starts cold) */

#define IVF_MAX_K 112 /* largest k of ivf_search / ivf_search_device */

typedef struct ivf_prefetch_stats {
    int32_t n_ranked;   /* clusters considered (sum over queries of min(nprobe, nlist)) */
    int32_t n_taken;    /* clusters whose copy was enqueued by this call */
    int32_t n_skipped;  /* clusters that did not fit the remaining budget or buffer */
    int32_t n_resident; /* clusters considered that were already resident */
    uint64_t bytes;     /* payload bytes enqueued by this call */
    uint64_t buffer_used; /* bytes of the device buffer in use after this call */
} ivf_prefetch_stats;

typedef struct ivf_search_stats {
    int32_t n_probed;      /* sum over queries of clusters selected */
    int32_t n_overlap;     /* of those, scanned on the GPU */
    int32_t n_miss;        /* of those, scanned on the host */
    float hit_rate;        /* mean over queries of |C_overlap| / |C_out| (Table 1 caption) */
    uint64_t bytes_gpu;    /* list bytes the GPU scan covered: sum n_c*d*elem over C_overlap */
    uint64_t bytes_host;   /* list bytes the host scan covered */
    float ms_total;        /* wall time of the call */
    float ms_probe;        /* until the selected clusters were known to the host (host placement) */
    float ms_host_scan;    /* host scan of C_miss */
    int32_t n_exact_gpu;   /* queries whose GPU part needed the exact second pass (see "Arithmetic" above) */
    int32_t n_exact_host;  /* queries whose host part needed it */
} ivf_search_stats;

typedef struct ivf_profile {
    uint64_t calls;        /* searches measured since ivf_profile_reset() */
    double ms_coarse;      /* summed HIP-event time of the coarse-scoring kernel */
    double ms_select;      /* ... of the top-nprobe selection kernel */
    double ms_scan;        /* ... of the list-scan kernel */
    double ms_merge;       /* ... of the merge / re-score kernel */
    uint64_t scan_bytes;   /* summed list bytes the scan kernels covered */
    uint64_t scan_rows;    /* summed rows the scan kernels covered */
} ivf_profile;

/*
 * Builds cluster-major lists from rows in input order (one-time; the a0 step:
 * the contiguous cluster-major region of Sec. "Implementation Details").
 *   vectors    host, n x d row-major in `dtype`
 *   centroids  host, nlist x d float32, copied to the device
 *   assign     host, n entries in [0, nlist): the list of each row
 *   ids        host, n entries >= 0, or NULL for ids 0..n-1
 *   device_buffer_bytes  size of the prefetch buffer (IVF_PLACE_HOST only)
 *   compute_stream, copy_stream  hipStream_t values, or NULL for streams the
 *              library creates; kernels run on the first, prefetch copies on
 *              the second; both must be of default priority
 * Rows keep their input order inside a list.  The library owns all storage it
 * creates (device lists, or a pinned host region for IVF_PLACE_HOST).
 */
int ivf_build_layout(const void* vectors, int64_t n, int32_t d, int dtype,
                     const float* centroids, int32_t nlist, const int32_t* assign,
                     const int64_t* ids, int metric, int placement,
                     size_t device_buffer_bytes, void* compute_stream, void* copy_stream,
                     ivf_index** out);

/*
 * Adopts rows that are already cluster-major, without copying them.
 *   lists      IVF_PLACE_DEVICE: device pointer; IVF_PLACE_HOST: pinned host pointer
 *              (allocated with hipHostMalloc, e.g. a torch pinned tensor).  Owned by the
 *              caller and must outlive the index.
 *   offsets    host, nlist + 1 entries: list c = rows offsets[c] .. offsets[c+1]
 *   ids        host, n entries >= 0, or NULL for ids = row position
 */
int ivf_adopt_layout(void* lists, const int64_t* offsets, const int64_t* ids, int64_t n,
                     int32_t d, int dtype, const float* centroids, int32_t nlist, int metric,
                     int placement, size_t device_buffer_bytes, void* compute_stream,
                     void* copy_stream, ivf_index** out);

void ivf_free(ivf_index* index);

/*
 * Lookahead step 1 (Sec. 4.1 "Predict & prefetch", Sec. 4.3 "Prefetching target").
 * For each of the nq queries q_in (host, nq x d float32): ranks all clusters, walks the
 * nprobe nearest in order and enqueues on copy_stream the copy of every cluster that is
 * not resident and fits both the remaining budget (budget_bytes / nq per query) and the
 * remaining device buffer; a cluster that does not fit is skipped whole and the walk goes
 * on.  A cluster's size is n_c * d * element size.  Returns once the copies are enqueued;
 * the next ivf_search waits for them on the device.  IVF_PLACE_HOST only.
 */
int ivf_prefetch(ivf_index* index, const float* q_in, int32_t nq, int32_t nprobe,
                 size_t budget_bytes, uint32_t flags, ivf_prefetch_stats* stats /* or NULL */);

/* Blocks the host until all enqueued prefetch copies have finished; *ms (or NULL) receives
 * the HIP-event time from the first to the last copy of the most recent ivf_prefetch. */
int ivf_prefetch_wait(ivf_index* index, float* ms);

/*
 * IVF search (App. B; with host placement: Sec. 4.1 steps 2-4).
 *   q_out  host, nq x d float32      ids    host, nq x k, nearest first
 *   dists  host, nq x k float32
 * On return the outputs are complete (for nq = 1 the call returns as soon as the last kernel
 * has published them; work enqueued later on compute_stream is ordered behind that kernel).
 * With IVF_PLACE_HOST the clusters selected for
 * q_out that are resident are scanned on the GPU while the others are scanned by host
 * threads; the result equals a search with every list resident.
 */
int ivf_search(ivf_index* index, const float* q_out, int32_t nq, int32_t nprobe, int32_t k,
               int64_t* ids, float* dists, ivf_search_stats* stats /* or NULL */);

/*
 * The same search with device-resident queries and outputs (all device pointers), enqueued
 * on compute_stream without waiting: outputs are complete once that stream has reached
 * this point (with a pipeline depth above 1: see ivf_set_pipeline_depth; searched list-major:
 * see ivf_set_batch_mode, after ivf_synchronize()).  q_dev must be 16-byte aligned; q_dev, ids_dev
 * and dists_dev must stay valid until the outputs are complete.  IVF_PLACE_DEVICE only.  nq, nprobe and k must not exceed what
 * ivf_reserve() or an earlier search has sized the workspace for, else the call sizes it
 * itself, which synchronises the device.
 */
int ivf_search_device(ivf_index* index, const float* q_dev, int32_t nq, int32_t nprobe,
                      int32_t k, int64_t* ids_dev, float* dists_dev);

/* Sizes the workspace for searches up to (nq, nprobe, k) so that later calls allocate nothing. */
int ivf_reserve(ivf_index* index, int32_t nq, int32_t nprobe, int32_t k);

/*
 * ivf_search_device for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same results as a
 * query-by-query ivf_search_device, enqueued on compute_stream, but the workspace (coarse scores,
 * selected clusters and their tables, the scan wavefronts' candidate lists, the flags and lists of
 * the exact second pass) lives in one fixed
 * device array of IVF_NOALLOC_SCRATCH_BYTES that the library holds on every GPU it runs on until
 * the process ends.  The call allocates and frees nothing, on the host side of HIP or on the device.
 *   - A search whose workspace does not fit (roughly nq x (8 nlist + 32 nprobe) + 2100 x grid x nq
 *     bytes for k <= 56, twice the second term above that, grid <= 2 x compute units per query and
 *     fewer per query when nq is large: one query of a 1024-list index needs 1.1 MB) is refused with
 *     IVF_ELIMIT and nothing is enqueued.
 *   - Always query by query (the batch mode and the pipeline depth are ignored).  IVF_PLACE_DEVICE only.
 *   - Every call on a GPU shares that GPU's array, also across indexes: calls whose kernels could
 *     overlap on one GPU (other streams, other threads) race.  Calls on one compute_stream are
 *     ordered by the stream.  IVF_ESTATE while a list-major ivf_search_device batch is unfinished.
 */
#define IVF_NOALLOC_SCRATCH_BYTES (8u << 20)
int ivf_search_device_noalloc(ivf_index* index, const float* q_dev, int32_t nq, int32_t nprobe,
                              int32_t k, int64_t* ids_dev, float* dists_dev);

/*
 * Overlap of independent searches (batch-1 serving: one query's coarse scoring, selection and
 * merge run on a few compute units while another query's scan streams its lists).  With depth
 * n > 1, successive ivf_search_device calls rotate over n internal streams (the first is
 * compute_stream), each with its own workspace; inputs must be complete when the call is made,
 * and outputs are complete after ivf_synchronize() (which also runs the exact second pass for
 * the queries that need it; with depth 1 that pass follows every search on the stream).  List-major batches overlap in the same way
 * (the kernels that prepare one batch run beside the scan of the one before).  Depth 1 (the
 * default) keeps everything on compute_stream.  Changing the depth synchronises the device.  IVF_PLACE_DEVICE only; depth
 * in [1, 16].
 */
int ivf_set_pipeline_depth(ivf_index* index, int32_t depth);
/* Blocks the host until every search enqueued by ivf_search_device has finished. */
int ivf_synchronize(ivf_index* index);

/*
 * How a call with several queries is executed (Sec. 4.2 "Batching").
 *   0  automatic: batches of 4 or more queries on a device-resident fp16 / bf16 inner-product
 *      index with d a multiple of 64 are searched list-major (each selected cluster is read
 *      once per group of up to 32 queries that probe it, scores by MFMA); anything else query
 *      by query
 *   1  always query by query
 *   2  list-major from 2 queries on; IVF_ESTATE (and the mode stays) when the index has no
 *      list-major path
 * An index has the list-major path when all its rows are in HBM (IVF_PLACE_DEVICE), there are
 * fewer than 2^32 of them, and d is a multiple of 64 whose group of queries (32 of fp16 / bf16, 16
 * of fp32) fits LDS; any storage type, both metrics.
 * The results are the same in every mode (the MFMA scores only filter rows; the ranking uses
 * fp64 re-scores with the fp32 query).  A list-major batch may leave a few queries to be
 * searched again one by one (their candidate lists overflowed): ivf_search does that before it
 * returns; ivf_search_device returns without waiting and the library finishes the batch when
 * its stream is next needed or in ivf_synchronize(), so the outputs of a list-major
 * ivf_search_device call are complete after ivf_synchronize() only, and q_dev, ids_dev and
 * dists_dev must stay valid until then.  With bytes_gpu of ivf_search_stats a list-major call
 * reports the bytes of the union of the selected clusters.
 */
int ivf_set_batch_mode(ivf_index* index, int32_t mode);

/* Stage-level entry points, used by the parity tests. */
/* coarse scores of App. B's first step: scores (host, nq x nlist fp64), raw metric values */
int ivf_coarse_scores(ivf_index* index, const float* q, int32_t nq, double* scores);
/* the nprobe nearest clusters, nearest first: clusters (host, nq x min(nprobe, nlist)) */
int ivf_probe(ivf_index* index, const float* q, int32_t nq, int32_t nprobe, int32_t* clusters);
/*
 * The scores the list-major scan filters with (Sec. 4.2 "Batching": the matrix-matrix product), for
 * every row of one cluster against nq <= 32 queries: scores (host, nq x rows of the cluster, in row
 * order) are the filter scores, larger is better: the MFMA accumulators (query rounded to the
 * storage type, fp32 accumulation) for the inner product, 2 <q, y> - |y|^2 - |q|^2 from the same
 * accumulators and the stored row norms for squared L2; eps (host, nq) is the bound the scan
 * assumes for |score - exact value| (exact: <q, y>, or -|q - y|^2, with the fp32 query).
 * Only for an index that has the list-major path (see ivf_set_batch_mode), clusters of at most
 * 65536 rows.
 */
int ivf_batched_scores(ivf_index* index, const float* q, int32_t nq, int32_t cluster, float* scores, float* eps);
/* resident clusters in ascending order; *n in: capacity of clusters, out: count */
int ivf_resident(ivf_index* index, int32_t* clusters, int32_t* n);
/* layout as built: offsets (host, nlist + 1) and/or ids (host, n); either may be NULL */
int ivf_get_layout(ivf_index* index, int64_t* offsets, int64_t* ids);
/*
 * The plan of ivf_prefetch on its own (Sec. 4.3 "Prefetching target", Sec. 4.2 "Batching"): the
 * budget walk over clusters that are already ranked.  Needs no index and no GPU; ivf_prefetch runs
 * the same code after ranking on the GPU.
 *   ranked        host, nq x nprobe cluster numbers, nearest first for each query
 *   offsets       host, nlist + 1 row offsets; a cluster's size is its rows x row_bytes
 *   resident_off  host, nlist entries, in/out: row offset of a resident cluster in the buffer, -1 = absent
 *   *buffer_used  in/out: bytes of the buffer in use (clusters are placed at this mark)
 *   taken         host, room for nq x nprobe entries: the clusters to copy, in order; *n_taken = count
 * stats (or NULL) as ivf_prefetch fills it.
 */
int ivf_prefetch_plan(const int32_t* ranked, int32_t nq, int32_t nprobe, const int64_t* offsets,
                      int32_t nlist, size_t row_bytes, size_t budget_bytes, size_t buffer_bytes,
                      int64_t* resident_off, size_t* buffer_used, int32_t* taken, int32_t* n_taken,
                      ivf_prefetch_stats* stats /* or NULL */);
/*
 * The host part of ivf_cache_end_round on its own (Sec. 4.2 "Cache design"), after the hotness
 * update: which clusters leave and how the survivors are moved.  Needs no index and no GPU;
 * ivf_cache_end_round runs the same code and then performs the moves with device copies.
 *   hotness       host, nlist float32, in/out: evicted clusters get -1
 *   resident_off  host, nlist, in/out: row offset in the buffer, -1 = not cached
 *   *buffer_used  in/out: bytes in use
 *   evicted       host, room for nlist entries, in the order the clusters leave; *n_evicted = count
 *   moves         host, room for nlist entries, in the order to carry them out; *n_moves = count.
 *                 A move copies `bytes` bytes from from_byte to to_byte of the buffer; via_staging = 1
 *                 when source and destination overlap (copy out to a staging area first).
 */
typedef struct ivf_cache_move {
    int32_t cluster;
    int32_t via_staging;
    uint64_t from_byte, to_byte, bytes;
} ivf_cache_move;
int ivf_cache_plan(float* hotness, const int64_t* offsets, int32_t nlist, size_t row_bytes,
                   int64_t* resident_off, size_t* buffer_used, size_t buffer_bytes, float fraction,
                   int32_t* evicted, int32_t* n_evicted, ivf_cache_move* moves, int32_t* n_moves);

/*
 * How much to prefetch (App. C "Finding Prefetching Amount"; Sec. 4.1 "Prefetching amount"): the byte
 * budget b_p that minimises t_1 + t_2, where t_1 = t_llm while b_p <= bandwidth * t_llm and
 * b_p / bandwidth beyond it (the copy overlaps the generation that precedes the retrieval) and
 * t_2 = r_miss(b_p) * nprobe * t_cc (the host searches the missed clusters one after the other).
 *   bandwidth   host-to-device bytes per second, > 0        t_llm   seconds of generation, >= 0
 *   nprobe      clusters a search selects, >= 1             t_cc    host seconds per missed cluster, >= 0
 *   budgets, miss_rates   host, n >= 1 measured points of the miss-rate curve: budgets (bytes) strictly
 *               increasing, miss rates in [0, 1] and not rising; the curve is taken as linear between
 *               the points and constant outside them
 *   *amount     out: the best budget in bytes: bandwidth * t_llm (App. C's case 1) unless a measured
 *               point beyond it gives a strictly smaller time (case 2; of equal ones the smallest)
 *   *seconds    out, or NULL: the model's t_1 + t_2 at that budget
 *   *which      out, or NULL: 1 or 2, the case
 * t_1 + t_2 is piecewise linear in b_p, so no other amount can be better.  IVF_EINVAL for arguments
 * outside the stated ranges.  Needs no index and no GPU.  Caller keeps every array.
 */
int ivf_prefetch_amount(double bandwidth, double t_llm, int32_t nprobe, double t_cc,
                        const double* budgets, const double* miss_rates, int32_t n,
                        double* amount, double* seconds, int32_t* which);

/*
 * The host part of the hybrid search on its own (Sec. 4.1 step 3: the clusters of q_out that were
 * not prefetched are searched by CPU threads).  Needs no index and no GPU.
 *   lists     host, cluster-major rows of `dtype`, list c = rows offsets[c] .. offsets[c+1]
 *   offsets   host, enough entries for every listed cluster (c + 1 is read)
 *   ids       host, row -> id, or NULL (id = row)
 *   q         host, d float32         clusters  host, n_clusters lists to scan
 *   out_ids / out_scores   host, room for ivf_host_scan_capacity(k) entries: the candidates the merge step
 *             would receive, unordered, with their float64 scores (inner product, or squared L2)
 *   *n_out    number of candidates written; the k best by (score, id) are among them
 * threads: host threads to use (at least 1).  Caller keeps every array.
 */
int ivf_host_scan(const void* lists, const int64_t* offsets, const int64_t* ids, int32_t d, int dtype,
                  int metric, const float* q, const int32_t* clusters, int32_t n_clusters, int32_t k,
                  int32_t threads, int64_t* out_ids, double* out_scores, int32_t* n_out);
/* Entries ivf_host_scan may write for a search of k results (k' of "Arithmetic" above); 0 when k is
 * outside 1 .. IVF_MAX_K. */
int32_t ivf_host_scan_capacity(int32_t k);

/* Kernel timing with HIP events on compute_stream around each kernel of every search while
 * enabled (adds event records to the stream; leave off when timing throughput). */
int ivf_profile_enable(ivf_index* index, int on);
int ivf_profile_read(ivf_index* index, ivf_profile* out); /* synchronises compute_stream */
int ivf_profile_reset(ivf_index* index);

/*
 * Cluster cache (Sec. 4.2 "Cache design"; appendix on scheduling and cache: decay-based hotness,
 * cache fraction, eviction and consolidation after each batch).  IVF_PLACE_HOST only.
 *
 * With the cache configured, a cluster copied in by ivf_prefetch is cached with hotness h_init.
 * ivf_cache_end_round closes a round: every cached cluster's hotness becomes h / decay, plus
 * h_inc if a search since the previous round selected the cluster while it was resident; then,
 * while the resident bytes exceed fraction * device_buffer_bytes, the cached cluster of lowest
 * hotness is evicted (equal hotness: the larger cluster index first); the survivors are moved
 * to the front of the device buffer, in their order, so that the freed space is contiguous.
 * The moves run on copy_stream and the call returns when they are enqueued (the next prefetch and
 * the next search are ordered behind them); passing `stats` waits for them, to report their time.
 * Call it between batches, with no ivf_prefetch reset in between that should keep the cache:
 * IVF_PREFETCH_RESET drops the cache too.  Hotness is single precision on the device.
 *   fraction in [0, 1]; h_init >= 0; decay >= 1; h_inc >= 0.  fraction < 0 switches the cache off.
 * ivf_cache_hotness: host array of nlist floats, < 0 for clusters that are not cached.
 */
typedef struct ivf_cache_stats {
    int32_t n_cached;      /* cached clusters when the round ended, before eviction */
    int32_t n_evicted;
    uint64_t bytes_cached; /* their payload bytes, before eviction */
    uint64_t bytes_kept;   /* payload bytes still cached afterwards (= device buffer in use) */
    uint64_t bytes_moved;  /* bytes moved inside the device buffer by the consolidation */
    float ms_update;       /* hotness kernel + read-back */
    float ms_compact;      /* the moves inside the device buffer */
    int32_t n_launches;    /* kernels that carried them out (one per group of moves that do not disturb each other) */
} ivf_cache_stats;
int ivf_cache_configure(ivf_index* index, float fraction, float h_init, float decay, float h_inc);
int ivf_cache_end_round(ivf_index* index, ivf_cache_stats* stats /* or NULL */);
int ivf_cache_hotness(ivf_index* index, float* hotness);

/*
 * Prefetching scheduler (Sec. 4.2 "Scheduling optimization for prefetching"): groups the nq
 * queries of a global batch (host, nq x d float32, nq <= 4096) into micro-batches of `micro`
 * by a greedy search on squared L2 distance, on the GPU.  While queries remain, the remaining
 * query of lowest index seeds a micro-batch and the micro - 1 remaining queries nearest to it
 * follow, nearest first (equal distance: lower index first).  order (host, nq entries) receives
 * the query indices micro-batch after micro-batch; the last micro-batch may be short.
 * *ms_gpu (or NULL) receives the time of the two kernels.  Blocks until order is filled.
 */
int ivf_schedule(ivf_index* index, const float* q, int32_t nq, int32_t micro, int32_t* order, float* ms_gpu);

/* Number of host threads used for the scan of C_miss (default: hardware threads, at most 64). */
int ivf_set_host_threads(ivf_index* index, int32_t n);

const char* ivf_strerror(int status);
const char* ivf_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* IVF_H */
