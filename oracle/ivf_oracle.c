/*
 * CPU oracle for IVF-Flat search with lookahead prefetch (TeleRAG, arxiv 2502.20969).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP path is checked against.  It shares no code, header, table or helper
 * with the GPU library; only tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it.
 *
 * Everything is written out as the paper's Appendix B defines it:
 *   - coarse search:  the L clusters whose centroids are nearest to the query
 *                     (App. B, "L-argmin over centroids");
 *   - fine search:    the k nearest rows among the rows of those L clusters
 *                     (App. B, "k-argmin over the union of the L clusters",
 *                     followed by a sort);
 *   - lookahead:      rank clusters by distance to q_in, add whole clusters in
 *                     that order under a byte budget, skipping a cluster that
 *                     does not fit (Sec. 4.1 steps 1-4; Sec. 4.3 "Prefetching
 *                     target"); split the clusters of q_out into those that
 *                     are resident (C_overlap) and those that are not (C_miss);
 *                     search both parts and merge.
 *
 * Arithmetic: every score is accumulated in double, term by term in index
 * order t = 0..d-1.  Stored fp16 / bf16 values are widened exactly.  There is
 * no blocking, no SIMD intrinsic and no reordering.  OpenMP only distributes
 * independent candidates over threads; each candidate's sum is still the plain
 * sequential loop.
 *
 * Readings of points the paper leaves open:
 *   - "inner product" as a distance means: larger is nearer;
 *   - "L2" is the squared Euclidean distance, smaller is nearer;
 *   - the same metric is used for the coarse and the fine stage;
 *   - ties are broken by the smaller cluster index (coarse) or the smaller
 *     vector id (fine);
 *   - an over-budget cluster is skipped and the walk continues down the
 *     ranked list, never beyond the first L clusters.
 *
 * Parity status: every exported function below is pinned by tests that do not
 * call it to produce their expected values (hand-worked dyadic example,
 * brute-force kNN through a library matmul + argsort, set identities of the
 * lookahead split, closed-form budget cases; the prefetch amount of App. C by
 * its closed forms for a linear and an exponential miss-rate curve).  None is
 * "parity unpinned".
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_IP = 0, ORC_L2 = 1 };
enum { ORC_F32 = 0, ORC_F16 = 1, ORC_BF16 = 2 };

/* ---- exact widening of stored element types -------------------------------- */

/* IEEE binary16 -> double, from the bit fields (sign, 5-bit exponent, 10-bit fraction). */
static double widen_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);               /* zero and subnormals: f * 2^-24 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -v : v;
}

/* bfloat16 is the upper half of an IEEE binary32. */
static double widen_bf16(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double element(const void *base, int dtype, int64_t idx)
{
    switch (dtype) {
    case ORC_F32:  return (double)((const float *)base)[idx];
    case ORC_F16:  return widen_f16(((const uint16_t *)base)[idx]);
    default:       return widen_bf16(((const uint16_t *)base)[idx]);
    }
}

int orc_elem_size(int dtype) { return dtype == ORC_F32 ? 4 : 2; }

/* Exposed so the widening itself can be pinned against a library conversion. */
double orc_widen(uint16_t bits, int dtype)
{
    return dtype == ORC_F16 ? widen_f16(bits) : widen_bf16(bits);
}

/* ---- the distance function d(x, y) of App. B -------------------------------- */

/* Raw score of query x against row `row` of a row-major matrix with d columns.
 * IP: sum_t x_t*y_t.  L2: sum_t (x_t-y_t)^2. */
double orc_score(const float *x, const void *rows, int dtype, int64_t row, int32_t d, int metric)
{
    double acc = 0.0;
    for (int32_t t = 0; t < d; ++t) {
        double xt = (double)x[t];
        double yt = element(rows, dtype, row * (int64_t)d + t);
        if (metric == ORC_IP) {
            acc += xt * yt;
        } else {
            double diff = xt - yt;
            acc += diff * diff;
        }
    }
    return acc;
}

/* a is nearer than b?  IP: larger score.  L2: smaller score. */
static int nearer(double a, double b, int metric)
{
    return metric == ORC_IP ? (a > b) : (a < b);
}

typedef struct { double score; int64_t id; int64_t aux; } cand_t;

static int g_metric; /* comparator context; the sort is called from one thread */

static int cand_cmp(const void *pa, const void *pb)
{
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (nearer(a->score, b->score, g_metric)) return -1;
    if (nearer(b->score, a->score, g_metric)) return 1;
    if (a->id < b->id) return -1;
    if (a->id > b->id) return 1;
    return 0;
}

static void sort_nearest_first(cand_t *c, int64_t n, int metric)
{
    g_metric = metric;
    qsort(c, (size_t)n, sizeof *c, cand_cmp);
}

/* ---- layout: cluster-major lists from an assignment (Sec. "Implementation
 * Details": cluster data sits in one contiguous region) ------------------------ */

/* Stable grouping of rows by cluster.  off[c]..off[c+1] is the range of list c;
 * perm[p] is the input row that sits at position p.  Returns 0, or -1 when an
 * assignment is outside [0, nlist). */
int orc_build_layout(const int32_t *assign, int64_t n, int32_t nlist, int64_t *off, int64_t *perm)
{
    for (int32_t c = 0; c <= nlist; ++c) off[c] = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (assign[i] < 0 || assign[i] >= nlist) return -1;
        off[assign[i] + 1] += 1;
    }
    for (int32_t c = 0; c < nlist; ++c) off[c + 1] += off[c];
    int64_t *cursor = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nlist > 0 ? nlist : 1));
    if (!cursor) return -2;
    for (int32_t c = 0; c < nlist; ++c) cursor[c] = off[c];
    for (int64_t i = 0; i < n; ++i) perm[cursor[assign[i]]++] = i;
    free(cursor);
    return 0;
}

/* ---- coarse search (App. B, first step) ------------------------------------- */

/* The L nearest centroids of x, nearest first, ties by smaller cluster index.
 * L is clamped to nlist.  out_scores may be NULL.  Returns the number written. */
int32_t orc_probe(const float *centroids, int32_t nlist, int32_t d, int metric,
                  const float *x, int32_t L, int32_t *out_clusters, double *out_scores)
{
    if (L > nlist) L = nlist;
    if (L <= 0) return 0;
    cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)nlist);
    if (!c) return -2;
    for (int32_t j = 0; j < nlist; ++j) {
        c[j].score = orc_score(x, centroids, ORC_F32, j, d, metric);
        c[j].id = j;
        c[j].aux = 0;
    }
    sort_nearest_first(c, nlist, metric);
    for (int32_t i = 0; i < L; ++i) {
        out_clusters[i] = (int32_t)c[i].id;
        if (out_scores) out_scores[i] = c[i].score;
    }
    free(c);
    return L;
}

/* ---- fine search over a given set of clusters (App. B, second step) ---------- */

/* Scores every row of every listed cluster, sorts all of them, returns the k
 * nearest (score, id), nearest first.  Short results are padded with id -1 and
 * the worst possible score.  ids == NULL means row position is the id. */
static int search_clusters(const void *lists, int dtype, const int64_t *off, const int64_t *ids,
                           int32_t d, int metric, const float *x,
                           const int32_t *clusters, int32_t nclusters, int32_t k,
                           int64_t *out_ids, double *out_scores)
{
    int64_t total = 0;
    for (int32_t i = 0; i < nclusters; ++i) total += off[clusters[i] + 1] - off[clusters[i]];
    cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)(total > 0 ? total : 1));
    if (!c) return -2;
    int64_t pos = 0;
    for (int32_t i = 0; i < nclusters; ++i)
        for (int64_t r = off[clusters[i]]; r < off[clusters[i] + 1]; ++r) {
            c[pos].aux = r;
            c[pos].id = ids ? ids[r] : r;
            ++pos;
        }
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < total; ++p)
        c[p].score = orc_score(x, lists, dtype, c[p].aux, d, metric);
    sort_nearest_first(c, total, metric);
    for (int32_t i = 0; i < k; ++i) {
        if (i < total) {
            out_ids[i] = c[i].id;
            out_scores[i] = c[i].score;
        } else {
            out_ids[i] = -1;
            out_scores[i] = metric == ORC_IP ? -INFINITY : INFINITY;
        }
    }
    free(c);
    return 0;
}

/* Exposed for the per-stage parity checks (scan of an explicit cluster set). */
int orc_search_clusters(const void *lists, int dtype, const int64_t *off, const int64_t *ids,
                        int32_t d, int metric, const float *x,
                        const int32_t *clusters, int32_t nclusters, int32_t k,
                        int64_t *out_ids, double *out_scores)
{
    return search_clusters(lists, dtype, off, ids, d, metric, x, clusters, nclusters, k,
                           out_ids, out_scores);
}

/* IVF search of one query: probe L clusters, then the k nearest rows in them. */
int orc_search(const void *lists, int dtype, const int64_t *off, const int64_t *ids,
               const float *centroids, int32_t nlist, int32_t d, int metric,
               const float *x, int32_t L, int32_t k, int64_t *out_ids, double *out_scores)
{
    if (L > nlist) L = nlist;
    int32_t *probe = (int32_t *)malloc(sizeof(int32_t) * (size_t)(L > 0 ? L : 1));
    if (!probe) return -2;
    int32_t got = orc_probe(centroids, nlist, d, metric, x, L, probe, NULL);
    int rc = search_clusters(lists, dtype, off, ids, d, metric, x, probe, got, k, out_ids, out_scores);
    free(probe);
    return rc;
}

/* ---- lookahead retrieval (Sec. 4.1; Sec. 4.3 "Prefetching target") ----------- */

/* Plans one prefetch for q_in.  Walks the L clusters nearest to q_in, nearest
 * first.  A cluster already resident is passed over at no cost.  Otherwise its
 * payload is n_c*d*elem_size bytes; it is taken when it fits both the rest of
 * this call's budget and the rest of the device buffer (cap - *used), else it is
 * skipped whole and the walk goes on.  Taken clusters are marked in resident[]
 * and listed in chosen[] in the order taken.
 * Returns the number taken; *n_skipped counts clusters that did not fit;
 * *bytes_taken is the sum of their payloads. */
int32_t orc_prefetch(const float *centroids, int32_t nlist, int32_t d, int metric,
                     const int64_t *off, int dtype, const float *x_in, int32_t L,
                     uint64_t budget, uint64_t cap, uint8_t *resident, uint64_t *used,
                     int32_t *chosen, int32_t *n_skipped, uint64_t *bytes_taken)
{
    if (L > nlist) L = nlist;
    int32_t *ranked = (int32_t *)malloc(sizeof(int32_t) * (size_t)(L > 0 ? L : 1));
    if (!ranked) return -2;
    int32_t got = orc_probe(centroids, nlist, d, metric, x_in, L, ranked, NULL);
    uint64_t remaining = budget;
    uint64_t taken_bytes = 0;
    int32_t taken = 0, skipped = 0;
    for (int32_t i = 0; i < got; ++i) {
        int32_t c = ranked[i];
        if (resident[c]) continue;
        uint64_t bytes = (uint64_t)(off[c + 1] - off[c]) * (uint64_t)d * (uint64_t)orc_elem_size(dtype);
        if (bytes <= remaining && bytes <= cap - *used) {
            resident[c] = 1;
            remaining -= bytes;
            *used += bytes;
            taken_bytes += bytes;
            chosen[taken++] = c;
        } else {
            ++skipped;
        }
    }
    free(ranked);
    if (n_skipped) *n_skipped = skipped;
    if (bytes_taken) *bytes_taken = taken_bytes;
    return taken;
}

/* Splits the clusters of q_out into C_overlap (resident) and C_miss (not), each
 * kept in probe order.  Returns |C_out|. */
int32_t orc_split(const float *centroids, int32_t nlist, int32_t d, int metric,
                  const float *x_out, int32_t L, const uint8_t *resident,
                  int32_t *overlap, int32_t *n_overlap, int32_t *miss, int32_t *n_miss)
{
    if (L > nlist) L = nlist;
    int32_t *probe = (int32_t *)malloc(sizeof(int32_t) * (size_t)(L > 0 ? L : 1));
    if (!probe) return -2;
    int32_t got = orc_probe(centroids, nlist, d, metric, x_out, L, probe, NULL);
    int32_t no = 0, nm = 0;
    for (int32_t i = 0; i < got; ++i) {
        if (resident[probe[i]]) overlap[no++] = probe[i];
        else miss[nm++] = probe[i];
    }
    free(probe);
    *n_overlap = no;
    *n_miss = nm;
    return got;
}

/* Hybrid search: the k nearest of C_overlap, the k nearest of C_miss, merged
 * by one more sort (Sec. 4.1 step 4).  Also reports the hit rate
 * |C_overlap| / |C_out| (caption of Table 1). */
int orc_hybrid(const void *lists, int dtype, const int64_t *off, const int64_t *ids,
               const float *centroids, int32_t nlist, int32_t d, int metric,
               const float *x_out, int32_t L, int32_t k, const uint8_t *resident,
               int64_t *out_ids, double *out_scores, double *hit_rate)
{
    if (L > nlist) L = nlist;
    size_t cap = (size_t)(L > 0 ? L : 1);
    int32_t *overlap = (int32_t *)malloc(sizeof(int32_t) * cap);
    int32_t *miss = (int32_t *)malloc(sizeof(int32_t) * cap);
    cand_t *m = (cand_t *)malloc(sizeof(cand_t) * 2 * (size_t)(k > 0 ? k : 1));
    int64_t *pid = (int64_t *)malloc(sizeof(int64_t) * 2 * (size_t)(k > 0 ? k : 1));
    double *psc = (double *)malloc(sizeof(double) * 2 * (size_t)(k > 0 ? k : 1));
    if (!overlap || !miss || !m || !pid || !psc) return -2;
    int32_t no = 0, nm = 0;
    int32_t got = orc_split(centroids, nlist, d, metric, x_out, L, resident, overlap, &no, miss, &nm);
    search_clusters(lists, dtype, off, ids, d, metric, x_out, overlap, no, k, pid, psc);
    search_clusters(lists, dtype, off, ids, d, metric, x_out, miss, nm, k, pid + k, psc + k);
    int64_t cnt = 0;
    for (int32_t i = 0; i < 2 * k; ++i)
        if (pid[i] >= 0) { m[cnt].score = psc[i]; m[cnt].id = pid[i]; m[cnt].aux = 0; ++cnt; }
    sort_nearest_first(m, cnt, metric);
    for (int32_t i = 0; i < k; ++i) {
        if (i < cnt) { out_ids[i] = m[i].id; out_scores[i] = m[i].score; }
        else { out_ids[i] = -1; out_scores[i] = metric == ORC_IP ? -INFINITY : INFINITY; }
    }
    if (hit_rate) *hit_rate = got > 0 ? (double)no / (double)got : 0.0;
    free(overlap); free(miss); free(m); free(pid); free(psc);
    return 0;
}

/* ---- cluster cache with decaying hotness (Sec. 4.2 "Cache design"; appendix on
 *      scheduling and cache: the hotness transition and the cache fraction) ------- */

/* A cluster that has just been fetched is cached and starts with hotness h_init.
 * hot[c] < 0 means "not cached". */
void orc_cache_admit(float *hot, const uint8_t *resident, int32_t nlist, float h_init)
{
    for (int32_t c = 0; c < nlist; ++c)
        if (resident[c] && hot[c] < 0.0f) hot[c] = h_init;
}

/* One hotness round followed by the eviction that ends a batch.
 *
 * Hotness: for every cached cluster h <- h / decay, plus h_inc when the cluster
 * was used in the round that ends (used[c] != 0); used[] is cleared.  The
 * arithmetic is single precision, one division and one addition per cluster,
 * because the outcome decides an integer (which clusters leave) and the device
 * keeps hotness in single precision.
 *
 * Eviction: the cache may hold at most fraction*cap bytes.  While the resident
 * bytes exceed that, the cached cluster of lowest hotness leaves (equal
 * hotness: the larger cluster index leaves first); its resident flag is
 * cleared, its hotness becomes -1 and its payload n_c*d*elem_size is given back.
 * Returns the number evicted, listed in evicted[] in the order they left. */
int32_t orc_cache_round(float *hot, uint8_t *used_flags, uint8_t *resident, const int64_t *off,
                        int32_t nlist, int32_t d, int dtype, float decay, float h_inc,
                        double fraction, uint64_t cap, uint64_t *used_bytes, int32_t *evicted)
{
    for (int32_t c = 0; c < nlist; ++c) {
        if (resident[c] && hot[c] >= 0.0f) {
            float h = hot[c] / decay;
            if (used_flags[c]) h = h + h_inc;
            hot[c] = h;
        }
        used_flags[c] = 0;
    }
    const uint64_t limit = (uint64_t)(fraction * (double)cap);
    int32_t n_evicted = 0;
    while (*used_bytes > limit) {
        int32_t victim = -1;
        for (int32_t c = 0; c < nlist; ++c) {
            if (!resident[c]) continue;
            if (victim < 0 || hot[c] < hot[victim] || (hot[c] == hot[victim] && c > victim)) victim = c;
        }
        if (victim < 0) break;
        uint64_t bytes = (uint64_t)(off[victim + 1] - off[victim]) * (uint64_t)d * (uint64_t)orc_elem_size(dtype);
        resident[victim] = 0;
        hot[victim] = -1.0f;
        *used_bytes -= bytes;
        evicted[n_evicted++] = victim;
    }
    return n_evicted;
}

/* ---- prefetching scheduler (Sec. 4.2 "Scheduling optimization for prefetching") -- */

/* Groups the B queries of a global batch into micro-batches of m by a greedy
 * search on squared L2 distance.  While queries remain: the seed is the
 * remaining query of lowest index; its micro-batch is the seed followed by the
 * m-1 remaining queries nearest to the seed, nearest first (equal distance:
 * lower index first).  order[] receives the B query indices, micro-batch after
 * micro-batch (the last one may be short).  Distances are plain double sums of
 * squared differences in index order. */
int32_t orc_schedule(const float *q, int32_t B, int32_t d, int32_t m, int32_t *order)
{
    if (B < 1 || d < 1 || m < 1) return -1;
    uint8_t *taken = (uint8_t *)calloc((size_t)B, 1);
    if (!taken) return -2;
    int32_t pos = 0;
    while (pos < B) {
        int32_t seed = 0;
        while (taken[seed]) ++seed;
        taken[seed] = 1;
        order[pos++] = seed;
        for (int32_t slot = 1; slot < m && pos < B; ++slot) {
            int32_t best = -1;
            double best_dist = 0.0;
            for (int32_t j = 0; j < B; ++j) {
                if (taken[j]) continue;
                double dist = 0.0;
                for (int32_t t = 0; t < d; ++t) {
                    double diff = (double)q[(int64_t)seed * d + t] - (double)q[(int64_t)j * d + t];
                    dist += diff * diff;
                }
                if (best < 0 || dist < best_dist) { best = j; best_dist = dist; }
            }
            taken[best] = 1;
            order[pos++] = best;
        }
    }
    free(taken);
    return B;
}

/* ---- prefetch amount (App. C "Finding Prefetching Amount") ------------------------ */

/* Miss rate after prefetching b bytes, from n measured points (bs[i], rs[i]) with
 * bs increasing: linear between neighbouring points, constant before the first
 * and after the last. */
static double miss_rate_at(double b, const double *bs, const double *rs, int32_t n)
{
    if (b <= bs[0]) return rs[0];
    for (int32_t i = 1; i < n; ++i)
        if (b <= bs[i]) {
            const double x = (b - bs[i - 1]) / (bs[i] - bs[i - 1]);      /* 1 exactly at the measured point */
            return x >= 1.0 ? rs[i] : rs[i - 1] + (rs[i] - rs[i - 1]) * x;
        }
    return rs[n - 1];
}

/* The amount b_p that minimises t_1 + t_2 of App. C, by trying every amount on a
 * grid: t_1 = t_LLM up to b_p = B * t_LLM and b_p / B beyond (generation and
 * prefetch overlap), t_2 =
 * r_miss(b_p) * nprobe * t_cc (the CPU searches the missed clusters one after the
 * other).  Amounts tried: 0, step, 2 step, ... up to the larger of B * t_LLM and
 * the last measured point, and B * t_LLM itself (the boundary of App. C's case 1).
 * Of several amounts with the same smallest time the one nearest to B * t_LLM is
 * returned (case 1: "pushing b_p to the boundary").  *t_total receives the time. */
double orc_prefetch_amount(double B, double t_llm, int32_t nprobe, double t_cc,
                           const double *bs, const double *rs, int32_t n, double step, double *t_total)
{
    const double b1 = B * t_llm;
    const double hi = b1 > bs[n - 1] ? b1 : bs[n - 1];
    double best_b = b1;
    double best_t = t_llm + miss_rate_at(b1, bs, rs, n) * (double)nprobe * t_cc;
    for (int64_t g = 0; (double)g * step <= hi; ++g) {
        const double b = (double)g * step;
        const double t1 = b <= b1 ? t_llm : b / B;           /* App. C's piecewise t_1 */
        const double t = t1 + miss_rate_at(b, bs, rs, n) * (double)nprobe * t_cc;
        const double gap = b > b1 ? b - b1 : b1 - b, best_gap = best_b > b1 ? best_b - b1 : b1 - best_b;
        if (t < best_t || (t == best_t && gap < best_gap)) { best_t = t; best_b = b; }
    }
    if (t_total) *t_total = best_t;
    return best_b;
}

/* Number of OpenMP threads the scoring loop will use (for the baseline report). */
int orc_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
