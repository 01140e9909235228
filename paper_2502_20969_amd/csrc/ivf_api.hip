// C-ABI of libivf (include/ivf.h): index construction, lookahead prefetch planning and copies,
// and the search drivers that enqueue the kernels of ivf_kernels.hip.
#include "../../include/ivf.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <chrono>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "host_plan.h"
#include "host_scan.h"
#include "ivf_internal.h"

using namespace ivf;

// ---- errors -----------------------------------------------------------------------------------
static thread_local std::string g_last_error;

static int fail(int status, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return status;
}

#define HIP_TRY(expr)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess)                                                               \
            return fail(e_ == hipErrorOutOfMemory ? IVF_ENOMEM : IVF_EHIP, "%s: %s", #expr, \
                        hipGetErrorString(e_));                                             \
    } while (0)

extern "C" const char* ivf_strerror(int status) {
    switch (status) {
    case IVF_OK: return "ok";
    case IVF_EINVAL: return "invalid argument";
    case IVF_ENOMEM: return "out of memory";
    case IVF_EHIP: return "HIP call failed";
    case IVF_ESTATE: return "call not valid for this index";
    case IVF_ELIMIT: return "size above what this build supports";
    default: return "unknown status";
    }
}

extern "C" const char* ivf_last_error(void) { return g_last_error.c_str(); }

// ---- the index ----------------------------------------------------------------------------------
namespace {

constexpr int kMaxD = 4096;             // coarse kernel stages 4 queries x d floats in 64 KB of LDS
constexpr int kProfileRing = 2048;      // searches whose events are kept before a drain

struct Workspace {
    int nq = 0, nprobe = 0, k = 0, kprime = 0;
    size_t wg_cap = 0;               // scan workgroups (all queries of a call together) the tables below hold
    uint32_t pad = 0;
    float* d_q = nullptr;
    double* d_scores = nullptr;
    int32_t* d_probe = nullptr;
    SlotTables slots{nullptr, nullptr, nullptr, nullptr};
    uint64_t* d_sort_keys = nullptr;
    uint32_t* d_sort_idx = nullptr;
    WgDesc* d_desc = nullptr;
    uint64_t* d_part = nullptr;      // packed candidates: one list per scan wavefront
    uint64_t* d_heads = nullptr;     // the lists' best entries, densely
    int64_t* d_out_ids = nullptr;
    float* d_out_dists = nullptr;
    // exact second pass: per query a flag, the k-th best score found and a counter; its wavefronts' lists
    uint32_t* d_redo_flag = nullptr;
    double* d_redo_thr = nullptr;
    uint32_t* d_redo_ticket = nullptr;
    unsigned long long* d_redo_key = nullptr;
    long long* d_redo_id = nullptr;
    uint32_t* h_flag = nullptr;      // pinned copy of the flags for searches with host outputs
    uint32_t* hd_flag = nullptr;     // ... as the device addresses it
    // pinned host staging
    float* h_q = nullptr;
    float* hd_q = nullptr;           // h_q as the device addresses it
    unsigned long long* h_done = nullptr;    // completion word of single-query host searches (pinned)
    unsigned long long* hd_done = nullptr;   // ... as the device addresses it
    unsigned long long done_seq = 0;
    int32_t* h_probe = nullptr;
    int64_t* h_out_ids = nullptr;
    float* h_out_dists = nullptr;
    int64_t* hd_out_ids = nullptr;   // the same pinned buffers as the device addresses them: the merge
    float* hd_out_dists = nullptr;   // kernel of ivf_search writes its few results straight to the host
    HostCand* h_cand = nullptr;
    int32_t* h_cand_count = nullptr;
    double* h_scores = nullptr;   // only for ivf_coarse_scores (allocated on demand)
    size_t h_scores_len = 0;
    // batched (list-major) search
    int b_nq = 0, b_nprobe = 0;
    void* d_q_store = nullptr;
    float* d_thr = nullptr;
    float* d_thr_part = nullptr;
    float *d_cand_score = nullptr, *d_eps = nullptr, *d_qq = nullptr;
    uint32_t* d_surv_row = nullptr;
    uint32_t *d_list_count = nullptr, *d_cursor = nullptr, *d_qstart = nullptr, *d_tstart = nullptr, *d_qidx = nullptr;
    BatchTask* d_tasks = nullptr;
    uint32_t *d_cand_count = nullptr, *d_cand_row = nullptr;
    uint64_t* d_cand_key = nullptr;
    int32_t *d_overflow = nullptr, *h_overflow = nullptr;
};

struct ProfSet { hipEvent_t e[8]; };   // begin/end of the coarse, select, scan and merge kernels

}  // namespace

struct ivf_index {
    int64_t n = 0;
    int d = 0, dtype = 0, nlist = 0, metric = 0, placement = 0;
    size_t row_bytes = 0;
    int device = 0, n_cu = 256;
    size_t max_lds = 65536;        // LDS bytes one workgroup may use
    hipStream_t compute = nullptr, copy = nullptr;
    bool own_compute = false, own_copy = false;

    float* d_centroids = nullptr;
    int64_t* d_off = nullptr;
    int64_t* d_ids = nullptr;
    float row_norm_max = 0.f;        // largest Euclidean norm of a stored row
    float err_coef = 0.f;            // rounding bound of the scan kernel (scan_error_coef)
    // cluster cache (host placement): hotness per cluster (< 0 = not cached), use marks of the round
    bool cache_on = false;
    float cache_fraction = 0.5f, cache_h_init = 1.f, cache_decay = 2.f, cache_h_inc = 1.f;
    float* d_hot = nullptr;
    uint32_t* d_used = nullptr;
    void* d_move_tmp = nullptr;      // staging for a cluster whose old and new place overlap
    size_t move_tmp_bytes = 0;
    hipEvent_t ev_cache[4] = {nullptr, nullptr, nullptr, nullptr};
    hipEvent_t ev_round = nullptr;   // the searches of the round are done (recorded on the compute stream)
    MoveDesc* h_moves = nullptr;     // pinned: the moves of a consolidation, uploaded to d_moves
    MoveDesc* d_moves = nullptr;
    size_t moves_cap = 0;
    float* h_hot_stage = nullptr;    // pinned copy of the hotness values for their upload
    int64_t* d_res_off = nullptr;
    void* d_buf = nullptr;          // device lists (device placement) or the prefetch buffer
    size_t buf_bytes = 0;
    bool own_buf = false;

    std::vector<int64_t> h_off;
    std::vector<int64_t> h_ids;     // empty when id = row position
    void* h_lists = nullptr;        // pinned host lists (host placement)
    bool own_h_lists = false;
    std::vector<int64_t> h_res_off; // host mirror of d_res_off
    int64_t* h_res_stage = nullptr; // pinned copy used as the source of the table upload
    size_t buf_used = 0;
    hipEvent_t ev_pf_begin = nullptr, ev_pf_done = nullptr, ev_probe = nullptr, ev_pf_table = nullptr;
    bool pf_recorded = false;

    std::vector<uint64_t> rows_desc_prefix;   // prefix sums of list sizes, largest first
    int resident_grid[2] = {0, 0};            // scan workgroups resident at once, for kprime <= 64 / > 64
    int batched_grid = 0;                     // resident workgroups of the batched scan kernel
    int batch_mode = 0;                       // 0 auto, 1 always query by query, 2 list-major when eligible
    unsigned int* d_row_norm_max = nullptr;   // largest squared row norm (float bits); device placement
    float* d_row_norm = nullptr;              // squared norm of every row; device placement with squared L2
    ScanShape shape{0, 0, 0, 4};
    // Searches through ivf_search_device rotate over `lanes` (stream + workspace each) so that
    // independent queries overlap; lane 0 runs on compute_stream.  cs / cw: lane in use.
    // What a lane still owes for its last call (settle_lane).  A list-major batch: the queries whose
    // candidate lists overflowed have to be searched again one by one.  A query-by-query call of a
    // pipelined index: the queries whose result the merge could not prove get the exact second pass.
    struct Pending { bool on = false; bool list_major = false; const float* q = nullptr; int nq = 0, nprobe = 0, k = 0;
                     int64_t* ids = nullptr; float* dists = nullptr; unsigned long long done_seq = 0; };
    struct Lane { hipStream_t stream = nullptr; bool own = false; Workspace ws; Pending pending; };
    std::vector<Lane> lanes;
    size_t next_lane = 0;
    hipStream_t cs = nullptr;
    Workspace* cw = nullptr;
    std::unique_ptr<ThreadPool> pool;

    bool profiling = false;
    std::vector<ProfSet> prof_sets;
    size_t prof_used = 0;
    ivf_profile prof{};
    unsigned long long* d_prof_rows = nullptr;
};

static int enqueue_per_query(ivf_index* ix, const float* q_dev, int nq, int nprobe, int k,
                             int64_t* ids_dev, float* dists_dev, bool lazy = false);
static bool wait_done_word(const unsigned long long* word, unsigned long long want);

// ---- workspace for callers that cannot allocate (ivf_search_device_noalloc) -----------------------
// One fixed array per GPU, held until the process ends.  In host code the array's name is only a
// handle: its device address is looked up once per device (scratch_for_device) and that pointer
// is what is carved into buffers and handed to the kernels.
constexpr size_t kScratchBytes = IVF_NOALLOC_SCRATCH_BYTES;
constexpr int kScratchMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
static unsigned char* g_scratch_ptr[kScratchMaxDevices];

// device address of `scratch` on the current device (which must be `device`); looked up on first use
static int scratch_for_device(int device, unsigned char** out) {
    if (device < 0 || device >= kScratchMaxDevices) return fail(IVF_ELIMIT, "device %d has no scratch slot", device);
    if (!g_scratch_ptr[device]) {
        unsigned char* p = nullptr;
        hipError_t e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(IVF_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return IVF_OK;
}

namespace {

// releases without a status: used on teardown and on error paths, where nothing can be done about a failure
void dfree(void* p) { if (p) (void)hipFree(p); }
void hfree(void* p) { if (p) (void)hipHostFree(p); }

void free_workspace(Workspace& w) {
    dfree(w.d_q); dfree(w.d_scores); dfree(w.d_probe);
    dfree(w.slots.base); dfree(w.slots.grow); dfree(w.slots.nrows); dfree(w.slots.rprefix);
    dfree(w.d_sort_keys); dfree(w.d_sort_idx); dfree(w.d_part); dfree(w.d_heads);
    dfree(w.d_desc);
    dfree(w.d_out_ids); dfree(w.d_out_dists);
    dfree(w.d_redo_flag); dfree(w.d_redo_thr); dfree(w.d_redo_ticket);
    dfree(w.d_redo_id); dfree(w.d_redo_key); hfree(w.h_flag);
    hfree(w.h_q); hfree(w.h_done); hfree(w.h_probe); hfree(w.h_out_ids); hfree(w.h_out_dists);
    hfree(w.h_cand); hfree(w.h_cand_count); hfree(w.h_scores);
    dfree(w.d_thr_part); dfree(w.d_cand_score); dfree(w.d_eps); dfree(w.d_surv_row); dfree(w.d_qq);
    dfree(w.d_q_store); dfree(w.d_thr); dfree(w.d_list_count); dfree(w.d_cursor); dfree(w.d_qstart);
    dfree(w.d_tstart); dfree(w.d_qidx); dfree(w.d_tasks); dfree(w.d_cand_count); dfree(w.d_cand_row);
    dfree(w.d_cand_key); dfree(w.d_overflow); hfree(w.h_overflow);
    w = Workspace{};
}

// Number of scan workgroups per query for a call of `nq` searches of `nprobe` clusters with
// `kprime` candidates.  One query: as many as are resident at once (the rows are split statically),
// and no more wavefronts than the largest possible scan has batches.  Several queries share the
// GPU: together they get about four rounds of resident workgroups, at least one per query.
int scan_grid_for(ivf_index* ix, int nprobe, int kprime, int nq) {
    const int cls = kprime > 64 ? 1 : 0;
    if (ix->resident_grid[cls] == 0)
        ix->resident_grid[cls] = scan_resident_grid(ix->shape, ix->dtype, ix->metric, cls ? 128 : 64, ix->d, ix->n_cu);
    uint64_t rows = ix->rows_desc_prefix[std::min<size_t>(nprobe, ix->rows_desc_prefix.size() - 1)];
    uint64_t batches = rows / ix->shape.rows_per_batch + (uint64_t)nprobe;
    uint64_t g = (batches + kScanWaves - 1) / kScanWaves;
    uint64_t cap = (uint64_t)ix->resident_grid[cls];
    if (g > cap) g = cap;
    const uint64_t shared = (4 * cap + (uint64_t)nq - 1) / (uint64_t)nq;
    if (g > shared) g = shared;
    if (g < 1) g = 1;
    return (int)g;
}
// scan workgroups of all queries of a call together: an upper bound of nq * scan_grid_for(.., nq') for nq' <= nq
size_t scan_workgroup_bound(const ivf_index* ix, int nq) { return (size_t)4 * ix->n_cu * kScanMaxWgPerCu + (size_t)nq; }
// workgroups per query of the exact second pass: 64 for one query, fewer when a call has many
int redo_grid_for(int nq) { return std::max(1, 64 / std::max(nq, 1)); }
// entries of the lists it leaves behind, all queries of a call together (a bound for every nq' <= nq)
size_t redo_entries_bound(int nq, int k) { return (size_t)std::max(64, nq) * kRedoListsPerWg * (size_t)k; }

int enqueue_redo(ivf_index* ix, const float* q_dev, int nq, int nprobe, int k, int kprime, bool with_host,
                 int64_t* out_ids, float* out_dists);

void use_lane(ivf_index* ix, size_t i) {
    ix->cs = ix->lanes[i].stream;
    ix->cw = &ix->lanes[i].ws;
}

// waits on the host for every lane other than lane 0, then selects lane 0
// Finishes what lane i still owes: waits for its list-major batch and searches the queries whose
// candidate lists overflowed again, one by one.  Leaves the lane idle.  The lane in use is kept.
int settle_lane(ivf_index* ix, size_t i) {
    ivf_index::Lane& l = ix->lanes[i];
    if (!l.pending.on) return IVF_OK;
    hipStream_t cs = ix->cs; Workspace* cw = ix->cw;
    use_lane(ix, i);
    l.pending.on = false;
    const ivf_index::Pending pd = l.pending;
    int r = IVF_OK;
    hipError_t e = hipSuccess;
    // one query: its merge kernel set a completion word behind the flags; otherwise wait for the stream
    if (pd.list_major || pd.nq != 1 || !wait_done_word(l.ws.h_done, pd.done_seq)) e = hipStreamSynchronize(l.stream);
    if (e != hipSuccess) r = fail(IVF_EHIP, "hipStreamSynchronize: %s", hipGetErrorString(e));
    const bool was_profiling = ix->profiling;
    ix->profiling = false;
    bool redone = false;
    if (pd.list_major) {
        for (int qi = 0; qi < pd.nq && r == IVF_OK; ++qi)
            if (l.ws.h_overflow[qi]) {
                r = enqueue_per_query(ix, pd.q + (size_t)qi * ix->d, 1, pd.nprobe, pd.k, pd.ids + (size_t)qi * pd.k,
                                      pd.dists + (size_t)qi * pd.k);
                redone = true;
            }
    } else if (r == IVF_OK) {
        for (int qi = 0; qi < pd.nq; ++qi) redone = redone || l.ws.h_flag[qi] != 0;
        if (redone) r = enqueue_redo(ix, pd.q, pd.nq, pd.nprobe, pd.k, kprime_for(pd.k), false, pd.ids, pd.dists);
    }
    ix->profiling = was_profiling;
    if (r == IVF_OK && redone) {
        e = hipStreamSynchronize(l.stream);
        if (e != hipSuccess) r = fail(IVF_EHIP, "hipStreamSynchronize: %s", hipGetErrorString(e));
    }
    ix->cs = cs; ix->cw = cw;
    return r;
}

int settle_on_lane0(ivf_index* ix) {
    int rc;
    for (size_t i = 0; i < ix->lanes.size(); ++i)
        if ((rc = settle_lane(ix, i))) return rc;
    for (size_t i = 1; i < ix->lanes.size(); ++i) HIP_TRY(hipStreamSynchronize(ix->lanes[i].stream));
    use_lane(ix, 0);
    return IVF_OK;
}

int ensure_workspace(ivf_index* ix, int nq, int nprobe, int k) {
    Workspace& w = *ix->cw;
    const int kprime = kprime_for(k);
    const uint32_t pad = select_sort_pad(ix->nlist, nprobe);
    if (nq <= w.nq && nprobe <= w.nprobe && k <= w.k && pad <= w.pad) return IVF_OK;
    const int nq2 = std::max(nq, w.nq), np2 = std::max(nprobe, w.nprobe), k2 = std::max(k, w.k);
    const uint32_t pad2 = std::max(pad, w.pad);
    const int kp2 = std::max(kprime, w.kprime);
    HIP_TRY(hipDeviceSynchronize());
    free_workspace(w);
    const size_t nqz = nq2, npz = np2;
    HIP_TRY(hipMalloc(&w.d_q, nqz * ix->d * sizeof(float)));
    HIP_TRY(hipMalloc(&w.d_scores, nqz * ix->nlist * sizeof(double)));
    HIP_TRY(hipMalloc(&w.d_probe, nqz * npz * sizeof(int32_t)));
    HIP_TRY(hipMalloc(&w.slots.base, nqz * npz * sizeof(int64_t)));
    HIP_TRY(hipMalloc(&w.slots.grow, nqz * npz * sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&w.slots.nrows, nqz * npz * sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&w.slots.rprefix, nqz * (npz + 1) * sizeof(uint32_t)));
    const size_t wgs = scan_workgroup_bound(ix, nq2);
    HIP_TRY(hipMalloc(&w.d_desc, wgs * sizeof(WgDesc)));
    if (pad2 > (uint32_t)kSortLdsCap) {
        HIP_TRY(hipMalloc(&w.d_sort_keys, nqz * pad2 * sizeof(uint64_t)));
        HIP_TRY(hipMalloc(&w.d_sort_idx, nqz * pad2 * sizeof(uint32_t)));
    }
    HIP_TRY(hipMalloc(&w.d_part, wgs * kScanWaves * cand_slots(kp2) * sizeof(uint64_t)));
    HIP_TRY(hipMalloc(&w.d_heads, wgs * kScanWaves * sizeof(uint64_t)));
    HIP_TRY(hipMalloc(&w.d_out_ids, nqz * k2 * sizeof(int64_t)));
    HIP_TRY(hipMalloc(&w.d_out_dists, nqz * k2 * sizeof(float)));
    HIP_TRY(hipMalloc(&w.d_redo_flag, nqz * sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&w.d_redo_thr, nqz * sizeof(double)));
    HIP_TRY(hipMalloc(&w.d_redo_ticket, nqz * sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&w.d_redo_key, redo_entries_bound(nq2, k2) * sizeof(unsigned long long)));
    HIP_TRY(hipMalloc(&w.d_redo_id, redo_entries_bound(nq2, k2) * sizeof(long long)));
    HIP_TRY(hipHostMalloc(&w.h_flag, nqz * sizeof(uint32_t)));
    HIP_TRY(hipHostGetDevicePointer((void**)&w.hd_flag, w.h_flag, 0));
    memset(w.h_flag, 0, nqz * sizeof(uint32_t));
    HIP_TRY(hipHostMalloc(&w.h_q, nqz * ix->d * sizeof(float)));
    HIP_TRY(hipHostGetDevicePointer((void**)&w.hd_q, w.h_q, 0));
    HIP_TRY(hipHostMalloc(&w.h_done, sizeof(unsigned long long)));
    HIP_TRY(hipHostGetDevicePointer((void**)&w.hd_done, w.h_done, 0));
    *w.h_done = 0; w.done_seq = 0;
    HIP_TRY(hipHostMalloc(&w.h_probe, nqz * npz * sizeof(int32_t)));
    HIP_TRY(hipHostMalloc(&w.h_out_ids, nqz * k2 * sizeof(int64_t)));
    HIP_TRY(hipHostMalloc(&w.h_out_dists, nqz * k2 * sizeof(float)));
    HIP_TRY(hipHostGetDevicePointer((void**)&w.hd_out_ids, w.h_out_ids, 0));
    HIP_TRY(hipHostGetDevicePointer((void**)&w.hd_out_dists, w.h_out_dists, 0));
    HIP_TRY(hipHostMalloc(&w.h_cand, nqz * kp2 * sizeof(HostCand)));
    HIP_TRY(hipHostMalloc(&w.h_cand_count, nqz * sizeof(int32_t)));
    memset(w.h_cand_count, 0, nqz * sizeof(int32_t));
    w.nq = nq2; w.nprobe = np2; w.k = k2; w.kprime = kp2; w.pad = pad2; w.wg_cap = wgs;
    return IVF_OK;
}

int check_query_args(const ivf_index* ix, const void* q, int32_t nq, int32_t nprobe) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    if (!q) return fail(IVF_EINVAL, "query pointer is NULL");
    if (nq < 1) return fail(IVF_EINVAL, "nq must be at least 1 (got %d)", nq);
    if (nprobe < 1) return fail(IVF_EINVAL, "nprobe must be at least 1 (got %d)", nprobe);
    return IVF_OK;
}

// ---- profiling events ---------------------------------------------------------------------
int drain_profile(ivf_index* ix) {
    for (size_t i = 0; i < ix->lanes.size(); ++i) {
        int rc = settle_lane(ix, i);
        if (rc) return rc;
    }
    if (ix->prof_used == 0) return IVF_OK;
    for (auto& l : ix->lanes) HIP_TRY(hipStreamSynchronize(l.stream));
    for (size_t i = 0; i < ix->prof_used; ++i) {
        float ms[4];
        for (int j = 0; j < 4; ++j)
            HIP_TRY(hipEventElapsedTime(&ms[j], ix->prof_sets[i].e[2 * j], ix->prof_sets[i].e[2 * j + 1]));
        ix->prof.ms_coarse += ms[0]; ix->prof.ms_select += ms[1];
        ix->prof.ms_scan += ms[2]; ix->prof.ms_merge += ms[3];
        ix->prof.calls += 1;
    }
    ix->prof_used = 0;
    unsigned long long rows = 0;
    HIP_TRY(hipMemcpy(&rows, ix->d_prof_rows, sizeof rows, hipMemcpyDeviceToHost));
    ix->prof.scan_rows = rows;
    ix->prof.scan_bytes = rows * ix->row_bytes;
    return IVF_OK;
}

// events for kernel `which` (0 coarse .. 3 merge) of the search being enqueued, or nulls
int prof_events(ivf_index* ix, int which, hipEvent_t* e0, hipEvent_t* e1) {
    *e0 = *e1 = nullptr;
    if (!ix->profiling) return IVF_OK;
    if (which == 0 && ix->prof_used == ix->prof_sets.size()) {
        int rc = drain_profile(ix);
        if (rc) return rc;
    }
    *e0 = ix->prof_sets[ix->prof_used].e[2 * which];
    *e1 = ix->prof_sets[ix->prof_used].e[2 * which + 1];
    if (which == 3) ix->prof_used += 1;
    return IVF_OK;
}

// ---- kernel sequences ---------------------------------------------------------------------
// queries from the caller's host memory into d_q of the current workspace (which holds nq of them):
// through the pinned buffer, then by a kernel when they are few and by the copy engine otherwise
static int stage_queries(ivf_index* ix, const float* q_host, int nq) {
    Workspace& w = *ix->cw;
    const size_t n = (size_t)nq * ix->d;
    memcpy(w.h_q, q_host, n * sizeof(float));
    if (n * sizeof(float) <= (size_t)256 << 10) HIP_TRY(launch_stage_query(w.hd_q, w.d_q, n, ix->cs));
    else HIP_TRY(hipMemcpyAsync(w.d_q, w.h_q, n * sizeof(float), hipMemcpyHostToDevice, ix->cs));
    return IVF_OK;
}

// coarse scoring + selection for nq queries already in d_q (device); leaves the probe lists
// and slot tables in the workspace
int enqueue_probe(ivf_index* ix, const float* q_dev, int nq, int nprobe, int grid, bool count_rows = true,
                  bool is_search = false) {
    Workspace& w = *ix->cw;
    int rc;
    // the per-workgroup tables of the workspace were sized for w.wg_cap workgroups and w.nq queries
    if ((size_t)grid * nq > w.wg_cap || nq > w.nq)
        return fail(IVF_ESTATE, "workspace holds %zu scan workgroups and %d queries, asked for %d x %d", w.wg_cap, w.nq, grid, nq);
    hipEvent_t e0, e1;
    if ((rc = prof_events(ix, 0, &e0, &e1))) return rc;
    CoarseArgs ca{ix->d_centroids, q_dev, w.d_scores, ix->nlist, ix->d, nq, ix->metric};
    HIP_TRY(launch_coarse(ca, ix->cs, e0, e1));
    if ((rc = prof_events(ix, 1, &e0, &e1))) return rc;
    SelectArgs sa{};
    sa.scores = w.d_scores; sa.probe = w.d_probe; sa.off = ix->d_off; sa.res_off = ix->d_res_off;
    sa.slots = w.slots; sa.sort_keys = w.d_sort_keys; sa.sort_idx = w.d_sort_idx;
    sa.nlist = ix->nlist; sa.nprobe = nprobe; sa.nq = nq; sa.metric = ix->metric;
    sa.grid = grid;
    sa.desc = w.d_desc;
    sa.rows_counter = ix->profiling && count_rows ? ix->d_prof_rows : nullptr;
    sa.used = is_search && ix->cache_on ? ix->d_used : nullptr;
    HIP_TRY(launch_select(sa, ix->cs, e0, e1));
    return IVF_OK;
}

int enqueue_scan(ivf_index* ix, const float* q_dev, int nq, int nprobe, int kprime, int grid) {
    Workspace& w = *ix->cw;
    ScanArgs sc{};
    sc.buf = ix->d_buf; sc.q = q_dev; sc.slots = w.slots;
    sc.part = w.d_part; sc.heads = w.d_heads;
    sc.desc = w.d_desc;
    sc.d = ix->d; sc.dtype = ix->dtype; sc.metric = ix->metric; sc.nprobe = nprobe; sc.nq = nq;
    sc.kprime = kprime; sc.grid = grid; sc.shape = ix->shape;
    hipEvent_t e0, e1;
    int rc = prof_events(ix, 2, &e0, &e1);
    if (rc) return rc;
    HIP_TRY(launch_scan(sc, ix->cs, e0, e1));
    return IVF_OK;
}

// host_flags: the proof flags also go to the pinned array (searches whose caller waits on the host)
int enqueue_merge(ivf_index* ix, const float* q_dev, int nq, int nprobe, int k, int kprime, int grid,
                  bool with_host, int64_t* out_ids, float* out_dists, bool signal_done = false, bool host_flags = false) {
    Workspace& w = *ix->cw;
    MergeArgs ma{};
    ma.buf = ix->d_buf; ma.q = q_dev; ma.ids = ix->d_ids; ma.slots = w.slots;
    ma.err_coef = ix->err_coef; ma.row_norm_max = ix->row_norm_max;
    ma.redo_flag = w.d_redo_flag; ma.redo_thr = w.d_redo_thr; ma.redo_ticket = w.d_redo_ticket;
    ma.host_flag = host_flags ? w.hd_flag : nullptr;
    ma.part = w.d_part; ma.heads = w.d_heads;
    ma.host_cand = with_host ? w.h_cand : nullptr;
    ma.host_count = with_host ? w.h_cand_count : nullptr;
    ma.out_ids = out_ids; ma.out_dists = out_dists;
    ma.d = ix->d; ma.dtype = ix->dtype; ma.metric = ix->metric; ma.nprobe = nprobe; ma.nq = nq;
    ma.k = k; ma.kprime = kprime; ma.nparts = grid * kScanWaves; ma.list_len = cand_slots(kprime);
    ma.identity = ix->placement == IVF_PLACE_DEVICE;
    if (signal_done) { ma.done = w.hd_done; ma.done_value = ++w.done_seq; }
    hipEvent_t e0, e1;
    int rc = prof_events(ix, 3, &e0, &e1);
    if (rc) return rc;
    HIP_TRY(launch_merge(ma, ix->cs, e0, e1));
    return IVF_OK;
}

// The exact second pass for the queries whose merge could not prove its result; queries that were
// proven cost one workgroup round that leaves at once.
int enqueue_redo(ivf_index* ix, const float* q_dev, int nq, int nprobe, int k, int kprime, bool with_host,
                 int64_t* out_ids, float* out_dists) {
    Workspace& w = *ix->cw;
    RedoArgs ra{};
    ra.buf = ix->d_buf; ra.q = q_dev; ra.ids = ix->d_ids; ra.slots = w.slots;
    ra.redo_flag = w.d_redo_flag; ra.redo_thr = w.d_redo_thr; ra.redo_ticket = w.d_redo_ticket;
    ra.list_key = w.d_redo_key; ra.list_id = w.d_redo_id;
    ra.host_cand = with_host ? w.h_cand : nullptr;
    ra.host_count = with_host ? w.h_cand_count : nullptr;
    ra.out_ids = out_ids; ra.out_dists = out_dists;
    ra.d = ix->d; ra.dtype = ix->dtype; ra.metric = ix->metric; ra.nprobe = nprobe; ra.nq = nq; ra.k = k;
    ra.kprime = kprime;
    HIP_TRY(launch_redo(ra, redo_grid_for(nq), ix->cs));
    return IVF_OK;
}

// ---- batched (list-major) search ----------------------------------------------------------------
constexpr int kCandCap = 65536;          // candidates a query may collect in the batched scan
constexpr int kSurvCap = 4096;           // of those, rows re-scored in fp64

bool batched_eligible(const ivf_index* ix, int nq) {
    if (ix->batch_mode == 1 || nq < 2) return false;
    if (ix->placement != IVF_PLACE_DEVICE || !ix->d_row_norm_max || ix->n >= (int64_t)1 << 32) return false;
    if (ix->metric != IVF_IP && !ix->d_row_norm) return false;
    if (ix->d % 64 != 0) return false;                          // the MFMA kernels walk whole blocks of elements
    if (batched_scan_lds(ix->d, ix->dtype) > ix->max_lds) return false;    // a group's queries must fit LDS
    return ix->batch_mode == 2 || nq >= 4;
}

int ensure_batched_workspace(ivf_index* ix, int nq, int nprobe) {
    Workspace& w = *ix->cw;
    if (nq <= w.b_nq && nprobe <= w.b_nprobe) return IVF_OK;
    const int nq2 = std::max(nq, w.b_nq), np2 = std::max(nprobe, w.b_nprobe);
    HIP_TRY(hipDeviceSynchronize());
    dfree(w.d_thr_part); dfree(w.d_cand_score); dfree(w.d_eps); dfree(w.d_surv_row); dfree(w.d_qq);
    dfree(w.d_q_store); dfree(w.d_thr); dfree(w.d_list_count); dfree(w.d_cursor); dfree(w.d_qstart);
    dfree(w.d_tstart); dfree(w.d_qidx); dfree(w.d_tasks); dfree(w.d_cand_count); dfree(w.d_cand_row);
    dfree(w.d_cand_key); dfree(w.d_overflow); hfree(w.h_overflow);
    w.d_thr_part = nullptr; w.d_cand_score = nullptr; w.d_eps = nullptr; w.d_surv_row = nullptr; w.d_qq = nullptr;
    w.d_q_store = nullptr; w.d_thr = nullptr; w.d_list_count = w.d_cursor = w.d_qstart = w.d_tstart = w.d_qidx = nullptr;
    w.d_tasks = nullptr; w.d_cand_count = w.d_cand_row = nullptr; w.d_cand_key = nullptr; w.d_overflow = w.h_overflow = nullptr;
    w.b_nq = w.b_nprobe = 0;
    const size_t nqz = nq2, nl = ix->nlist;
    const uint64_t task_cap = batched_task_bound(ix->h_off.data(), ix->nlist, nq2, ix->dtype);
    HIP_TRY(hipMalloc(&w.d_q_store, nqz * ix->d * 2));
    HIP_TRY(hipMalloc(&w.d_qq, nqz * sizeof(float)));
    HIP_TRY(hipMalloc(&w.d_thr, nqz * sizeof(float)));
    HIP_TRY(hipMalloc(&w.d_thr_part, batched_thr_part_floats(nq2) * sizeof(float)));
    HIP_TRY(hipMalloc(&w.d_list_count, (nl + 1) * sizeof(uint32_t)));      // + the scan's task counter
    HIP_TRY(hipMalloc(&w.d_cursor, nl * sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&w.d_qstart, (nl + 1) * sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&w.d_tstart, (nl + 1) * sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&w.d_qidx, nqz * np2 * sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&w.d_tasks, task_cap * sizeof(BatchTask)));
    HIP_TRY(hipMalloc(&w.d_cand_count, nqz * sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&w.d_cand_row, nqz * kCandCap * sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&w.d_cand_score, nqz * kCandCap * sizeof(float)));
    HIP_TRY(hipMalloc(&w.d_eps, nqz * sizeof(float)));
    HIP_TRY(hipMalloc(&w.d_surv_row, nqz * kSurvCap * sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&w.d_cand_key, nqz * kSurvCap * sizeof(uint64_t)));
    HIP_TRY(hipMalloc(&w.d_overflow, nqz * sizeof(int32_t)));
    HIP_TRY(hipHostMalloc(&w.h_overflow, nqz * sizeof(int32_t)));
    w.b_nq = nq2; w.b_nprobe = np2;
    return IVF_OK;
}

// the parts of the batched scan's arguments that do not depend on the call
static void fill_batched_args(const ivf_index* ix, const Workspace& w, BatchedArgs& b) {
    b.lists = ix->d_buf; b.off = ix->d_off; b.ids = ix->d_ids; b.probe = w.d_probe;
    b.q_store = w.d_q_store; b.thr = w.d_thr; b.thr_part = w.d_thr_part; b.row_norm_max_bits = ix->d_row_norm_max;
    b.list_count = w.d_list_count; b.cursor = w.d_cursor; b.qstart = w.d_qstart; b.tstart = w.d_tstart;
    b.ticket = w.d_list_count + ix->nlist;
    b.qidx = w.d_qidx; b.tasks = w.d_tasks; b.cand_count = w.d_cand_count; b.cand_row = w.d_cand_row;
    b.cand_key = w.d_cand_key; b.cand_score = w.d_cand_score; b.eps = w.d_eps; b.qq = w.d_qq; b.row_norm = ix->d_row_norm;
    b.surv_row = w.d_surv_row; b.overflow = w.d_overflow;
    b.nlist = ix->nlist; b.d = ix->d; b.dtype = ix->dtype; b.metric = ix->metric;
    b.cand_cap = kCandCap; b.surv_cap = kSurvCap;
    b.group_q = batched_group_q(ix->dtype);
    b.acc_coef = (float)ix->d * 0x1p-23f;            // d products accumulated in fp32, in an order the hardware chooses
    b.samp_coef = batched_sample_coef(ix->d, ix->dtype, ix->metric);
}

// coarse + select for the batch, then the list-major scan and the final ranking into (out_ids,
// out_dists) (device pointers); the overflow flags land in the workspace
int enqueue_batched(ivf_index* ix, const float* q_dev, int nq, int nprobe, int k, int64_t* out_ids, float* out_dists) {
    Workspace& w = *ix->cw;
    int rc;
    if ((rc = enqueue_probe(ix, q_dev, nq, nprobe, 1, false, true))) return rc;
    if (ix->batched_grid == 0) ix->batched_grid = batched_resident_grid(ix->dtype, ix->metric, ix->d, ix->n_cu);
    BatchedArgs b{};
    fill_batched_args(ix, w, b);
    b.q = q_dev; b.out_ids = out_ids; b.out_dists = out_dists;
    b.rows_counter = ix->profiling ? ix->d_prof_rows : nullptr;
    b.nq = nq; b.nprobe = nprobe; b.k = k; b.kprime = kprime_for(k);
    hipEvent_t e0, e1, m0, m1;
    if ((rc = prof_events(ix, 2, &e0, &e1))) return rc;
    if ((rc = prof_events(ix, 3, &m0, &m1))) return rc;
    HIP_TRY(launch_batched(b, ix->batched_grid, ix->cs, e0, e1));
    if (m0) { HIP_TRY(hipEventRecord(m0, ix->cs)); HIP_TRY(hipEventRecord(m1, ix->cs)); }
    HIP_TRY(hipMemcpyAsync(w.h_overflow, w.d_overflow, (size_t)nq * sizeof(int32_t), hipMemcpyDeviceToHost, ix->cs));
    return IVF_OK;
}

// ---- construction helpers --------------------------------------------------------------------
int init_common(ivf_index* ix, int64_t n, int32_t d, int dtype, const float* centroids, int32_t nlist,
                int metric, int placement, void* compute_stream, void* copy_stream) {
    ix->n = n; ix->d = d; ix->dtype = dtype; ix->nlist = nlist; ix->metric = metric;
    ix->placement = placement;
    ix->row_bytes = (size_t)d * (dtype == IVF_F32 ? 4 : 2);
    HIP_TRY(hipGetDevice(&ix->device));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, ix->device));
    ix->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    if (prop.sharedMemPerBlock > 0) ix->max_lds = prop.sharedMemPerBlock;
    if (compute_stream) ix->compute = (hipStream_t)compute_stream;
    else { HIP_TRY(hipStreamCreateWithFlags(&ix->compute, hipStreamNonBlocking)); ix->own_compute = true; }
    ix->lanes.resize(1);
    ix->lanes[0].stream = ix->compute;
    ix->cs = ix->compute;
    ix->cw = &ix->lanes[0].ws;
    if (copy_stream) ix->copy = (hipStream_t)copy_stream;
    else { HIP_TRY(hipStreamCreateWithFlags(&ix->copy, hipStreamNonBlocking)); ix->own_copy = true; }
    HIP_TRY(hipEventCreate(&ix->ev_pf_begin));
    HIP_TRY(hipEventCreate(&ix->ev_pf_done));
    HIP_TRY(hipEventCreateWithFlags(&ix->ev_probe, hipEventDisableTiming));
    HIP_TRY(hipEventCreateWithFlags(&ix->ev_pf_table, hipEventDisableTiming));
    HIP_TRY(hipMalloc(&ix->d_centroids, (size_t)nlist * d * sizeof(float)));
    HIP_TRY(hipMemcpy(ix->d_centroids, centroids, (size_t)nlist * d * sizeof(float), hipMemcpyHostToDevice));
    HIP_TRY(hipMalloc(&ix->d_off, (size_t)(nlist + 1) * sizeof(int64_t)));
    HIP_TRY(hipMalloc(&ix->d_res_off, (size_t)nlist * sizeof(int64_t)));
    HIP_TRY(hipMalloc(&ix->d_prof_rows, sizeof(unsigned long long)));
    HIP_TRY(hipMemset(ix->d_prof_rows, 0, sizeof(unsigned long long)));
    HIP_TRY(hipDeviceSynchronize());
    ix->shape = pick_scan_shape(d, dtype);
    ix->err_coef = scan_error_coef(ix->shape, d, dtype, metric);
    // looked up here so that the entry point that must not allocate does no first-use work
    unsigned char* sp = nullptr;
    int rc = scratch_for_device(ix->device, &sp);
    if (rc) return rc;
    for (int cls = 0; cls < 2; ++cls)
        ix->resident_grid[cls] = scan_resident_grid(ix->shape, dtype, metric, cls ? 128 : 64, d, ix->n_cu);
    return IVF_OK;
}

// after h_off / h_ids are set: uploads them and initialises residency
int finish_tables(ivf_index* ix, size_t device_buffer_bytes) {
    const int nlist = ix->nlist;
    HIP_TRY(hipMemcpy(ix->d_off, ix->h_off.data(), (size_t)(nlist + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
    if (!ix->h_ids.empty()) {
        HIP_TRY(hipMalloc(&ix->d_ids, (size_t)ix->n * sizeof(int64_t)));
        HIP_TRY(hipMemcpy(ix->d_ids, ix->h_ids.data(), (size_t)ix->n * sizeof(int64_t), hipMemcpyHostToDevice));
    }
    ix->h_res_off.assign(nlist, -1);
    if (ix->placement == IVF_PLACE_DEVICE) {
        for (int c = 0; c < nlist; ++c) ix->h_res_off[c] = ix->h_off[c];
    } else {
        ix->buf_bytes = device_buffer_bytes;
        if (device_buffer_bytes > 0) HIP_TRY(hipMalloc(&ix->d_buf, device_buffer_bytes));
        ix->own_buf = true;
        HIP_TRY(hipHostMalloc(&ix->h_res_stage, (size_t)nlist * sizeof(int64_t)));
        unsigned hw = std::thread::hardware_concurrency();
        int nt = hw == 0 ? 8 : (int)std::min(hw, 64u);
        ix->pool.reset(new ThreadPool(nt));
    }
    HIP_TRY(hipMemcpy(ix->d_res_off, ix->h_res_off.data(), (size_t)nlist * sizeof(int64_t), hipMemcpyHostToDevice));
    // the largest row norm: part of the rounding bounds of the scans
    if (ix->placement == IVF_PLACE_DEVICE) {
        HIP_TRY(hipMalloc(&ix->d_row_norm_max, sizeof(unsigned int)));
        HIP_TRY(hipMemset(ix->d_row_norm_max, 0, sizeof(unsigned int)));
        HIP_TRY(hipDeviceSynchronize());
        // squared L2 also keeps every row's norm: the list-major scan turns inner products into distances with them
        if (ix->metric != IVF_IP && ix->n > 0) HIP_TRY(hipMalloc(&ix->d_row_norm, (size_t)ix->n * sizeof(float)));
        HIP_TRY(launch_row_norms(ix->d_buf, ix->dtype, ix->n, ix->d, ix->d_row_norm_max, ix->d_row_norm, ix->compute));
        HIP_TRY(hipStreamSynchronize(ix->compute));
        unsigned int bits = 0;
        HIP_TRY(hipMemcpy(&bits, ix->d_row_norm_max, sizeof bits, hipMemcpyDeviceToHost));
        float sq;
        memcpy(&sq, &bits, sizeof sq);
        ix->row_norm_max = sqrtf(sq) * 1.0001f;         // the squared norm was rounded to fp32, and so is the root
    } else {
        ix->row_norm_max = host_row_norm_max(ix->h_lists, ix->dtype, ix->n, ix->d, *ix->pool) * 1.0001f;
    }
    std::vector<uint64_t> sizes(nlist);
    for (int c = 0; c < nlist; ++c) sizes[c] = (uint64_t)(ix->h_off[c + 1] - ix->h_off[c]);
    std::sort(sizes.begin(), sizes.end(), std::greater<uint64_t>());
    ix->rows_desc_prefix.assign(nlist + 1, 0);
    for (int c = 0; c < nlist; ++c) ix->rows_desc_prefix[c + 1] = ix->rows_desc_prefix[c] + sizes[c];
    return IVF_OK;
}

int check_build_args(const void* data, int64_t n, int32_t d, int dtype, const float* centroids,
                     int32_t nlist, int metric, int placement, ivf_index** out) {
    if (!data && n > 0) return fail(IVF_EINVAL, "vector data pointer is NULL");
    if (!centroids || !out) return fail(IVF_EINVAL, "centroids or out is NULL");
    if (n < 0 || d < 1 || nlist < 1) return fail(IVF_EINVAL, "need n >= 0, d >= 1, nlist >= 1");
    if (dtype < IVF_F32 || dtype > IVF_BF16) return fail(IVF_EINVAL, "unknown dtype %d", dtype);
    if (metric != IVF_IP && metric != IVF_L2) return fail(IVF_EINVAL, "unknown metric %d", metric);
    if (placement != IVF_PLACE_DEVICE && placement != IVF_PLACE_HOST)
        return fail(IVF_EINVAL, "unknown placement %d", placement);
    if (d > kMaxD) return fail(IVF_ELIMIT, "d = %d is above the supported %d", d, kMaxD);
    if (n >= 0xFFFFFFFFll) return fail(IVF_ELIMIT, "n = %lld does not fit 32-bit row numbers", (long long)n);
    if (placement == IVF_PLACE_HOST &&
        !(__builtin_cpu_supports("avx2") && __builtin_cpu_supports("fma") && __builtin_cpu_supports("f16c")))
        return fail(IVF_ESTATE, "host placement needs a CPU with AVX2, FMA and F16C");
    return IVF_OK;
}

}  // namespace

extern "C" void ivf_free(ivf_index* ix) {
    if (!ix) return;
    for (size_t i = 0; i < ix->lanes.size(); ++i) (void)settle_lane(ix, i);     // what the lanes still owe their callers
    (void)hipDeviceSynchronize();
    for (auto& l : ix->lanes) { free_workspace(l.ws); if (l.own) (void)hipStreamDestroy(l.stream); }
    for (auto& s : ix->prof_sets) for (auto& e : s.e) (void)hipEventDestroy(e);
    dfree(ix->d_centroids); dfree(ix->d_off); dfree(ix->d_ids);
    dfree(ix->d_hot); dfree(ix->d_used); dfree(ix->d_move_tmp);
    for (auto& e : ix->ev_cache) if (e) (void)hipEventDestroy(e);
    if (ix->ev_round) (void)hipEventDestroy(ix->ev_round);
    hfree(ix->h_moves); hfree(ix->h_hot_stage); dfree(ix->d_moves);
    dfree(ix->d_res_off);
    dfree(ix->d_prof_rows); dfree(ix->d_row_norm_max); dfree(ix->d_row_norm);
    if (ix->own_buf) dfree(ix->d_buf);
    if (ix->own_h_lists) hfree(ix->h_lists);
    hfree(ix->h_res_stage);
    if (ix->ev_pf_begin) (void)hipEventDestroy(ix->ev_pf_begin);
    if (ix->ev_pf_done) (void)hipEventDestroy(ix->ev_pf_done);
    if (ix->ev_probe) (void)hipEventDestroy(ix->ev_probe);
    if (ix->ev_pf_table) (void)hipEventDestroy(ix->ev_pf_table);
    if (ix->own_compute) (void)hipStreamDestroy(ix->compute);
    if (ix->own_copy) (void)hipStreamDestroy(ix->copy);
    delete ix;
}

extern "C" int ivf_build_layout(const void* vectors, int64_t n, int32_t d, int dtype,
                                const float* centroids, int32_t nlist, const int32_t* assign,
                                const int64_t* ids, int metric, int placement,
                                size_t device_buffer_bytes, void* compute_stream, void* copy_stream,
                                ivf_index** out) {
    int rc = check_build_args(vectors, n, d, dtype, centroids, nlist, metric, placement, out);
    if (rc) return rc;
    if (!assign && n > 0) return fail(IVF_EINVAL, "assign is NULL");
    // stable grouping by cluster: pos[i] = position of input row i in cluster-major order
    std::vector<int64_t> off(nlist + 1, 0);
    for (int64_t i = 0; i < n; ++i) {
        if (assign[i] < 0 || assign[i] >= nlist)
            return fail(IVF_EINVAL, "assign[%lld] = %d is outside [0, %d)", (long long)i, assign[i], nlist);
        off[assign[i] + 1] += 1;
    }
    for (int c = 0; c < nlist; ++c) off[c + 1] += off[c];
    std::vector<int64_t> pos(n), cursor(off.begin(), off.end() - 1);
    for (int64_t i = 0; i < n; ++i) pos[i] = cursor[assign[i]]++;

    ivf_index* ix = new (std::nothrow) ivf_index();
    if (!ix) return fail(IVF_ENOMEM, "host allocation failed");
    rc = init_common(ix, n, d, dtype, centroids, nlist, metric, placement, compute_stream, copy_stream);
    if (rc) { ivf_free(ix); return rc; }
    ix->h_off = off;
    ix->h_ids.resize(n);
    for (int64_t i = 0; i < n; ++i) {
        int64_t id = ids ? ids[i] : i;
        if (id < 0) { ivf_free(ix); return fail(IVF_EINVAL, "ids[%lld] is negative", (long long)i); }
        ix->h_ids[pos[i]] = id;
    }
    const size_t rb = ix->row_bytes;
    auto body = [&]() -> int {
        if (placement == IVF_PLACE_DEVICE) {
            ix->buf_bytes = (size_t)n * rb;
            ix->own_buf = true;
            if (n > 0) HIP_TRY(hipMalloc(&ix->d_buf, ix->buf_bytes));
            // upload input rows in chunks and scatter them to their cluster-major positions
            const int64_t chunk = std::max<int64_t>(1, std::min<int64_t>(n, (int64_t)((256u << 20) / rb)));
            void* d_stage = nullptr; int64_t* d_pos = nullptr;
            if (n > 0) {
                HIP_TRY(hipMalloc(&d_stage, (size_t)chunk * rb));
                HIP_TRY(hipMalloc(&d_pos, (size_t)chunk * sizeof(int64_t)));
            }
            int status = IVF_OK;
            for (int64_t i0 = 0; i0 < n && status == IVF_OK; i0 += chunk) {
                int64_t cnt = std::min(chunk, n - i0);
                hipError_t e = hipMemcpy(d_stage, (const char*)vectors + (size_t)i0 * rb, (size_t)cnt * rb, hipMemcpyHostToDevice);
                if (e == hipSuccess) e = hipMemcpy(d_pos, pos.data() + i0, (size_t)cnt * sizeof(int64_t), hipMemcpyHostToDevice);
                if (e == hipSuccess) e = launch_scatter_rows(d_stage, ix->d_buf, d_pos, cnt, rb, ix->cs);
                if (e == hipSuccess) e = hipStreamSynchronize(ix->cs);
                if (e != hipSuccess) status = fail(IVF_EHIP, "layout upload: %s", hipGetErrorString(e));
            }
            dfree(d_stage); dfree(d_pos);
            if (status) return status;
        } else {
            if (n > 0) HIP_TRY(hipHostMalloc(&ix->h_lists, (size_t)n * rb));
            ix->own_h_lists = true;
            for (int64_t i = 0; i < n; ++i)
                memcpy((char*)ix->h_lists + (size_t)pos[i] * rb, (const char*)vectors + (size_t)i * rb, rb);
        }
        return finish_tables(ix, device_buffer_bytes);
    };
    rc = body();
    if (rc) { ivf_free(ix); return rc; }
    *out = ix;
    return IVF_OK;
}

extern "C" int ivf_adopt_layout(void* lists, const int64_t* offsets, const int64_t* ids, int64_t n,
                                int32_t d, int dtype, const float* centroids, int32_t nlist,
                                int metric, int placement, size_t device_buffer_bytes,
                                void* compute_stream, void* copy_stream, ivf_index** out) {
    int rc = check_build_args(lists, n, d, dtype, centroids, nlist, metric, placement, out);
    if (rc) return rc;
    if (!offsets) return fail(IVF_EINVAL, "offsets is NULL");
    if (offsets[0] != 0 || offsets[nlist] != n) return fail(IVF_EINVAL, "offsets must run from 0 to n");
    for (int c = 0; c < nlist; ++c)
        if (offsets[c + 1] < offsets[c]) return fail(IVF_EINVAL, "offsets decrease at cluster %d", c);
    ivf_index* ix = new (std::nothrow) ivf_index();
    if (!ix) return fail(IVF_ENOMEM, "host allocation failed");
    rc = init_common(ix, n, d, dtype, centroids, nlist, metric, placement, compute_stream, copy_stream);
    if (rc) { ivf_free(ix); return rc; }
    ix->h_off.assign(offsets, offsets + nlist + 1);
    if (ids) {
        for (int64_t i = 0; i < n; ++i)
            if (ids[i] < 0) { ivf_free(ix); return fail(IVF_EINVAL, "ids[%lld] is negative", (long long)i); }
        ix->h_ids.assign(ids, ids + n);
    }
    if (placement == IVF_PLACE_DEVICE) {
        ix->d_buf = lists; ix->buf_bytes = (size_t)n * ix->row_bytes; ix->own_buf = false;
    } else {
        ix->h_lists = lists; ix->own_h_lists = false;
    }
    rc = finish_tables(ix, device_buffer_bytes);
    if (rc) { ivf_free(ix); return rc; }
    *out = ix;
    return IVF_OK;
}

extern "C" int ivf_reserve(ivf_index* ix, int32_t nq, int32_t nprobe, int32_t k) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    if (nq < 1 || nprobe < 1 || k < 1) return fail(IVF_EINVAL, "nq, nprobe and k must be at least 1");
    if (k > IVF_MAX_K) return fail(IVF_ELIMIT, "k = %d is above IVF_MAX_K = %d", k, IVF_MAX_K);
    for (size_t i = 0; i < ix->lanes.size(); ++i) {
        int rc = settle_lane(ix, i);           // a workspace that grows is freed first
        if (rc) return rc;
    }
    for (size_t i = 0; i < ix->lanes.size(); ++i) {
        use_lane(ix, i);
        int rc = ensure_workspace(ix, nq, std::min(nprobe, ix->nlist), k);
        if (rc) { use_lane(ix, 0); return rc; }
    }
    use_lane(ix, 0);
    return IVF_OK;
}

extern "C" int ivf_set_pipeline_depth(ivf_index* ix, int32_t depth) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    if (depth < 1 || depth > 16) return fail(IVF_EINVAL, "pipeline depth must be in [1, 16]");
    if (ix->placement != IVF_PLACE_DEVICE) return fail(IVF_ESTATE, "pipelining needs a device-resident index");
    for (size_t i = 0; i < ix->lanes.size(); ++i) {
        int rc = settle_lane(ix, i);
        if (rc) return rc;
    }
    HIP_TRY(hipDeviceSynchronize());
    while ((int)ix->lanes.size() > depth) {
        auto& l = ix->lanes.back();
        free_workspace(l.ws);
        if (l.own) (void)hipStreamDestroy(l.stream);
        ix->lanes.pop_back();
    }
    while ((int)ix->lanes.size() < depth) {
        ivf_index::Lane l;
        const hipError_t e = hipStreamCreateWithFlags(&l.stream, hipStreamNonBlocking);
        if (e != hipSuccess) {
            use_lane(ix, 0);          // the lanes may have moved in memory: point at lane 0 again before leaving
            return fail(IVF_EHIP, "hipStreamCreateWithFlags: %s", hipGetErrorString(e));
        }
        l.own = true;
        ix->lanes.push_back(l);
    }
    ix->next_lane = 0;
    use_lane(ix, 0);
    return IVF_OK;
}

extern "C" int ivf_synchronize(ivf_index* ix) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    for (size_t i = 0; i < ix->lanes.size(); ++i) {
        int rc = settle_lane(ix, i);
        if (rc) return rc;
    }
    for (auto& l : ix->lanes) HIP_TRY(hipStreamSynchronize(l.stream));
    return IVF_OK;
}

// ---- search -------------------------------------------------------------------------------------
static double now_ms() {
    using namespace std::chrono;
    return duration<double, std::milli>(steady_clock::now().time_since_epoch()).count();
}

// Watches a completion word for up to two milliseconds; false when it did not arrive in that time
// (the caller then waits for the stream, which also brings any launch error to light).
static bool wait_done_word(const unsigned long long* word, unsigned long long want) {
    if (__atomic_load_n(word, __ATOMIC_ACQUIRE) == want) return true;
    const double t_end = now_ms() + 2.0;
    for (;;) {
        for (int i = 0; i < 256; ++i) {
            if (__atomic_load_n(word, __ATOMIC_ACQUIRE) == want) return true;
            __builtin_ia32_pause();
        }
        if (now_ms() > t_end) return false;
    }
}

// Device-pointer search of nq queries, query by query in one launch sequence (grid.y = nq).
// lazy: no second pass is enqueued; the proof flags go to the pinned array (and, for one query, a
// completion word follows them) and the caller looks at them later (settle_lane)
static int enqueue_per_query(ivf_index* ix, const float* q_dev, int nq, int nprobe, int k,
                             int64_t* ids_dev, float* dists_dev, bool lazy) {
    int r;
    if ((r = ensure_workspace(ix, nq, nprobe, k))) return r;
    const int kprime = kprime_for(k);
    const int grid = scan_grid_for(ix, nprobe, kprime, nq);
    if ((r = enqueue_probe(ix, q_dev, nq, nprobe, grid, true, true))) return r;
    if ((r = enqueue_scan(ix, q_dev, nq, nprobe, kprime, grid))) return r;
    if ((r = enqueue_merge(ix, q_dev, nq, nprobe, k, kprime, grid, false, ids_dev, dists_dev, lazy && nq == 1, lazy))) return r;
    if (lazy) return IVF_OK;
    return enqueue_redo(ix, q_dev, nq, nprobe, k, kprime, false, ids_dev, dists_dev);
}

// List-major batched search into device outputs.  Synchronises the stream to read the overflow
// flags; a query whose candidate list overflowed is searched again on its own.
static int run_batched(ivf_index* ix, size_t lane, const float* q_dev, int nq, int nprobe, int k,
                       int64_t* ids_dev, float* dists_dev, bool defer) {
    int r;
    if ((r = ensure_workspace(ix, nq, nprobe, k))) return r;
    if ((r = ensure_batched_workspace(ix, nq, nprobe))) return r;
    if ((r = enqueue_batched(ix, q_dev, nq, nprobe, k, ids_dev, dists_dev))) return r;
    ivf_index::Pending& pd = ix->lanes[lane].pending;
    pd.on = true; pd.list_major = true; pd.q = q_dev; pd.nq = nq; pd.nprobe = nprobe; pd.k = k; pd.ids = ids_dev; pd.dists = dists_dev;
    // the overflow flags are looked at when the lane is next needed (or at ivf_synchronize), so that
    // the first kernels of the next batch, on another lane, run beside this batch's scan
    return defer ? IVF_OK : settle_lane(ix, lane);
}

extern "C" int ivf_set_batch_mode(ivf_index* ix, int32_t mode) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    if (mode < 0 || mode > 2) return fail(IVF_EINVAL, "batch mode must be 0, 1 or 2");
    if (mode == 2) {
        const int saved = ix->batch_mode;
        ix->batch_mode = 2;
        const bool ok = batched_eligible(ix, 2);
        ix->batch_mode = saved;
        if (!ok) return fail(IVF_ESTATE, "this index has no list-major scan (needs all rows in HBM, fewer than 2^32 of them, and d a multiple of 64 that fits LDS)");
    }
    ix->batch_mode = mode;
    return IVF_OK;
}

extern "C" int ivf_search_device(ivf_index* ix, const float* q_dev, int32_t nq, int32_t nprobe,
                                 int32_t k, int64_t* ids_dev, float* dists_dev) {
    int rc = check_query_args(ix, q_dev, nq, nprobe);
    if (rc) return rc;
    if (!ids_dev || !dists_dev) return fail(IVF_EINVAL, "output pointer is NULL");
    if (k < 1) return fail(IVF_EINVAL, "k must be at least 1 (got %d)", k);
    if (k > IVF_MAX_K) return fail(IVF_ELIMIT, "k = %d is above IVF_MAX_K = %d", k, IVF_MAX_K);
    if (ix->placement != IVF_PLACE_DEVICE)
        return fail(IVF_ESTATE, "ivf_search_device needs a device-resident index");
    if (((uintptr_t)q_dev & 15u) != 0) return fail(IVF_EINVAL, "q_dev must be 16-byte aligned");
    nprobe = std::min(nprobe, ix->nlist);
    const size_t lane = ix->next_lane;
    if ((rc = settle_lane(ix, lane))) return rc;
    use_lane(ix, lane);
    ix->next_lane = (ix->next_lane + 1) % ix->lanes.size();
    if (batched_eligible(ix, nq)) rc = run_batched(ix, lane, q_dev, nq, nprobe, k, ids_dev, dists_dev, true);
    else {
        // one stream: the exact second pass follows every merge on the stream, outputs are complete in
        // stream order.  Several: it is decided when the lane is next needed or in ivf_synchronize.
        const bool lazy = ix->lanes.size() > 1;
        rc = enqueue_per_query(ix, q_dev, nq, nprobe, k, ids_dev, dists_dev, lazy);
        if (rc == IVF_OK && lazy) {
            ivf_index::Pending& pd = ix->lanes[lane].pending;
            pd.on = true; pd.list_major = false; pd.q = q_dev; pd.nq = nq; pd.nprobe = nprobe; pd.k = k;
            pd.ids = ids_dev; pd.dists = dists_dev; pd.done_seq = ix->lanes[lane].ws.done_seq;
        }
    }
    use_lane(ix, 0);
    return rc;
}

// Carves the device buffers of a query-by-query search out of `base` (256-byte aligned pieces) and
// returns the bytes needed; with base == nullptr only the size is computed.
static size_t carve_search_buffers(Workspace& w, unsigned char* base, const ivf_index* ix, int nq, int nprobe,
                                   int k, int kprime, int grid, uint32_t pad) {
    size_t at = 0;
    auto take = [&](size_t bytes) -> void* {
        void* p = base ? base + at : nullptr;
        at += (bytes + 255) & ~(size_t)255;
        return p;
    };
    const size_t nqz = nq, npz = nprobe, gz = grid;
    w.d_scores = (double*)take(nqz * ix->nlist * sizeof(double));
    w.d_probe = (int32_t*)take(nqz * npz * sizeof(int32_t));
    w.slots.base = (int64_t*)take(nqz * npz * sizeof(int64_t));
    w.slots.grow = (uint32_t*)take(nqz * npz * sizeof(uint32_t));
    w.slots.nrows = (uint32_t*)take(nqz * npz * sizeof(uint32_t));
    w.slots.rprefix = (uint32_t*)take(nqz * (npz + 1) * sizeof(uint32_t));
    w.d_desc = (WgDesc*)take(nqz * gz * sizeof(WgDesc));
    if (pad > (uint32_t)kSortLdsCap) {
        w.d_sort_keys = (uint64_t*)take(nqz * pad * sizeof(uint64_t));
        w.d_sort_idx = (uint32_t*)take(nqz * pad * sizeof(uint32_t));
    }
    w.d_part = (uint64_t*)take(nqz * gz * kScanWaves * cand_slots(kprime) * sizeof(uint64_t));
    w.d_heads = (uint64_t*)take(nqz * gz * kScanWaves * sizeof(uint64_t));
    w.d_redo_flag = (uint32_t*)take(nqz * sizeof(uint32_t));
    w.d_redo_thr = (double*)take(nqz * sizeof(double));
    w.d_redo_ticket = (uint32_t*)take(nqz * sizeof(uint32_t));
    const size_t redo_entries = nqz * redo_grid_for(nq) * kRedoListsPerWg * (size_t)k;
    w.d_redo_key = (unsigned long long*)take(redo_entries * sizeof(unsigned long long));
    w.d_redo_id = (long long*)take(redo_entries * sizeof(long long));
    return at;
}

extern "C" int ivf_search_device_noalloc(ivf_index* ix, const float* q_dev, int32_t nq, int32_t nprobe,
                                         int32_t k, int64_t* ids_dev, float* dists_dev) {
    int rc = check_query_args(ix, q_dev, nq, nprobe);
    if (rc) return rc;
    if (!ids_dev || !dists_dev) return fail(IVF_EINVAL, "output pointer is NULL");
    if (k < 1) return fail(IVF_EINVAL, "k must be at least 1 (got %d)", k);
    if (k > IVF_MAX_K) return fail(IVF_ELIMIT, "k = %d is above IVF_MAX_K = %d", k, IVF_MAX_K);
    if (ix->placement != IVF_PLACE_DEVICE)
        return fail(IVF_ESTATE, "ivf_search_device_noalloc needs a device-resident index");
    if (((uintptr_t)q_dev & 15u) != 0) return fail(IVF_EINVAL, "q_dev must be 16-byte aligned");
    for (auto& l : ix->lanes)
        if (l.pending.on) return fail(IVF_ESTATE, "a list-major batch is unfinished: call ivf_synchronize() first");
    nprobe = std::min(nprobe, ix->nlist);
    const int kprime = kprime_for(k);
    const int grid = scan_grid_for(ix, nprobe, kprime, nq);
    const uint32_t pad = select_sort_pad(ix->nlist, nprobe);
    Workspace w{};
    const size_t need = carve_search_buffers(w, nullptr, ix, nq, nprobe, k, kprime, grid, pad);
    if (need > kScratchBytes)
        return fail(IVF_ELIMIT, "this search needs %zu bytes of workspace, the fixed scratch area holds %zu "
                    "(nq %d, nprobe %d, k %d): use ivf_search_device", need, kScratchBytes, nq, nprobe, k);
    unsigned char* sp = nullptr;
    if ((rc = scratch_for_device(ix->device, &sp))) return rc;
    carve_search_buffers(w, sp, ix, nq, nprobe, k, kprime, grid, pad);
    w.nq = nq; w.nprobe = nprobe; w.k = k; w.kprime = kprime; w.pad = pad; w.wg_cap = (size_t)grid * nq;
    // the kernels of one call only ever read what an earlier kernel of the same call wrote, so
    // nothing in the area has to start at zero
    hipStream_t cs = ix->cs; Workspace* cw = ix->cw;
    ix->cs = ix->compute; ix->cw = &w;
    rc = enqueue_probe(ix, q_dev, nq, nprobe, grid, true, true);
    if (!rc) rc = enqueue_scan(ix, q_dev, nq, nprobe, kprime, grid);
    if (!rc) rc = enqueue_merge(ix, q_dev, nq, nprobe, k, kprime, grid, false, ids_dev, dists_dev);
    if (!rc) rc = enqueue_redo(ix, q_dev, nq, nprobe, k, kprime, false, ids_dev, dists_dev);
    ix->cs = cs; ix->cw = cw;
    return rc;
}


extern "C" int ivf_search(ivf_index* ix, const float* q_out, int32_t nq, int32_t nprobe, int32_t k,
                          int64_t* ids, float* dists, ivf_search_stats* stats) {
    int rc = check_query_args(ix, q_out, nq, nprobe);
    if (rc) return rc;
    if (!ids || !dists) return fail(IVF_EINVAL, "output pointer is NULL");
    if (k < 1) return fail(IVF_EINVAL, "k must be at least 1 (got %d)", k);
    if (k > IVF_MAX_K) return fail(IVF_ELIMIT, "k = %d is above IVF_MAX_K = %d", k, IVF_MAX_K);
    const double t0 = now_ms();
    nprobe = std::min(nprobe, ix->nlist);
    if ((rc = settle_on_lane0(ix))) return rc;
    if ((rc = ensure_workspace(ix, nq, nprobe, k))) return rc;
    Workspace& w = *ix->cw;
    const int kprime = kprime_for(k);
    const int grid = scan_grid_for(ix, nprobe, kprime, nq);
    const bool hybrid = ix->placement == IVF_PLACE_HOST;
    ivf_search_stats st{};

    if ((rc = stage_queries(ix, q_out, nq))) return rc;
    if (batched_eligible(ix, nq)) {
        // list-major batched search: every selected cluster is read once per group of 32 queries
        if ((rc = run_batched(ix, 0, w.d_q, nq, nprobe, k, w.d_out_ids, w.d_out_dists, false))) return rc;
        HIP_TRY(hipMemcpy(ids, w.d_out_ids, (size_t)nq * k * sizeof(int64_t), hipMemcpyDeviceToHost));
        HIP_TRY(hipMemcpy(dists, w.d_out_dists, (size_t)nq * k * sizeof(float), hipMemcpyDeviceToHost));
        if (stats) {
            HIP_TRY(hipMemcpy(w.h_probe, w.d_probe, (size_t)nq * nprobe * sizeof(int32_t), hipMemcpyDeviceToHost));
            std::vector<uint8_t> seen(ix->nlist, 0);
            for (size_t i = 0; i < (size_t)nq * nprobe; ++i) {
                int32_t c = w.h_probe[i];
                if (!seen[c]) { seen[c] = 1; st.bytes_gpu += (uint64_t)(ix->h_off[c + 1] - ix->h_off[c]) * ix->row_bytes; }
            }
            st.n_probed = nq * nprobe; st.n_overlap = nq * nprobe; st.hit_rate = 1.f;
            st.ms_total = (float)(now_ms() - t0);
            *stats = st;
        }
        return IVF_OK;
    }
    if (hybrid && ix->pf_recorded) HIP_TRY(hipStreamWaitEvent(ix->cs, ix->ev_pf_done, 0));
    if ((rc = enqueue_probe(ix, w.d_q, nq, nprobe, grid, true, true))) return rc;
    const bool want_probe = hybrid || stats;
    if (want_probe) {
        HIP_TRY(hipMemcpyAsync(w.h_probe, w.d_probe, (size_t)nq * nprobe * sizeof(int32_t), hipMemcpyDeviceToHost, ix->cs));
        HIP_TRY(hipEventRecord(ix->ev_probe, ix->cs));
    }
    if ((rc = enqueue_scan(ix, w.d_q, nq, nprobe, kprime, grid))) return rc;

    if (want_probe) {
        HIP_TRY(hipEventSynchronize(ix->ev_probe));
        st.ms_probe = (float)(now_ms() - t0);
        double hit_sum = 0.0;
        std::vector<int32_t> miss;
        const double ts = now_ms();
        for (int qi = 0; qi < nq; ++qi) {
            miss.clear();
            int overlap = 0;
            for (int i = 0; i < nprobe; ++i) {
                int32_t c = w.h_probe[(size_t)qi * nprobe + i];
                uint64_t bytes = (uint64_t)(ix->h_off[c + 1] - ix->h_off[c]) * ix->row_bytes;
                if (ix->h_res_off[c] >= 0) { ++overlap; st.bytes_gpu += bytes; }
                else { miss.push_back(c); st.bytes_host += bytes; }
            }
            st.n_probed += nprobe; st.n_overlap += overlap; st.n_miss += (int)miss.size();
            hit_sum += (double)overlap / (double)nprobe;
            if (hybrid) {
                HostScanArgs ha{ix->h_lists, ix->h_off.data(), ix->h_ids.empty() ? nullptr : ix->h_ids.data(),
                                ix->d, ix->dtype, ix->metric, q_out + (size_t)qi * ix->d,
                                miss.data(), (int)miss.size(), kprime, k, ix->row_norm_max};
                bool exact_pass = false;
                w.h_cand_count[qi] = host_scan_query(ha, *ix->pool, w.h_cand + (size_t)qi * kprime, nullptr, &exact_pass);
                st.n_exact_host += exact_pass ? 1 : 0;
            }
        }
        st.ms_host_scan = (float)(now_ms() - ts);
        st.hit_rate = (float)(hit_sum / nq);
    }
    // nq x k results: the kernel stores them in the pinned host buffers itself (no copy to enqueue)
    // One query: the kernel also sets a completion word after the results; the host watches that
    // word instead of waiting for the stream to drain (the stream keeps its order for later calls).
    const bool watch = nq == 1;
    if ((rc = enqueue_merge(ix, w.d_q, nq, nprobe, k, kprime, grid, hybrid, w.hd_out_ids, w.hd_out_dists, watch, true))) return rc;
    if (!watch || !wait_done_word(w.h_done, w.done_seq)) HIP_TRY(hipStreamSynchronize(ix->cs));
    // a query whose result the merge could not prove gets the exact second pass (rare)
    bool redo = false;
    for (int qi = 0; qi < nq; ++qi) { redo = redo || w.h_flag[qi] != 0; st.n_exact_gpu += w.h_flag[qi] != 0 ? 1 : 0; }
    if (redo) {
        if ((rc = enqueue_redo(ix, w.d_q, nq, nprobe, k, kprime, hybrid, w.hd_out_ids, w.hd_out_dists))) return rc;
        HIP_TRY(hipStreamSynchronize(ix->cs));
    }
    memcpy(ids, w.h_out_ids, (size_t)nq * k * sizeof(int64_t));
    memcpy(dists, w.h_out_dists, (size_t)nq * k * sizeof(float));
    st.ms_total = (float)(now_ms() - t0);
    if (stats) *stats = st;
    return IVF_OK;
}

// ---- lookahead prefetch --------------------------------------------------------------------------
extern "C" int ivf_prefetch_plan(const int32_t* ranked, int32_t nq, int32_t nprobe, const int64_t* offsets,
                                 int32_t nlist, size_t row_bytes, size_t budget_bytes, size_t buffer_bytes,
                                 int64_t* resident_off, size_t* buffer_used, int32_t* taken, int32_t* n_taken,
                                 ivf_prefetch_stats* stats) {
    if (!ranked || !offsets || !resident_off || !buffer_used || !taken || !n_taken) return fail(IVF_EINVAL, "NULL argument");
    if (nq < 1 || nprobe < 1 || nlist < 1 || row_bytes < 1) return fail(IVF_EINVAL, "nq, nprobe, nlist and row_bytes must be at least 1");
    if (*buffer_used > buffer_bytes) return fail(IVF_EINVAL, "buffer_used is above buffer_bytes");
    for (size_t i = 0; i < (size_t)nq * nprobe; ++i)
        if (ranked[i] < 0 || ranked[i] >= nlist) return fail(IVF_EINVAL, "ranked[%zu] = %d is not a cluster", i, ranked[i]);
    std::vector<int32_t> t;
    ivf_prefetch_stats st{};
    plan_prefetch(ranked, nq, nprobe, offsets, row_bytes, budget_bytes, buffer_bytes, *buffer_used, resident_off, t, st);
    std::copy(t.begin(), t.end(), taken);
    *n_taken = (int32_t)t.size();
    if (stats) *stats = st;
    return IVF_OK;
}

extern "C" int ivf_prefetch_amount(double bandwidth, double t_llm, int32_t nprobe, double t_cc,
                                   const double* budgets, const double* miss_rates, int32_t n,
                                   double* amount, double* seconds, int32_t* which) {
    if (!budgets || !miss_rates || !amount) return fail(IVF_EINVAL, "NULL argument");
    if (!(bandwidth > 0.0) || !(t_llm >= 0.0) || !(t_cc >= 0.0) || nprobe < 1 || n < 1 ||
        !std::isfinite(bandwidth) || !std::isfinite(t_llm) || !std::isfinite(t_cc))
        return fail(IVF_EINVAL, "bandwidth must be positive, t_llm and t_cc not negative, nprobe and n at least 1");
    for (int32_t i = 0; i < n; ++i) {
        if (!(budgets[i] >= 0.0) || !std::isfinite(budgets[i]) || !(miss_rates[i] >= 0.0) || !(miss_rates[i] <= 1.0))
            return fail(IVF_EINVAL, "point %d of the miss-rate curve is not a budget >= 0 with a rate in [0, 1]", i);
        if (i > 0 && !(budgets[i] > budgets[i - 1])) return fail(IVF_EINVAL, "budgets must increase (point %d)", i);
        if (i > 0 && miss_rates[i] > miss_rates[i - 1]) return fail(IVF_EINVAL, "miss rates must not rise with the budget (point %d)", i);
    }
    const PrefetchAmount r = plan_prefetch_amount(bandwidth, t_llm, nprobe, t_cc, budgets, miss_rates, n);
    *amount = r.amount;
    if (seconds) *seconds = r.seconds;
    if (which) *which = r.which;
    return IVF_OK;
}

extern "C" int ivf_prefetch(ivf_index* ix, const float* q_in, int32_t nq, int32_t nprobe,
                            size_t budget_bytes, uint32_t flags, ivf_prefetch_stats* stats) {
    int rc = check_query_args(ix, q_in, nq, nprobe);
    if (rc) return rc;
    if (ix->placement != IVF_PLACE_HOST) return fail(IVF_ESTATE, "ivf_prefetch needs a host-placed index");
    if (flags & ~IVF_PREFETCH_RESET) return fail(IVF_EINVAL, "unknown prefetch flags 0x%x", flags);
    nprobe = std::min(nprobe, ix->nlist);
    if ((rc = ensure_workspace(ix, nq, nprobe, 1))) return rc;
    Workspace& w = *ix->cw;
    // rank the clusters by q_in on the GPU
    if ((rc = stage_queries(ix, q_in, nq))) return rc;
    const bool was_profiling = ix->profiling;
    ix->profiling = false;
    rc = enqueue_probe(ix, w.d_q, nq, nprobe, 1);
    ix->profiling = was_profiling;
    if (rc) return rc;
    HIP_TRY(hipMemcpyAsync(w.h_probe, w.d_probe, (size_t)nq * nprobe * sizeof(int32_t), hipMemcpyDeviceToHost, ix->cs));
    HIP_TRY(hipStreamSynchronize(ix->cs));

    // The plan is made on copies of the residency mirror: it becomes the index's state only when every
    // copy and the table that describes them have been enqueued.
    std::vector<int64_t> res_off(ix->h_res_off);
    size_t buf_used = ix->buf_used;
    if (flags & IVF_PREFETCH_RESET) {
        std::fill(res_off.begin(), res_off.end(), (int64_t)-1);
        buf_used = 0;
    }
    ivf_prefetch_stats st{};
    const size_t rb = ix->row_bytes;
    std::vector<int32_t> taken;
    plan_prefetch(w.h_probe, nq, nprobe, ix->h_off.data(), rb, budget_bytes, ix->buf_bytes, buf_used, res_off.data(), taken, st);
    auto enqueue = [&]() -> int {
        HIP_TRY(hipEventRecord(ix->ev_pf_begin, ix->copy));
        for (int32_t c : taken) {
            const size_t bytes = (size_t)(ix->h_off[c + 1] - ix->h_off[c]) * rb;
            if (bytes > 0)
                HIP_TRY(hipMemcpyAsync((char*)ix->d_buf + (size_t)res_off[c] * rb,
                                       (const char*)ix->h_lists + (size_t)ix->h_off[c] * rb, bytes,
                                       hipMemcpyHostToDevice, ix->copy));
        }
        // the residency table follows the data on the same stream; the pinned staging copy is reused,
        // so the previous upload from it must have finished
        if (ix->pf_recorded) HIP_TRY(hipEventSynchronize(ix->ev_pf_table));
        memcpy(ix->h_res_stage, res_off.data(), (size_t)ix->nlist * sizeof(int64_t));
        HIP_TRY(hipMemcpyAsync(ix->d_res_off, ix->h_res_stage, (size_t)ix->nlist * sizeof(int64_t), hipMemcpyHostToDevice, ix->copy));
        HIP_TRY(hipEventRecord(ix->ev_pf_table, ix->copy));
        if (ix->cache_on)     // clusters that arrived are cached from now on; a reset drops the cache
            HIP_TRY(launch_cache_admit(ix->d_hot, ix->d_used, ix->d_res_off, ix->nlist, ix->cache_h_init,
                                       (flags & IVF_PREFETCH_RESET) ? 1 : 0, ix->copy));
        HIP_TRY(hipEventRecord(ix->ev_pf_done, ix->copy));
        return IVF_OK;
    };
    rc = enqueue();
    if (rc != IVF_OK) {
        // Some copies may be on their way into places the device table does not know, or the table may
        // be stale: nothing is resident any more, on either side (best effort for the device side).
        const std::string why = g_last_error;
        (void)hipStreamSynchronize(ix->copy);
        std::fill(ix->h_res_off.begin(), ix->h_res_off.end(), (int64_t)-1);
        ix->buf_used = 0;
        (void)hipMemcpy(ix->d_res_off, ix->h_res_off.data(), (size_t)ix->nlist * sizeof(int64_t), hipMemcpyHostToDevice);
        g_last_error = why + " (the residency was dropped)";
        return rc;
    }
    ix->h_res_off.swap(res_off);
    ix->buf_used = buf_used;
    ix->pf_recorded = true;
    st.buffer_used = ix->buf_used;
    if (stats) *stats = st;
    return IVF_OK;
}

// ---- prefetching scheduler ---------------------------------------------------------------------------
extern "C" int ivf_schedule(ivf_index* ix, const float* q, int32_t nq, int32_t micro, int32_t* order, float* ms_gpu) {
    if (!ix || !q || !order) return fail(IVF_EINVAL, "index, q or order is NULL");
    if (nq < 1 || micro < 1) return fail(IVF_EINVAL, "nq and micro must be at least 1");
    if (nq > kScheduleMaxQueries) return fail(IVF_ELIMIT, "at most %d queries per global batch", kScheduleMaxQueries);
    int rc = settle_on_lane0(ix);
    if (rc) return rc;
    float* d_q = nullptr; double* d_dist = nullptr; int32_t* d_order = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    auto cleanup = [&]() {
        dfree(d_q); dfree(d_dist); dfree(d_order);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    };
#define SCHED_TRY(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { cleanup(); return fail(IVF_EHIP, "%s: %s", #call, hipGetErrorString(e_)); } } while (0)
    SCHED_TRY(hipMalloc(&d_q, (size_t)nq * ix->d * sizeof(float)));
    SCHED_TRY(hipMalloc(&d_dist, (size_t)nq * nq * sizeof(double)));
    SCHED_TRY(hipMalloc(&d_order, (size_t)nq * sizeof(int32_t)));
    SCHED_TRY(hipEventCreate(&e0));
    SCHED_TRY(hipEventCreate(&e1));
    SCHED_TRY(hipMemcpyAsync(d_q, q, (size_t)nq * ix->d * sizeof(float), hipMemcpyHostToDevice, ix->cs));
    SCHED_TRY(hipEventRecord(e0, ix->cs));
    SCHED_TRY(launch_schedule(d_q, nq, ix->d, micro, d_dist, d_order, ix->cs));
    SCHED_TRY(hipEventRecord(e1, ix->cs));
    SCHED_TRY(hipMemcpyAsync(order, d_order, (size_t)nq * sizeof(int32_t), hipMemcpyDeviceToHost, ix->cs));
    SCHED_TRY(hipStreamSynchronize(ix->cs));
    if (ms_gpu) SCHED_TRY(hipEventElapsedTime(ms_gpu, e0, e1));
#undef SCHED_TRY
    cleanup();
    return IVF_OK;
}

// ---- cluster cache -------------------------------------------------------------------------------------
extern "C" int ivf_cache_configure(ivf_index* ix, float fraction, float h_init, float decay, float h_inc) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    if (ix->placement != IVF_PLACE_HOST) return fail(IVF_ESTATE, "the cluster cache needs a host-placed index");
    if (fraction < 0.f) { ix->cache_on = false; return IVF_OK; }
    if (!(fraction <= 1.f) || !(h_init >= 0.f) || !(decay >= 1.f) || !(h_inc >= 0.f))
        return fail(IVF_EINVAL, "cache parameters: fraction in [0, 1], h_init >= 0, decay >= 1, h_inc >= 0");
    int rc = settle_on_lane0(ix);
    if (rc) return rc;
    if (!ix->d_hot) {
        HIP_TRY(hipMalloc(&ix->d_hot, (size_t)ix->nlist * sizeof(float)));
        HIP_TRY(hipMalloc(&ix->d_used, (size_t)ix->nlist * sizeof(uint32_t)));
        for (auto& e : ix->ev_cache) HIP_TRY(hipEventCreate(&e));
        HIP_TRY(hipEventCreateWithFlags(&ix->ev_round, hipEventDisableTiming));
        HIP_TRY(hipHostMalloc(&ix->h_hot_stage, (size_t)ix->nlist * sizeof(float)));
    }
    ix->cache_fraction = fraction; ix->cache_h_init = h_init; ix->cache_decay = decay; ix->cache_h_inc = h_inc;
    // what is resident now becomes cached at h_init; nothing has been used yet
    if (ix->pf_recorded) HIP_TRY(hipStreamWaitEvent(ix->cs, ix->ev_pf_done, 0));
    HIP_TRY(launch_cache_admit(ix->d_hot, ix->d_used, ix->d_res_off, ix->nlist, h_init, 1, ix->cs));
    HIP_TRY(hipStreamSynchronize(ix->cs));
    ix->cache_on = true;
    return IVF_OK;
}

extern "C" int ivf_cache_hotness(ivf_index* ix, float* hotness) {
    if (!ix || !hotness) return fail(IVF_EINVAL, "index or hotness is NULL");
    if (!ix->cache_on) return fail(IVF_ESTATE, "the cluster cache is not configured");
    int rc = settle_on_lane0(ix);
    if (rc) return rc;
    if (ix->pf_recorded) HIP_TRY(hipEventSynchronize(ix->ev_pf_done));
    HIP_TRY(hipStreamSynchronize(ix->cs));
    HIP_TRY(hipMemcpy(hotness, ix->d_hot, (size_t)ix->nlist * sizeof(float), hipMemcpyDeviceToHost));
    return IVF_OK;
}

extern "C" int ivf_cache_plan(float* hotness, const int64_t* offsets, int32_t nlist, size_t row_bytes,
                              int64_t* resident_off, size_t* buffer_used, size_t buffer_bytes, float fraction,
                              int32_t* evicted, int32_t* n_evicted, ivf_cache_move* moves, int32_t* n_moves) {
    if (!hotness || !offsets || !resident_off || !buffer_used || !evicted || !n_evicted || !moves || !n_moves)
        return fail(IVF_EINVAL, "NULL argument");
    if (nlist < 1 || row_bytes < 1) return fail(IVF_EINVAL, "nlist and row_bytes must be at least 1");
    if (!(fraction >= 0.f && fraction <= 1.f)) return fail(IVF_EINVAL, "fraction must be in [0, 1]");
    std::vector<int32_t> ev;
    std::vector<ivf_cache_move> mv;
    size_t need_tmp = 0;
    ivf_cache_stats st{};
    plan_cache_round(hotness, offsets, nlist, row_bytes, resident_off, *buffer_used, buffer_bytes, fraction, ev, mv, need_tmp, st);
    std::copy(ev.begin(), ev.end(), evicted);
    std::copy(mv.begin(), mv.end(), moves);
    *n_evicted = (int32_t)ev.size();
    *n_moves = (int32_t)mv.size();
    return IVF_OK;
}

extern "C" int ivf_cache_end_round(ivf_index* ix, ivf_cache_stats* stats) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    if (!ix->cache_on) return fail(IVF_ESTATE, "the cluster cache is not configured");
    int rc = settle_on_lane0(ix);
    if (rc) return rc;
    const int nlist = ix->nlist;
    const size_t rb = ix->row_bytes;
    ivf_cache_stats st{};
    // 1. hotness update on the device, after every copy and search of the round
    if (ix->pf_recorded) HIP_TRY(hipStreamWaitEvent(ix->cs, ix->ev_pf_done, 0));
    HIP_TRY(hipEventRecord(ix->ev_cache[0], ix->cs));
    HIP_TRY(launch_cache_round(ix->d_hot, ix->d_used, nlist, ix->cache_decay, ix->cache_h_inc, ix->cs));
    std::vector<float> hot((size_t)nlist);
    HIP_TRY(hipMemcpyAsync(hot.data(), ix->d_hot, (size_t)nlist * sizeof(float), hipMemcpyDeviceToHost, ix->cs));
    HIP_TRY(hipEventRecord(ix->ev_cache[1], ix->cs));
    HIP_TRY(hipStreamSynchronize(ix->cs));
    // 2. eviction and 3. consolidation: planned on the host, carried out on the copy stream by one
    //    kernel per group of moves that do not disturb each other (no destination of the group
    //    overlaps a source of the group; the moves all go towards lower addresses, so a group ends
    //    where the next destination would reach the group's first source).  A cluster that overlaps
    //    its own old place goes through the staging area.  The next prefetch and the next search
    //    are ordered behind the moves by the copy stream and its event.
    std::vector<int32_t> evicted;
    std::vector<ivf_cache_move> moves;
    size_t need_tmp = 0;
    const std::vector<int64_t> before(ix->h_res_off);
    plan_cache_round(hot.data(), ix->h_off.data(), nlist, rb, ix->h_res_off.data(), ix->buf_used, ix->buf_bytes,
                     ix->cache_fraction, evicted, moves, need_tmp, st);
    const bool changed = before != ix->h_res_off;        // evictions and moves both show in the table
    if (need_tmp > ix->move_tmp_bytes) {
        HIP_TRY(hipDeviceSynchronize());
        if (ix->d_move_tmp) HIP_TRY(hipFree(ix->d_move_tmp));
        ix->d_move_tmp = nullptr; ix->move_tmp_bytes = 0;
        HIP_TRY(hipMalloc(&ix->d_move_tmp, need_tmp));
        ix->move_tmp_bytes = need_tmp;
    }
    if (moves.size() + 1 > ix->moves_cap) {
        HIP_TRY(hipDeviceSynchronize());
        hfree(ix->h_moves); dfree(ix->d_moves);
        ix->h_moves = nullptr; ix->d_moves = nullptr; ix->moves_cap = 0;
        const size_t cap = std::max<size_t>(moves.size() + 1, (size_t)nlist + 1);
        HIP_TRY(hipHostMalloc(&ix->h_moves, cap * sizeof(MoveDesc)));
        HIP_TRY(hipMalloc(&ix->d_moves, cap * sizeof(MoveDesc)));
        ix->moves_cap = cap;
    } else if (ix->pf_recorded) {
        HIP_TRY(hipEventSynchronize(ix->ev_pf_done));     // the previous round's upload of the list is done
    }
    HIP_TRY(hipEventRecord(ix->ev_round, ix->cs));
    HIP_TRY(hipStreamWaitEvent(ix->copy, ix->ev_round, 0));
    HIP_TRY(hipEventRecord(ix->ev_cache[2], ix->copy));
    const std::vector<MoveGroup> groups = group_moves(moves);
    std::vector<uint32_t> group_chunks(groups.size(), 0u);
    for (size_t gi = 0; gi < groups.size(); ++gi) {
        if (groups[gi].through_staging) continue;
        uint32_t chunks = 0;
        for (size_t m = groups[gi].first; m < groups[gi].last; ++m) {
            ix->h_moves[m] = MoveDesc{moves[m].from_byte, moves[m].to_byte, moves[m].bytes, chunks, 0u};
            chunks += move_chunks(moves[m].bytes);
        }
        group_chunks[gi] = chunks;
    }
    if (!moves.empty())
        HIP_TRY(hipMemcpyAsync(ix->d_moves, ix->h_moves, moves.size() * sizeof(MoveDesc), hipMemcpyHostToDevice, ix->copy));
    for (size_t gi = 0; gi < groups.size(); ++gi) {
        const MoveGroup& g = groups[gi];
        if (g.through_staging) {
            const ivf_cache_move& m = moves[g.first];
            HIP_TRY(hipMemcpyAsync(ix->d_move_tmp, (const char*)ix->d_buf + m.from_byte, m.bytes, hipMemcpyDeviceToDevice, ix->copy));
            HIP_TRY(hipMemcpyAsync((char*)ix->d_buf + m.to_byte, ix->d_move_tmp, m.bytes, hipMemcpyDeviceToDevice, ix->copy));
        } else {
            HIP_TRY(launch_gather_moves(ix->d_buf, ix->d_moves + g.first, (int)(g.last - g.first), group_chunks[gi], ix->n_cu, ix->copy));
        }
        st.n_launches += 1;
    }
    HIP_TRY(hipEventRecord(ix->ev_cache[3], ix->copy));
    if (changed) {
        if (ix->pf_recorded) HIP_TRY(hipEventSynchronize(ix->ev_pf_table));    // the staging copy of the table is free again
        memcpy(ix->h_res_stage, ix->h_res_off.data(), (size_t)nlist * sizeof(int64_t));
        memcpy(ix->h_hot_stage, hot.data(), (size_t)nlist * sizeof(float));
        HIP_TRY(hipMemcpyAsync(ix->d_res_off, ix->h_res_stage, (size_t)nlist * sizeof(int64_t), hipMemcpyHostToDevice, ix->copy));
        HIP_TRY(hipMemcpyAsync(ix->d_hot, ix->h_hot_stage, (size_t)nlist * sizeof(float), hipMemcpyHostToDevice, ix->copy));
        HIP_TRY(hipEventRecord(ix->ev_pf_table, ix->copy));
    }
    HIP_TRY(hipEventRecord(ix->ev_pf_done, ix->copy));
    ix->pf_recorded = true;
    st.bytes_kept = ix->buf_used;
    HIP_TRY(hipEventElapsedTime(&st.ms_update, ix->ev_cache[0], ix->ev_cache[1]));
    if (stats) {
        // the time of the moves is known when they are done: asking for the numbers waits for them
        HIP_TRY(hipEventSynchronize(ix->ev_cache[3]));
        HIP_TRY(hipEventElapsedTime(&st.ms_compact, ix->ev_cache[2], ix->ev_cache[3]));
        *stats = st;
    }
    return IVF_OK;
}

extern "C" int ivf_prefetch_wait(ivf_index* ix, float* ms) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    if (ix->placement != IVF_PLACE_HOST) return fail(IVF_ESTATE, "not a host-placed index");
    if (ms) *ms = 0.f;
    if (!ix->pf_recorded) return IVF_OK;
    HIP_TRY(hipEventSynchronize(ix->ev_pf_done));
    if (ms) HIP_TRY(hipEventElapsedTime(ms, ix->ev_pf_begin, ix->ev_pf_done));
    return IVF_OK;
}

// ---- stage-level entry points ----------------------------------------------------------------------
extern "C" int ivf_coarse_scores(ivf_index* ix, const float* q, int32_t nq, double* scores) {
    int rc = check_query_args(ix, q, nq, 1);
    if (rc) return rc;
    if (!scores) return fail(IVF_EINVAL, "scores is NULL");
    if ((rc = settle_on_lane0(ix))) return rc;
    if ((rc = ensure_workspace(ix, nq, 1, 1))) return rc;
    Workspace& w = *ix->cw;
    if ((rc = stage_queries(ix, q, nq))) return rc;
    CoarseArgs ca{ix->d_centroids, w.d_q, w.d_scores, ix->nlist, ix->d, nq, ix->metric};
    HIP_TRY(launch_coarse(ca, ix->cs));
    HIP_TRY(hipStreamSynchronize(ix->cs));
    HIP_TRY(hipMemcpy(scores, w.d_scores, (size_t)nq * ix->nlist * sizeof(double), hipMemcpyDeviceToHost));
    return IVF_OK;
}

extern "C" int ivf_probe(ivf_index* ix, const float* q, int32_t nq, int32_t nprobe, int32_t* clusters) {
    int rc = check_query_args(ix, q, nq, nprobe);
    if (rc) return rc;
    if (!clusters) return fail(IVF_EINVAL, "clusters is NULL");
    nprobe = std::min(nprobe, ix->nlist);
    if ((rc = settle_on_lane0(ix))) return rc;
    if ((rc = ensure_workspace(ix, nq, nprobe, 1))) return rc;
    Workspace& w = *ix->cw;
    if ((rc = stage_queries(ix, q, nq))) return rc;
    const bool was_profiling = ix->profiling;
    ix->profiling = false;
    rc = enqueue_probe(ix, w.d_q, nq, nprobe, 1);
    ix->profiling = was_profiling;
    if (rc) return rc;
    HIP_TRY(hipMemcpyAsync(w.h_probe, w.d_probe, (size_t)nq * nprobe * sizeof(int32_t), hipMemcpyDeviceToHost, ix->cs));
    HIP_TRY(hipStreamSynchronize(ix->cs));
    memcpy(clusters, w.h_probe, (size_t)nq * nprobe * sizeof(int32_t));
    return IVF_OK;
}

extern "C" int ivf_batched_scores(ivf_index* ix, const float* q, int32_t nq, int32_t cluster, float* scores, float* eps) {
    int rc = check_query_args(ix, q, nq, 1);
    if (rc) return rc;
    if (!scores || !eps) return fail(IVF_EINVAL, "scores or eps is NULL");
    if (cluster < 0 || cluster >= ix->nlist) return fail(IVF_EINVAL, "cluster %d is outside [0, %d)", cluster, ix->nlist);
    if (nq > 32) return fail(IVF_ELIMIT, "at most 32 queries (one group of the list-major scan)");
    const int saved_mode = ix->batch_mode;
    ix->batch_mode = 2;
    const bool ok = batched_eligible(ix, 2);
    ix->batch_mode = saved_mode;
    if (!ok) return fail(IVF_ESTATE, "this index has no list-major scan (needs all rows in HBM, fewer than 2^32 of them, and d a multiple of 64 that fits LDS)");
    const int64_t n_c = ix->h_off[cluster + 1] - ix->h_off[cluster];
    if (n_c > kCandCap) return fail(IVF_ELIMIT, "the cluster has %lld rows, at most %d can be returned", (long long)n_c, kCandCap);
    if ((rc = settle_on_lane0(ix))) return rc;
    if ((rc = ensure_workspace(ix, nq, 1, 1))) return rc;
    if ((rc = ensure_batched_workspace(ix, nq, 1))) return rc;
    Workspace& w = *ix->cw;
    if ((rc = stage_queries(ix, q, nq))) return rc;
    // every query "selects" the one cluster
    std::vector<int32_t> probe((size_t)nq, cluster);
    HIP_TRY(hipMemcpyAsync(w.d_probe, probe.data(), (size_t)nq * sizeof(int32_t), hipMemcpyHostToDevice, ix->cs));
    HIP_TRY(hipStreamSynchronize(ix->cs));
    if (ix->batched_grid == 0) ix->batched_grid = batched_resident_grid(ix->dtype, ix->metric, ix->d, ix->n_cu);
    BatchedArgs b{};
    fill_batched_args(ix, w, b);
    b.q = w.d_q; b.out_ids = w.d_out_ids; b.out_dists = w.d_out_dists;
    b.nq = nq; b.nprobe = 1; b.k = 1; b.kprime = kprime_for(1); b.keep_all = 1;
    HIP_TRY(launch_batched(b, ix->batched_grid, ix->cs, nullptr, nullptr, false));
    HIP_TRY(hipStreamSynchronize(ix->cs));
    std::vector<uint32_t> count((size_t)nq), rows((size_t)n_c);
    std::vector<float> sc((size_t)n_c);
    HIP_TRY(hipMemcpy(count.data(), w.d_cand_count, (size_t)nq * sizeof(uint32_t), hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(eps, w.d_eps, (size_t)nq * sizeof(float), hipMemcpyDeviceToHost));
    for (int qi = 0; qi < nq; ++qi) {
        if ((int64_t)count[qi] != n_c) return fail(IVF_ESTATE, "query %d: %u of %lld rows came back", qi, count[qi], (long long)n_c);
        HIP_TRY(hipMemcpy(rows.data(), w.d_cand_row + (size_t)qi * kCandCap, (size_t)n_c * sizeof(uint32_t), hipMemcpyDeviceToHost));
        HIP_TRY(hipMemcpy(sc.data(), w.d_cand_score + (size_t)qi * kCandCap, (size_t)n_c * sizeof(float), hipMemcpyDeviceToHost));
        for (int64_t i = 0; i < n_c; ++i) scores[(size_t)qi * n_c + (rows[i] - (uint32_t)ix->h_off[cluster])] = sc[i];
    }
    return IVF_OK;
}

extern "C" int ivf_resident(ivf_index* ix, int32_t* clusters, int32_t* n) {
    if (!ix || !n) return fail(IVF_EINVAL, "index or n is NULL");
    int32_t cap = *n, cnt = 0;
    for (int c = 0; c < ix->nlist; ++c) {
        if (ix->h_res_off[c] < 0) continue;
        if (clusters && cnt < cap) clusters[cnt] = c;
        ++cnt;
    }
    *n = cnt;
    return IVF_OK;
}

extern "C" int ivf_get_layout(ivf_index* ix, int64_t* offsets, int64_t* ids) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    if (offsets) memcpy(offsets, ix->h_off.data(), (size_t)(ix->nlist + 1) * sizeof(int64_t));
    if (ids) {
        if (ix->h_ids.empty()) for (int64_t i = 0; i < ix->n; ++i) ids[i] = i;
        else memcpy(ids, ix->h_ids.data(), (size_t)ix->n * sizeof(int64_t));
    }
    return IVF_OK;
}

// ---- profiling ------------------------------------------------------------------------------------
extern "C" int ivf_profile_enable(ivf_index* ix, int on) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    if (on && ix->prof_sets.empty()) {
        ix->prof_sets.resize(kProfileRing);
        for (auto& s : ix->prof_sets) for (auto& e : s.e) HIP_TRY(hipEventCreate(&e));
    }
    if (!on) { int rc = drain_profile(ix); if (rc) return rc; }
    ix->profiling = on != 0;
    return IVF_OK;
}

extern "C" int ivf_profile_read(ivf_index* ix, ivf_profile* out) {
    if (!ix || !out) return fail(IVF_EINVAL, "index or out is NULL");
    int rc = drain_profile(ix);
    if (rc) return rc;
    *out = ix->prof;
    return IVF_OK;
}

extern "C" int ivf_profile_reset(ivf_index* ix) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    int rc = drain_profile(ix);
    if (rc) return rc;
    ix->prof = ivf_profile{};
    HIP_TRY(hipMemset(ix->d_prof_rows, 0, sizeof(unsigned long long)));
    HIP_TRY(hipDeviceSynchronize());
    return IVF_OK;
}

extern "C" int32_t ivf_host_scan_capacity(int32_t k) {
    return k >= 1 && k <= IVF_MAX_K ? kprime_for(k) : 0;
}

extern "C" int ivf_host_scan(const void* lists, const int64_t* offsets, const int64_t* ids, int32_t d, int dtype,
                             int metric, const float* q, const int32_t* clusters, int32_t n_clusters, int32_t k,
                             int32_t threads, int64_t* out_ids, double* out_scores, int32_t* n_out) {
    if (!lists || !offsets || !q || !out_ids || !out_scores || !n_out) return fail(IVF_EINVAL, "NULL argument");
    if (n_clusters > 0 && !clusters) return fail(IVF_EINVAL, "clusters is NULL");
    if (d < 1 || n_clusters < 0 || threads < 1 || threads > 256) return fail(IVF_EINVAL, "bad size (d %d, clusters %d, threads %d)", d, n_clusters, threads);
    if (dtype < IVF_F32 || dtype > IVF_BF16) return fail(IVF_EINVAL, "unknown dtype %d", dtype);
    if (metric != IVF_IP && metric != IVF_L2) return fail(IVF_EINVAL, "unknown metric %d", metric);
    if (k < 1) return fail(IVF_EINVAL, "k must be at least 1 (got %d)", k);
    if (k > IVF_MAX_K) return fail(IVF_ELIMIT, "k = %d is above IVF_MAX_K = %d", k, IVF_MAX_K);
    const int kprime = kprime_for(k);
    ThreadPool pool(threads);
    std::vector<HostCand> cand((size_t)kprime);
    HostScanArgs ha{lists, offsets, ids, d, dtype, metric, q, clusters, n_clusters, kprime, k, 0.f};
    const int n = host_scan_query(ha, pool, cand.data(), nullptr);
    for (int i = 0; i < n; ++i) {
        out_ids[i] = cand[i].id;
        out_scores[i] = metric == IVF_IP ? cand[i].key : -cand[i].key;
    }
    *n_out = n;
    return IVF_OK;
}

extern "C" int ivf_set_host_threads(ivf_index* ix, int32_t n) {
    if (!ix) return fail(IVF_EINVAL, "index is NULL");
    if (n < 1 || n > 256) return fail(IVF_EINVAL, "thread count must be in [1, 256]");
    if (ix->placement != IVF_PLACE_HOST) return fail(IVF_ESTATE, "not a host-placed index");
    ix->pool.reset(new ThreadPool(n));
    return IVF_OK;
}
