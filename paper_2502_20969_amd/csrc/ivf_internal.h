// Internal declarations shared by the host side (ivf_api.hip) and the kernel launchers
// (ivf_kernels.hip).  Not part of the public boundary (include/ivf.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ivf_host_types.h"

namespace ivf {

constexpr uint32_t kNoRow = 0xFFFFFFFFu;   // empty slot of a candidate list
constexpr int kMaxKPrime = 128;            // candidates kept per list: k + slack <= 128
constexpr int kScanWaves = 4;              // scan workgroup: 4 wavefronts, two workgroups per compute unit
constexpr int kScanThreads = kScanWaves * 64;
constexpr int kLaneTableSlots = 64;        // up to this many selected clusters the scan keeps the slot table in its lanes
constexpr int kScanBatches = 1;           // batches of rows a scan wavefront has in flight (measured: one small batch beats two larger ones)
constexpr int kScanMaxWgPerCu = 2;        // scan workgroups per compute unit at most (sizes the per-workgroup tables)
constexpr int kSelectThreads = 1024;       // select / merge workgroup: 16 wavefronts
constexpr int kSortLdsCap = 2048;          // select: pairs sorted in LDS up to this many
constexpr int kPrefixLdsCap = 8192;        // select: row-prefix table kept in LDS up to this nprobe

// candidates re-scored in fp64 per query: the requested k plus a margin that absorbs the
// rounding of the fp32 scan
// entries of one wavefront's candidate list: its loose candidates (up to 64) or its sorted list
inline int cand_slots(int kprime) { return kprime > 64 ? 128 : 64; }

inline int kprime_for(int k) {
    int slack = k / 8 > 8 ? k / 8 : 8;
    int kp = k + slack;
    return kp > kMaxKPrime ? kMaxKPrime : kp;
}

// How one scan kernel variant walks rows: a batch is up to `rows_per_batch` consecutive rows
// of one list; kScanBatches batches are in flight per wavefront.
struct ScanShape {
    int lanes_per_row;   // 16, 32 or 64; 0 selects the any-d fallback kernel
    int segments;        // 16-byte loads per lane per row
    int unroll;          // row groups per batch
    int rows_per_batch;
};
ScanShape pick_scan_shape(int d, int dtype);

// Per query and selected cluster ("slot", nearest first), written by the select kernel.
struct SlotTables {
    int64_t* base;           // [nq x nprobe]   row offset of the list in the device buffer, -1 = not resident
    uint32_t* grow;          // [nq x nprobe]   global row of the list's first row
    uint32_t* nrows;         // [nq x nprobe]   rows in the list
    uint32_t* rprefix;       // [nq x (nprobe+1)] exclusive prefix of rows over the resident slots
};

// The share of one scan workgroup: rows [r_begin, r_end) of the query's concatenated resident
// rows, and the slot that holds r_begin with its table entries inlined.
struct WgDesc {
    uint32_t r_begin, r_end;
    uint32_t slot;
    uint32_t slot_rbegin;    // rprefix[slot]
    uint32_t slot_rend;      // rprefix[slot + 1]
    uint32_t slot_grow;
    int64_t slot_base;
};

// Every launcher takes optional events that receive the kernel's own begin and end time.
struct CoarseArgs {
    const float* centroids; const float* q; double* scores;
    int nlist, d, nq, metric;
};
hipError_t launch_coarse(const CoarseArgs& a, hipStream_t s, hipEvent_t start = nullptr, hipEvent_t stop = nullptr);

struct SelectArgs {
    const double* scores;    // [nq x nlist]
    int32_t* probe;          // [nq x nprobe] out, nearest first
    const int64_t* off;      // [nlist+1]
    const int64_t* res_off;  // [nlist] row offset in the device buffer or -1
    SlotTables slots;
    WgDesc* desc;            // [nq x grid] out
    uint64_t* sort_keys;     // global scratch [nq x pad] when the sort does not fit LDS
    uint32_t* sort_idx;
    unsigned long long* rows_counter;  // nullable: receives the rows of all resident selected lists
    uint32_t* used;          // nullable [nlist]: set to 1 for every selected cluster that is resident
    int nlist, nprobe, nq, metric, grid;
};
hipError_t launch_select(const SelectArgs& a, hipStream_t s, hipEvent_t start = nullptr, hipEvent_t stop = nullptr);

struct ScanArgs {
    const void* buf;         // device buffer holding resident lists, row-major
    const float* q;          // [nq x d]
    SlotTables slots;
    const WgDesc* desc;      // [nq x grid]
    uint64_t* part;          // [nq x (grid x kScanWaves) x cand_slots(kprime)] out: one list of packed candidates
                             // (fp32 key image << 32 | ~global row) per wavefront, unordered, 0 = empty
    uint64_t* heads;         // [nq x (grid x kScanWaves)] out: the best entry of every list, packed densely for the merge
    int d, dtype, metric, nprobe, nq, kprime, grid;
    ScanShape shape;
};
hipError_t launch_scan(const ScanArgs& a, hipStream_t s, hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
// workgroups of the scan kernel for (shape, dtype, metric, kprime) that are resident at once
int scan_resident_grid(const ScanShape& shape, int dtype, int metric, int kprime, int d, int n_cu);

struct MergeArgs {
    const void* buf; const float* q;
    const int64_t* ids;          // [n] global row -> id, or nullptr (id = global row)
    SlotTables slots;
    const uint64_t* part;        // [nq x nparts x slots] packed candidates written by the scan, lists unordered
    const uint64_t* heads;       // [nq x nparts] the lists' best entries
    const HostCand* host_cand;   // [nq x kprime] device-visible, or nullptr
    const int32_t* host_count;   // [nq] valid entries in host_cand
    int64_t* out_ids; float* out_dists;   // [nq x k]
    int d, dtype, metric, nprobe, nq, k, kprime, nparts, list_len;   // list_len: entries per list
    int identity;            // 1: buffer row == global row (device placement)
    // Completion word in pinned host memory (device address) or nullptr: set to done_value after
    // the results are visible to the host.  Only for nq == 1 (one workgroup writes it).
    unsigned long long* done; unsigned long long done_value;
    // The proof that no dropped row belongs to the k nearest (merge_kernel, step 5): bound of the
    // scan's fp32 rounding and the largest row norm of the lists; redo_flag[qi] (nullable) receives 1
    // when the proof fails, with the k-th best score found in redo_thr[qi] and the counter of the
    // exact second pass zeroed; host_flag (nullable, pinned) receives the same flag for the host.
    float err_coef, row_norm_max;
    uint32_t* redo_flag; double* redo_thr; uint32_t* redo_ticket;
    uint32_t* host_flag;
};
hipError_t launch_merge(const MergeArgs& a, hipStream_t s, hipEvent_t start = nullptr, hipEvent_t stop = nullptr);

// The exact second pass (exact_redo_kernel) for the queries merge_kernel flagged: `grid` workgroups of
// kRedoListsPerWg wavefronts per query, each wavefront leaving a list of k entries.
constexpr int kRedoListsPerWg = 4;
struct RedoArgs {
    const void* buf; const float* q;
    const int64_t* ids;          // [n] global row -> id, or nullptr
    SlotTables slots;
    const uint32_t* redo_flag; const double* redo_thr; uint32_t* redo_ticket;
    unsigned long long* list_key;    // [nq x grid x kRedoListsPerWg x k] scores as ascending-order keys, 0 = empty
    long long* list_id;              // [same] the rows' ids
    const HostCand* host_cand; const int32_t* host_count;
    int64_t* out_ids; float* out_dists;
    unsigned long long* done; unsigned long long done_value;
    int d, dtype, metric, nprobe, nq, k, kprime;
};
hipError_t launch_redo(const RedoArgs& a, int grid, hipStream_t s);
// bound coefficient of the scan's fp32 rounding for (shape, d, metric): see result_is_safe
float scan_error_coef(const ScanShape& shape, int d, int dtype, int metric);

// One move of the buffer consolidation: bytes from from_byte to to_byte of the buffer; chunk0 = number of
// the move's first chunk in its launch (move_chunks(bytes) chunks per move, numbered through the launch).
struct MoveDesc { uint64_t from_byte, to_byte, bytes; uint32_t chunk0, pad; };
uint32_t move_chunks(uint64_t bytes);
// one launch for a group of moves that do not disturb each other; moves_dev holds n_moves entries
hipError_t launch_gather_moves(void* buf, const MoveDesc* moves_dev, int n_moves, uint32_t n_chunks, int n_cu, hipStream_t s);

// cluster cache bookkeeping: hot[c] < 0 = not cached
hipError_t launch_cache_admit(float* hot, uint32_t* used, const int64_t* res_off, int nlist, float h_init, int reset,
                              hipStream_t s);
hipError_t launch_cache_round(float* hot, uint32_t* used, int nlist, float decay, float h_inc, hipStream_t s);

// prefetching scheduler (ivf_sched.hip): pairwise squared L2 distances [B x B] and the greedy grouping
hipError_t launch_schedule(const float* q_dev, int B, int d, int m, double* dist, int32_t* order, hipStream_t s);
constexpr int kScheduleMaxQueries = 4096;

// ---- batched (list-major) search: ivf_batched.hip ------------------------------------------------
struct BatchTask { uint32_t cluster, group, tile; };    // tile: 256 rows of the cluster; group: up to 32 (fp32 rows: 16) of the queries probing it

struct BatchedArgs {
    const void* lists;           // device lists (device placement)
    const int64_t* off;          // [nlist+1]
    const int64_t* ids;          // [n] or nullptr
    const float* q;              // [nq x d] fp32 queries
    const int32_t* probe;        // [nq x nprobe] selected clusters
    void* q_store;               // [nq x d] queries rounded to the storage type (out)
    float* thr;                  // [nq] out: filter threshold
    float* thr_part;             // [batched_thr_part_floats(nq)] best sample keys per (query, part)
    const unsigned int* row_norm_max_bits;   // largest squared row norm of the lists, as float bits
    uint32_t* list_count;        // [nlist] queries probing each cluster
    uint32_t* cursor;            // [nlist]
    uint32_t* qstart;            // [nlist+1] prefix of list_count
    uint32_t* tstart;            // [nlist+1] prefix of tasks per cluster
    uint32_t* qidx;              // [nq x nprobe] queries grouped by cluster
    BatchTask* tasks;            // [task capacity]
    uint32_t* ticket;            // one counter, zero when the scan starts: the tasks handed out so far
    uint32_t* cand_count;        // [nq]
    uint32_t* cand_row;          // [nq x cand_cap] global rows that passed the filter
    float* cand_score;           // [nq x cand_cap] their approximate (MFMA) scores
    float* eps;                  // [nq] bound of |approximate - exact| score
    float* qq;                   // [nq] squared norms of the queries
    const float* row_norm;       // [n] squared norms of the rows (L2 only)
    uint32_t* surv_row;          // [nq x surv_cap] rows that survive the pruning by approximate score
    uint64_t* cand_key;          // [nq x surv_cap] fp64 re-scores as ascending keys
    int32_t* overflow;           // [nq] 1 when a query had more candidates than cand_cap
    int64_t* out_ids; float* out_dists;      // [nq x k]
    unsigned long long* rows_counter;        // nullable: rows covered by the scan tasks (profiling)
    int nlist, d, dtype, metric, nq, nprobe, k, kprime, cand_cap, surv_cap;
    int group_q;                 // queries per task: batched_group_q(dtype)
    float acc_coef;              // fp32 accumulation of the MFMA: |error| <= acc_coef |q| |y|
    float samp_coef;             // batched_sample_coef(d, dtype, metric)
    int keep_all;                // 1: the threshold is -inf, every scanned row becomes a candidate (stage-level test entry)
};
// upper bound of the number of tasks for a batch of nq queries
uint64_t batched_task_bound(const int64_t* off_host, int nlist, int nq, int dtype);
// squared row norms (fp64 sums rounded to fp32): the largest as float bits, all of them when out_norm is not null
hipError_t launch_row_norms(const void* lists, int dtype, int64_t n, int d, unsigned int* out_bits, float* out_norm, hipStream_t s);
int batched_group_q(int dtype);
float batched_sample_coef(int d, int dtype, int metric);
// with_merge = false stops after the scan: the candidate lists hold what passed the filter
hipError_t launch_batched(const BatchedArgs& a, int grid, hipStream_t s, hipEvent_t scan_start = nullptr,
                          hipEvent_t scan_stop = nullptr, bool with_merge = true);
int batched_resident_grid(int dtype, int metric, int d, int n_cu);
size_t batched_thr_part_floats(int nq);
size_t batched_scan_lds(int d, int dtype);      // LDS bytes of the batched scan kernel (one group of queries)

// scatters n rows to their cluster-major positions: dst[pos[i]] = src[i] (row_bytes each)
// n floats from a pinned host buffer (its device address) to device memory, by a kernel
hipError_t launch_stage_query(const float* src_pinned, float* dst, size_t n, hipStream_t s);
hipError_t launch_scatter_rows(const void* src, void* dst, const int64_t* pos, int64_t n,
                               size_t row_bytes, hipStream_t s);

uint32_t select_sort_pad(int nlist, int nprobe);

}  // namespace ivf
