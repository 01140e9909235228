// Batched list scan for query batches that share probed clusters (TeleRAG Sec. 4.2 "Batching":
// the GPU part of the search becomes a matrix-matrix product).  Each selected list is read from
// HBM once per group of queries that probe it (up to 32 for fp16 / bf16 rows, up to 16 for fp32
// rows); scores come from MFMA (v_mfma_f32_32x32x16 f16 / bf16 or v_mfma_f32_16x16x4 f32, fp32
// accumulate) and are only used to FILTER rows: a row whose approximate score reaches the query's
// threshold becomes a candidate, and the final ranking is done on fp64 re-scores with the fp32
// query, exactly as in the single-query path.
//
// Scores are "larger is better": <q, y> for the inner product, -|q - y|^2 for squared L2.  The
// MFMA always computes <q, y>; for L2 the filter score is 2 <q, y> - |y|^2 - |q|^2 with |y|^2
// from a table of row norms made when the index is built.
//
// Threshold of a query: the k-th best fp32 score over a sample of its nearest cluster (a lower
// bound of its k-th best score over all selected clusters), lowered by a bound eps on the error
// of the filter score (query rounded to the storage type, fp32 accumulation, rounded norms).
// Every true top-k row passes this filter.
#include "ivf_device.h"
#include <hip/hip_ext.h>

namespace ivf {
using namespace dev;

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kBatchWaves = 8;      // wavefronts of a batched scan workgroup
constexpr int kBatchThreads = kBatchWaves * 64;
constexpr int kTileRows = kBatchWaves * 32;     // rows per task: 32 per wavefront
constexpr int kStageLd = 64 + 8;   // elements per row of a wavefront's staging area: 64 + padding
constexpr int kGroupQ = 32;        // queries per task: one MFMA tile wide
constexpr int kQPad = 8;           // padding (elements) of a staged query row in LDS
constexpr int kStage16 = 2;        // 64-element blocks of a row per pipeline stage (fp16 / bf16 rows)

// ---- row norms of the lists (one-time, at build) ---------------------------------------------------
// Squared norms summed in fp64 and rounded once to fp32; the largest goes to out_bits, all of
// them to out_norm when that is not null.
__global__ void row_norm_kernel(const void* lists, int dtype, int64_t n, int d, unsigned int* out_bits, float* out_norm) {
    const int lane = threadIdx.x & 63;
    int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    float best = 0.f;
    for (int64_t r = wave; r < n; r += nwaves) {
        double s = 0.0;
        for (int t = lane; t < d; t += 64) {
            const double x = widen(lists, dtype, (size_t)r * d + t);
            s = fma(x, x, s);
        }
        const float f = (float)wave_sum(s);
        if (out_norm && lane == 0) out_norm[r] = f;
        best = fmaxf(best, f);
    }
    if (lane == 0) atomicMax(out_bits, __float_as_uint(best));   // non-negative floats order as integers
}

hipError_t launch_row_norms(const void* lists, int dtype, int64_t n, int d, unsigned int* out_bits, float* out_norm, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 3) / 4;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(row_norm_kernel, dim3((unsigned)blocks), dim3(256), 0, s, lists, dtype, n, d, out_bits, out_norm);
    return hipGetLastError();
}

// ---- threshold sample --------------------------------------------------------------------------------------
// fp32 scores (fp32 query; <q, y>, or -sum (q - y)^2 for L2) of the first 2048 rows of each query's (at most 64 nearest) selected
// clusters, taken in probe order (usually all from the nearest cluster; more clusters when those
// are small), reduced to the k-th best.  Any subset of the selected rows gives a valid lower bound of the k-th best
// score over all of them.  The sample of a query is split over kSampleParts workgroups of 128 rows;
// each writes its k best keys, and prep_queries_kernel merges the parts.
constexpr int kSampleParts = 16;
constexpr int kSamplePartRows = 128;

template <typename T>
__global__ __launch_bounds__(256) void thr_sample_kernel(BatchedArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ Cand m_cand[3 * kMaxKPrime];
    constexpr int EPL = T::kPerLoad;
    const int qi = blockIdx.x, part = blockIdx.y, lane = lane_id(), wave = wave_id();
    float* ql = (float*)smem;
    for (int i = threadIdx.x; i < a.d; i += blockDim.x) ql[i] = a.q[(size_t)qi * a.d + i];
    __syncthreads();
    // The rows of the first 64 selected clusters laid end to end: lane i holds cluster i's first
    // row and the running total of rows up to and including it (one parallel prefix, so that
    // finding the cluster of a sample row is a ballot instead of a walk through dependent loads).
    const int32_t* pr = a.probe + (size_t)qi * a.nprobe;
    int64_t my_lo = 0;
    uint32_t my_n = 0;
    if (lane < a.nprobe) {
        const int c = pr[lane];
        my_lo = a.off[c];
        my_n = (uint32_t)(a.off[c + 1] - my_lo);
    }
    uint32_t my_end = my_n;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(my_end, o);
        if (lane >= o) my_end += up;
    }
    auto locate = [&](uint32_t r) -> int64_t {           // global row of sample row r, -1 past the last row
        const uint64_t b = __ballot(r < my_end);
        if (b == 0) return -1;
        const int i = __ffsll((long long)b) - 1;
        const uint32_t end_i = read_lane(my_end, i), n_i = read_lane(my_n, i);
        const int64_t lo_i = ((int64_t)read_lane((uint32_t)((uint64_t)my_lo >> 32), i) << 32) | read_lane((uint32_t)my_lo, i);
        return lo_i + (int64_t)(r - (end_i - n_i));
    };
    const uint32_t r_begin = part * kSamplePartRows + wave * 32;
    const uint32_t r_end = r_begin + 32;
    const int chunks = a.d / EPL;
    WaveTopK<2, false> top;                     // ties inside the sample do not matter for a bound
    top.init();
    for (uint32_t r0 = r_begin; r0 < r_end; r0 += 4) {
        int64_t g[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) g[u] = locate(r0 + u);
        if (g[0] < 0) break;                              // the selected clusters hold no more rows
        float s[4] = {0.f, 0.f, 0.f, 0.f};
        for (int ch = lane; ch < chunks; ch += 64) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t row = g[u] >= 0 ? g[u] : g[0];      // past the end: re-read a valid row
                v[u] = *(const uint4*)((const unsigned char*)a.lists + (size_t)row * a.d * T::kBytes + (size_t)ch * 16);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float x[EPL];
                Unpack<T>::run(v[u], x);
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    if (a.metric == 0) s[u] = fmaf(ql[ch * EPL + e], x[e], s[u]);
                    else { const float df = ql[ch * EPL + e] - x[e]; s[u] = fmaf(df, df, s[u]); }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float ck = read_lane(group_total_last_lane<64>(s[u]), 63);
            if (a.metric != 0) ck = -ck;
            if (g[u] >= 0 && ck >= top.thr) top.push(ck, r0 + u);
        }
        if (top.pcount > 60) top.flush(a.k);
    }
    top.flush(a.k);
    if (wave > 0) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            int e = j * 64 + lane;
            if (e < a.k) m_cand[(wave - 1) * a.k + e] = top.top[j];
        }
    }
    __syncthreads();
    if (wave == 0) {
        for (int w = 0; w < 3; ++w) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                int e = j * 64 + lane;
                top.merge_run_if_useful(e < a.k ? m_cand[w * a.k + e] : (Cand)0, a.k);
            }
        }
        float* out = a.thr_part + ((size_t)qi * kSampleParts + part) * kMaxKPrime;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            int e = j * 64 + lane;
            if (e < a.k) out[e] = top.top[j] == 0 ? -INFINITY : cand_key(top.top[j]);
        }
    }
}

// ---- queries in the storage type, thresholds ---------------------------------------------------------
__global__ void prep_queries_kernel(BatchedArgs a) {
    const int qi = blockIdx.x, lane = threadIdx.x & 63;
    const float* q = a.q + (size_t)qi * a.d;
    float s = 0.f, res = 0.f;          // |q~|^2 of the rounded query and |q~ - q|^2 of the rounding
    double qq = 0.0;                   // |q|^2
    for (int t = threadIdx.x; t < a.d; t += 64) {
        float x = q[t], xr = x;
        if (a.dtype == 1) { _Float16 h = (_Float16)x; ((_Float16*)a.q_store)[(size_t)qi * a.d + t] = h; xr = (float)h; }
        else if (a.dtype == 2) { __bf16 h = (__bf16)x; ((__bf16*)a.q_store)[(size_t)qi * a.d + t] = h; xr = (float)h; }
        s = fmaf(xr, xr, s);
        res = fmaf(xr - x, xr - x, res);
        qq = fma((double)x, (double)x, qq);
    }
    s = group_sum<64>(s);
    res = group_sum<64>(res);
    qq = wave_sum(qq);
    // k-th best key over the sample parts
    WaveTopK<2, false> top;
    top.init();
    for (int part = 0; part < kSampleParts; ++part) {
        const float* in = a.thr_part + ((size_t)qi * kSampleParts + part) * kMaxKPrime;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            int e = j * 64 + lane;
            float key = e < a.k ? in[e] : -INFINITY;
            top.merge_run_if_useful(key == -INFINITY ? (Cand)0 : pack_cand(key, (uint32_t)(part * kMaxKPrime + e)), a.k);
        }
    }
    if (lane == 0) {
        // Bound of |filter score - exact score| for any row y.  Inner product from the MFMA: the
        // query rounding contributes |<q~ - q, y>| <= |q~ - q| |y| (Cauchy-Schwarz, with the
        // residual norm measured above), the fp32 accumulation at most acc_coef |q~| |y|.  The
        // fp32 sample score behind the threshold is off by at most samp_coef |q| |y| (inner
        // product) or samp_coef |q - y|^2 (L2: every term of the sum is positive).  The L2
        // filter score 2 <q, y> - |y|^2 - |q|^2 doubles the inner-product error and adds the
        // rounding of the two norms and of its two operations, each at most 2^-24 (|q| + |y|)^2.
        // A little slack absorbs the rounding of this arithmetic itself.
        const float ymax = sqrtf(__uint_as_float(*a.row_norm_max_bits));
        const float qn = sqrtf((float)qq);
        const float ip_err = (sqrtf(res) + a.acc_coef * sqrtf(s)) * ymax;
        float eps;
        if (a.metric == 0) eps = 1.01f * (ip_err + a.samp_coef * qn * ymax);
        else eps = 1.01f * (2.f * ip_err + (a.samp_coef + 0x1p-21f) * (qn + ymax) * (qn + ymax));
        a.thr[qi] = a.keep_all ? -INFINITY : top.thr - eps;        // -inf (fewer than k sampled rows) stays -inf
        a.eps[qi] = eps;
        a.qq[qi] = (float)qq;
        a.cand_count[qi] = 0;
    }
}

// ---- cluster -> queries map and the task list ------------------------------------------------------------
__global__ void zero_u32_kernel(uint32_t* p, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

__global__ void count_pairs_kernel(BatchedArgs a) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < a.nq * a.nprobe) atomicAdd(&a.list_count[a.probe[i]], 1u);
}

// one workgroup: prefix sums over all clusters of (queries per cluster) and (tasks per cluster)
__global__ __launch_bounds__(1024) void scan_lists_kernel(BatchedArgs a) {
    __shared__ uint32_t wsum_q[17], wsum_t[17];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t carry_q = 0, carry_t = 0;
    for (int base = 0; base < a.nlist; base += 1024) {
        int c = base + tid;
        uint32_t cq = 0, ct = 0;
        if (c < a.nlist) {
            cq = a.list_count[c];
            uint32_t n = (uint32_t)(a.off[c + 1] - a.off[c]);
            ct = cq ? ((n + kTileRows - 1) / kTileRows) * ((cq + a.group_q - 1) / a.group_q) : 0;
            a.cursor[c] = 0;
        }
        uint32_t iq = cq, it = ct;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            uint32_t uq = __shfl_up(iq, o), ut = __shfl_up(it, o);
            if (lane >= o) { iq += uq; it += ut; }
        }
        if (lane == 63) { wsum_q[wave] = iq; wsum_t[wave] = it; }
        __syncthreads();
        uint32_t oq = 0, ot = 0, tq = 0, tt = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < wave) { oq += wsum_q[w]; ot += wsum_t[w]; }
            tq += wsum_q[w]; tt += wsum_t[w];
        }
        if (c < a.nlist) { a.qstart[c] = carry_q + oq + iq - cq; a.tstart[c] = carry_t + ot + it - ct; }
        carry_q += tq; carry_t += tt;
        __syncthreads();
    }
    if (tid == 0) { a.qstart[a.nlist] = carry_q; a.tstart[a.nlist] = carry_t; }
    // rows the scan covers once per cluster (for the roofline accounting)
    if (a.rows_counter) {
        unsigned long long rows = 0;
        for (int c = tid; c < a.nlist; c += 1024) if (a.list_count[c]) rows += (unsigned long long)(a.off[c + 1] - a.off[c]);
        for (int m = 32; m >= 1; m >>= 1) rows += __shfl_xor(rows, m);
        if (lane == 0 && rows) atomicAdd(a.rows_counter, rows);
    }
}

__global__ void fill_pairs_kernel(BatchedArgs a) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.nq * a.nprobe) return;
    int c = a.probe[i];
    uint32_t pos = atomicAdd(&a.cursor[c], 1u);
    a.qidx[a.qstart[c] + pos] = (uint32_t)(i / a.nprobe);
}

// tasks of cluster c, ordered (query group, row tile) so that tiles of one group are consecutive
__global__ void make_tasks_kernel(BatchedArgs a) {
    for (int c = blockIdx.x; c < a.nlist; c += gridDim.x) {
        const uint32_t t0 = a.tstart[c], t1 = a.tstart[c + 1];
        if (t0 == t1) continue;
        const uint32_t n = (uint32_t)(a.off[c + 1] - a.off[c]);
        const uint32_t tiles = (n + kTileRows - 1) / kTileRows;
        for (uint32_t i = threadIdx.x; i < t1 - t0; i += blockDim.x) {
            BatchTask t;
            t.cluster = (uint32_t)c;
            t.group = i / tiles;
            t.tile = i % tiles;
            a.tasks[t0 + i] = t;
        }
    }
}

// ---- how the scan workgroups get their tasks ---------------------------------------------------------------
// The workgroups resident on the GPU draw runs of consecutive tasks from one counter (a.ticket,
// zero at launch) until the list is used up: compute units, and whole XCDs, differ by several
// per cent in how fast they stream from HBM, and with equal shares the slowest one sets the
// kernel's time.  A run has up to kRunMax tasks (tasks that follow each other mostly share their
// cluster and group of queries, which are staged once) and shrinks towards the end of the list
// (remaining / (4 x workgroups), at least one), so that all workgroups finish within about a task
// of each other.  Every workgroup leaves once a run starts past the end of the list.
constexpr uint32_t kRunMax = 8;
struct TaskFeed {
    uint32_t t, t_stop, total;      // same in all threads: next task, end of the run, end of the list
    uint32_t ahead_t0, ahead_n;     // thread 0: the run reserved ahead
    __device__ __forceinline__ uint32_t run_length(uint32_t counter_seen) const {
        const uint32_t left = total - min(total, counter_seen);
        return max(1u, min(kRunMax, left / (4u * gridDim.x)));
    }
    __device__ __forceinline__ void reserve(const BatchedArgs& a, uint32_t counter_seen) {
        ahead_n = run_length(counter_seen);
        ahead_t0 = atomicAdd(a.ticket, ahead_n);
    }
    __device__ __forceinline__ void start(const BatchedArgs& a) {
        total = (uint32_t)__builtin_amdgcn_readfirstlane((int)a.tstart[a.nlist]);
        t = t_stop = 0;
        ahead_t0 = ahead_n = 0;
        if (threadIdx.x == 0) reserve(a, 0);
    }
    // the next task's index, or false when the list is used up; all threads of the workgroup call it together.
    // s_run: four words of LDS (16 bytes, so that the dynamic LDS area behind the static one stays 16-byte aligned)
    __device__ __forceinline__ bool next(const BatchedArgs& a, uint32_t* s_run, uint32_t& index) {
        if (t == t_stop) {
            __syncthreads();                              // s_run of the previous run has been read by everyone
            if (threadIdx.x == 0) {
                s_run[0] = ahead_t0;
                s_run[1] = min(ahead_t0 + ahead_n, total);
            }
            __syncthreads();
            // (read from LDS: the compiler is told that the values are the same in every lane, so
            // that the task and everything derived from it stay in scalar registers)
            t = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_run[0]);
            t_stop = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_run[1]);
            if (t >= total) return false;
            // the run after this one: asked for behind the barrier, so that only this wavefront
            // waits for the counter while the others are already at work
            if (threadIdx.x == 0) reserve(a, ahead_t0 + ahead_n);
        }
        index = t++;
        return true;
    }
};

// ---- the MFMA scan -------------------------------------------------------------------------------------
template <typename T> struct Mfma;
template <> struct Mfma<F16> {
    typedef half8_t frag;
    __device__ static __forceinline__ float16_t run(frag a, frag b, float16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mfma<BF16> {
    typedef bf16x8_t frag;
    __device__ static __forceinline__ float16_t run(frag a, frag b, float16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};

// One workgroup (8 wavefronts) per task: 256 rows of one cluster against up to 32 of the queries
// that probe it.  The queries (storage type) are staged in LDS once per (cluster, group).  Each
// wavefront streams its 32 rows from HBM with coalesced loads (8 lanes cover one 128-byte line of
// a row, an instruction 8 rows), turns each block of 64 elements into MFMA A fragments (lane l:
// row l % 32, eight elements per step) through a small LDS area of its own, and reads the B
// fragments (lane l: query l % 32, the same elements) from the staged queries.  Scores that reach
// the query's threshold are appended to the query's candidate list.
template <typename T, int METRIC>
__global__ __launch_bounds__(kBatchThreads) void batched_scan_kernel(BatchedArgs a) {
    typedef typename Mfma<T>::frag frag;
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ uint32_t s_q[kGroupQ];
    __shared__ float s_thr[kGroupQ];
    __shared__ float s_qq[kGroupQ];
    const int lane = lane_id(), wave = wave_id();
    const int d = a.d, qstride = d + kQPad;
    uint16_t* qs = (uint16_t*)smem;                      // [kGroupQ][d + kQPad] storage-type queries
    uint16_t* stage = qs + (size_t)kGroupQ * qstride + (size_t)wave * 32 * kStageLd;   // [32][kStageLd], this wavefront's
    __shared__ __align__(16) uint32_t s_run[4];
    TaskFeed feed;
    feed.start(a);
    uint32_t staged_cluster = 0xFFFFFFFFu, staged_group = 0xFFFFFFFFu;
    const int col = lane & 31, khalf = lane >> 5;
    for (uint32_t t = 0; feed.next(a, s_run, t);) {
        const BatchTask task = a.tasks[t];
        const uint32_t c = task.cluster;
        const uint32_t qbase = a.qstart[c] + task.group * kGroupQ;
        const uint32_t nqg = min((uint32_t)kGroupQ, a.qstart[c + 1] - qbase);
        if (c != staged_cluster || task.group != staged_group) {
            __syncthreads();                              // everyone is done with the previous queries
            if (threadIdx.x < kGroupQ) {
                bool ok = threadIdx.x < nqg;
                uint32_t qi = ok ? a.qidx[qbase + threadIdx.x] : 0;
                s_q[threadIdx.x] = ok ? qi : 0xFFFFFFFFu;
                s_thr[threadIdx.x] = ok ? a.thr[qi] : INFINITY;
                s_qq[threadIdx.x] = ok ? a.qq[qi] : 0.f;
            }
            __syncthreads();
            const int chunks = d / 8;                     // 16-byte chunks per query row
            for (int i = threadIdx.x; i < kGroupQ * chunks; i += blockDim.x) {
                int qq = i / chunks, ch = i - qq * chunks;
                uint32_t qi = s_q[qq];
                uint4 v = make_uint4(0, 0, 0, 0);
                if (qi != 0xFFFFFFFFu) v = *(const uint4*)((const uint16_t*)a.q_store + (size_t)qi * d + ch * 8);
                *(uint4*)(qs + (size_t)qq * qstride + ch * 8) = v;
            }
            __syncthreads();
            staged_cluster = c; staged_group = task.group;
        }
        const int64_t lo = a.off[c];
        const uint32_t n = (uint32_t)(a.off[c + 1] - lo);
        const uint32_t r0 = task.tile * kTileRows + wave * 32;     // first row of this wavefront
        if (r0 >= n) continue;
        // Loading role of a lane: 16-byte chunk lane % 8 of rows lane / 8 + {0, 8, 16, 24} of each
        // 64-element block (rows past the end re-read the last one).  Element order inside the dot
        // product is free, so MFMA step j of a block takes, for the lane half h, elements
        // 32 h + 8 j .. + 7 of the block from both operands.
        const int lrow = lane >> 3, lchunk = lane & 7;
        const uint16_t* lptr[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            lptr[u] = (const uint16_t*)a.lists + ((size_t)lo + min(r0 + (uint32_t)(lrow + 8 * u), n - 1)) * d + lchunk * 8;
        const uint16_t* brow = qs + (size_t)col * qstride + khalf * 32;
        uint16_t* wpos = stage + lrow * kStageLd + lchunk * 8;
        const uint16_t* rpos = stage + col * kStageLd + khalf * 32;
        float16_t acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        float yy[16];                  // L2: squared norms of the rows this lane will hold scores of
        if (METRIC != 0) {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                yy[i] = a.row_norm[(size_t)lo + min(r0 + (uint32_t)((i / 4) * 8 + khalf * 4 + (i % 4)), n - 1)];
        }
        // kStage16 blocks (of 64 elements, 4 MFMA steps) per stage, the next stage's rows in flight
        uint4 av[2][4 * kStage16];
        auto issue = [&](int k0, uint4 (&v)[4 * kStage16]) {
#pragma unroll
            for (int b = 0; b < kStage16; ++b) {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    v[b * 4 + u] = k0 + b * 64 < d ? load_stream16(lptr[u] + k0 + b * 64) : make_uint4(0, 0, 0, 0);
            }
        };
        auto consume = [&](int k0, const uint4 (&v)[4 * kStage16]) {
#pragma unroll
            for (int b = 0; b < kStage16; ++b) {
                if (k0 + b * 64 < d) {
                    // through LDS: written in the loading layout, read back as fragments.  A
                    // wavefront's LDS operations complete in order, so no barrier is needed.
#pragma unroll
                    for (int u = 0; u < 4; ++u) *(uint4*)(wpos + u * 8 * kStageLd) = v[b * 4 + u];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint4 av4 = *(const uint4*)(rpos + j * 8);
                        const uint4 bv = *(const uint4*)(brow + k0 + b * 64 + j * 8);
                        acc = Mfma<T>::run(__builtin_bit_cast(frag, av4), __builtin_bit_cast(frag, bv), acc);
                    }
                }
            }
        };
        constexpr int kStep = kStage16 * 64;              // elements per stage
        issue(0, av[0]);
        for (int k0 = 0; k0 < d; k0 += 2 * kStep) {
            if (k0 + kStep < d) issue(k0 + kStep, av[1]);
            consume(k0, av[0]);
            if (k0 + kStep >= d) break;
            if (k0 + 2 * kStep < d) issue(k0 + 2 * kStep, av[0]);
            consume(k0 + kStep, av[1]);
        }
        // lane holds query `col`, rows (i / 4) * 8 + khalf * 4 + i % 4
        const float thr = s_thr[col];
        const uint32_t qi = s_q[col];
        if (METRIC != 0) {
            const float qq = s_qq[col];
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = fmaf(2.f, acc[i], -yy[i]) - qq;
        }
        uint32_t pass = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t r = r0 + (i / 4) * 8 + khalf * 4 + (i % 4);
            if (acc[i] >= thr && r < n) pass |= 1u << i;
        }
        if (pass) {
            // one reservation for all rows of this lane that passed
            uint32_t pos = atomicAdd(&a.cand_count[qi], (uint32_t)__popc(pass));
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if ((pass >> i) & 1u) {
                    if (pos < (uint32_t)a.cand_cap) {
                        a.cand_row[(size_t)qi * a.cand_cap + pos] = (uint32_t)(lo + r0 + (i / 4) * 8 + khalf * 4 + (i % 4));
                        a.cand_score[(size_t)qi * a.cand_cap + pos] = acc[i];
                    }
                    ++pos;
                }
            }
        }
    }
}

// fp32 rows: v_mfma_f32_16x16x4_f32 multiplies a 16 x 4 block of rows (lane l: row l % 16,
// element l / 16) with a 4 x 16 block of queries (lane l: query l % 16, the same element).  The
// order of the elements inside a dot product is free, so the MFMA lane (row i, part p) takes the
// 16-byte chunk p of each 16-element block of its row and the four values of the chunk feed four
// MFMA steps; the query operand is read the same way from the group's queries in LDS.  The rows
// are LOADED in another lane order, eight consecutive lanes on one 128-byte line of a row (MFMA
// lanes of one row are 16 lanes apart: loading in that order makes every group of four lanes touch
// four different lines, and half lines per instruction, which costs a quarter of the bandwidth),
// and register moves across lanes (a DPP row shift and a ds_bpermute per value: no LDS memory)
// take each value to its MFMA lane.  A wavefront scores two blocks of 16 rows against up to 16
// queries; four 32-element pieces of its 32 rows are in flight while the previous four are consumed
// (16 KB per wavefront: the depth per wavefront matters more here than a second workgroup per CU).
typedef float float4_t __attribute__((ext_vector_type(4)));
constexpr int kGroupQ32 = 16;      // queries per task for fp32 rows: one MFMA tile wide
constexpr int kQPad32 = 4;         // padding (floats) of a staged query row: consecutive queries start 4 banks apart
constexpr int kStage32 = 4;        // 32-element pieces of a row per pipeline stage

template <int METRIC>
__global__ __launch_bounds__(kBatchThreads) void batched_scan_f32_kernel(BatchedArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ uint32_t s_q[kGroupQ32];
    __shared__ float s_thr[kGroupQ32];
    __shared__ float s_qq[kGroupQ32];
    const int lane = lane_id(), wave = wave_id();
    const int d = a.d, qstride = d + kQPad32;
    float* qs = (float*)smem;                            // [kGroupQ32][d + kQPad32] queries
    __shared__ __align__(16) uint32_t s_run[4];
    TaskFeed feed;
    feed.start(a);
    uint32_t staged_cluster = 0xFFFFFFFFu, staged_group = 0xFFFFFFFFu;
    const int col = lane & 15, kq = lane >> 4;
    for (uint32_t t = 0; feed.next(a, s_run, t);) {
        const BatchTask task = a.tasks[t];
        const uint32_t c = task.cluster;
        const uint32_t qbase = a.qstart[c] + task.group * kGroupQ32;
        const uint32_t nqg = min((uint32_t)kGroupQ32, a.qstart[c + 1] - qbase);
        if (c != staged_cluster || task.group != staged_group) {
            __syncthreads();                              // everyone is done with the previous queries
            if (threadIdx.x < kGroupQ32) {
                bool ok = threadIdx.x < nqg;
                uint32_t qi = ok ? a.qidx[qbase + threadIdx.x] : 0;
                s_q[threadIdx.x] = ok ? qi : 0xFFFFFFFFu;
                s_thr[threadIdx.x] = ok ? a.thr[qi] : INFINITY;
                s_qq[threadIdx.x] = ok ? a.qq[qi] : 0.f;
            }
            __syncthreads();
            const int chunks = d / 4;                     // 16-byte chunks per query row
            for (int i = threadIdx.x; i < kGroupQ32 * chunks; i += blockDim.x) {
                int qq = i / chunks, ch = i - qq * chunks;
                uint32_t qi = s_q[qq];
                uint4 v = make_uint4(0, 0, 0, 0);
                if (qi != 0xFFFFFFFFu) v = *(const uint4*)(a.q + (size_t)qi * d + ch * 4);
                *(uint4*)(qs + (size_t)qq * qstride + ch * 4) = v;
            }
            __syncthreads();
            staged_cluster = c; staged_group = task.group;
        }
        const int64_t lo = a.off[c];
        const uint32_t n = (uint32_t)(a.off[c + 1] - lo);
        const uint32_t r0 = task.tile * kTileRows + wave * 32;     // first row of this wavefront
        if (r0 >= n) continue;
        // Loading role of a lane: 16-byte chunk lane % 8 of rows lane / 8 and lane / 8 + 8 of each row
        // block, for every 32-element (128-byte) piece of the rows; rows past the end re-read the last one.
        const float* lp[4];            // [row block][row half]
#pragma unroll
        for (int j = 0; j < 4; ++j)
            lp[j] = (const float*)a.lists + ((size_t)lo + min(r0 + 8u * j + (uint32_t)(lane >> 3), n - 1)) * d + (lane & 7) * 4;
        // lane that holds, after the exchange below, what this MFMA lane (row col, part kq) needs
        const int from = (((col & 7) << 3) | ((col >> 3) << 2) | kq) << 2;
        const float* bq = qs + (size_t)col * qstride + kq * 4;
        float4_t acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        float yy[8];                   // L2: squared norms of the rows this lane will hold scores of
        if (METRIC != 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                yy[i] = a.row_norm[(size_t)lo + min(r0 + (uint32_t)((i / 4) * 16 + kq * 4 + (i % 4)), n - 1)];
        }
        uint4 av[2][4 * kStage32];
        auto issue = [&](int k0, uint4 (&v)[4 * kStage32]) {
#pragma unroll
            for (int b = 0; b < kStage32; ++b) {
                const bool in = k0 + b * 32 < d;
#pragma unroll
                for (int j = 0; j < 4; ++j) v[4 * b + j] = in ? load_stream16(lp[j] + k0 + b * 32) : make_uint4(0, 0, 0, 0);
            }
        };
        // One loaded value to its MFMA lanes.  Lanes with chunk >= 4 hold the second 16-element
        // block of the piece.  A move by four lanes inside each row of 16 lanes (DPP row shift,
        // written only to the lanes of one chunk half) gathers the first block of both row halves
        // in one register (lane (r, c): row r + 8 (c / 4), chunk c % 4) and the second block in
        // another; one lane permutation each then puts them in MFMA order.
        auto to_mfma = [&](uint32_t lo_half, uint32_t hi_half, float& first, float& second) {
            const int f = __builtin_amdgcn_update_dpp((int)lo_half, (int)hi_half, 0x114, 0xF, 0xA, false);   // row_shr:4 into chunks 4..7
            const int g = __builtin_amdgcn_update_dpp((int)hi_half, (int)lo_half, 0x104, 0xF, 0x5, false);   // row_shl:4 into chunks 0..3
            first = __int_as_float(__builtin_amdgcn_ds_bpermute(from, f));
            second = __int_as_float(__builtin_amdgcn_ds_bpermute(from, g));
        };
        auto consume = [&](int k0, const uint4 (&v)[4 * kStage32]) {
#pragma unroll
            for (int b = 0; b < kStage32; ++b) {
                if (k0 + b * 32 < d) {
                    const float4 bv0 = *(const float4*)(bq + k0 + b * 32);
                    const float4 bv1 = *(const float4*)(bq + k0 + b * 32 + 16);
                    float x[2][2][4];          // [row block][16-element block][value of the chunk]
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb) {
                        const uint4 h0 = v[4 * b + 2 * rb], h1 = v[4 * b + 2 * rb + 1];
                        to_mfma(h0.x, h1.x, x[rb][0][0], x[rb][1][0]);
                        to_mfma(h0.y, h1.y, x[rb][0][1], x[rb][1][1]);
                        to_mfma(h0.z, h1.z, x[rb][0][2], x[rb][1][2]);
                        to_mfma(h0.w, h1.w, x[rb][0][3], x[rb][1][3]);
                    }
                    const float q0[4] = {bv0.x, bv0.y, bv0.z, bv0.w}, q1[4] = {bv1.x, bv1.y, bv1.z, bv1.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[0][0][e], q0[e], acc[0], 0, 0, 0);
                        acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[1][0][e], q0[e], acc[1], 0, 0, 0);
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[0][1][e], q1[e], acc[0], 0, 0, 0);
                        acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[1][1][e], q1[e], acc[1], 0, 0, 0);
                    }
                }
            }
        };
        constexpr int kStep = kStage32 * 32;              // elements per stage
        issue(0, av[0]);
        for (int k0 = 0; k0 < d; k0 += 2 * kStep) {
            if (k0 + kStep < d) issue(k0 + kStep, av[1]);
            consume(k0, av[0]);
            if (k0 + kStep >= d) break;
            if (k0 + 2 * kStep < d) issue(k0 + 2 * kStep, av[0]);
            consume(k0 + kStep, av[1]);
        }
        // lane holds query `col`, rows (i / 4) * 16 + kq * 4 + i % 4
        const float thr = s_thr[col];
        const uint32_t qi = s_q[col];
        float sc[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) { sc[i] = acc[0][i]; sc[4 + i] = acc[1][i]; }
        if (METRIC != 0) {
            const float qq = s_qq[col];
#pragma unroll
            for (int i = 0; i < 8; ++i) sc[i] = fmaf(2.f, sc[i], -yy[i]) - qq;
        }
        uint32_t pass = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t r = r0 + (i / 4) * 16 + kq * 4 + (i % 4);
            if (sc[i] >= thr && r < n) pass |= 1u << i;
        }
        if (pass) {
            uint32_t pos = atomicAdd(&a.cand_count[qi], (uint32_t)__popc(pass));
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if ((pass >> i) & 1u) {
                    if (pos < (uint32_t)a.cand_cap) {
                        a.cand_row[(size_t)qi * a.cand_cap + pos] = (uint32_t)(lo + r0 + (i / 4) * 16 + kq * 4 + (i % 4));
                        a.cand_score[(size_t)qi * a.cand_cap + pos] = sc[i];
                    }
                    ++pos;
                }
            }
        }
    }
}

// ---- final ranking of a query's candidates ------------------------------------------------------------------
// One workgroup per query: candidates are first pruned by their approximate scores, the survivors
// are re-scored in fp64 (fp32 query), and the k best by (score, id) come from a radix select on
// the 64-bit keys and a rank-by-counting.
__global__ __launch_bounds__(kSelectThreads) void batched_merge_kernel(BatchedArgs a) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh[8];
    __shared__ double f_key[2 * kMaxKPrime];
    __shared__ int64_t f_id[2 * kMaxKPrime];
    __shared__ unsigned long long best;
    const int tid = threadIdx.x, nt = blockDim.x, lane = lane_id();
    const int qi = blockIdx.x, k = a.k;
    const uint32_t raw = a.cand_count[qi];
    if (raw > (uint32_t)a.cand_cap) {                  // too many candidates: the host redoes this query
        if (tid == 0) a.overflow[qi] = 1;
        return;
    }
    // 1. prune by the approximate scores: with t = the k-th best approximate score, a row of the
    //    true top k has an approximate score of at least t - 2 eps (each score is within eps of
    //    the exact one), so only those rows are re-scored.
    const uint32_t n0 = raw;
    const float* sc = a.cand_score + (size_t)qi * a.cand_cap;
    const uint32_t* rows0 = a.cand_row + (size_t)qi * a.cand_cap;
    uint32_t* rows = a.surv_row + (size_t)qi * a.surv_cap;
    auto skey = [&](uint32_t i) { return ~ordered(sc[i]); };      // ascending key = best first
    if (tid == 0) { sh[4] = 0; sh[5] = 0; sh[6] = 0; }
    __syncthreads();
    float cut = -INFINITY;
    if (n0 > (uint32_t)k) {
        uint32_t mask, prefix, need, group;
        block_radix_select<uint32_t>(skey, n0, (uint32_t)k, hist, sh, mask, prefix, need, group);
        // key of the k-th best: the largest kept key
        uint32_t worst = 0;
        for (uint32_t i = tid; i < n0; i += nt) {
            uint32_t ky = skey(i), hi = ky & mask;
            if (hi < prefix || hi == prefix) worst = max(worst, (need == group || hi < prefix) ? ky : prefix);
        }
#pragma unroll
        for (int m2 = 32; m2 >= 1; m2 >>= 1) worst = max(worst, (uint32_t)__shfl_xor((int)worst, m2));
        if (lane == 0) atomicMax(&sh[6], worst);
        __syncthreads();
        const uint32_t o = ~sh[6];                        // ordered(float) of the k-th best approximate score
        const float kth = __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
        cut = kth - 2.f * a.eps[qi];
    }
    for (uint32_t i0 = 0; i0 < n0; i0 += nt) {
        uint32_t i = i0 + tid;
        bool ok = i < n0 && sc[i] >= cut;
        uint64_t bal = __ballot(ok);
        uint32_t base = 0;
        if (lane == 0 && bal) base = atomicAdd(&sh[5], (uint32_t)__popcll(bal));
        base = read_lane(base, 0);
        uint32_t p = base + __popcll(bal & ((1ull << lane) - 1ull));
        if (ok && p < (uint32_t)a.surv_cap) rows[p] = rows0[i];
    }
    __syncthreads();
    const uint32_t n = sh[5];
    if (n > (uint32_t)a.surv_cap) {                    // cannot happen unless scores are massively tied
        if (tid == 0) a.overflow[qi] = 1;
        return;
    }
    if (tid == 0) a.overflow[qi] = 0;
    // 2. fp64 re-score of the survivors
    uint64_t* keys = a.cand_key + (size_t)qi * a.surv_cap;
    const float* q = a.q + (size_t)qi * a.d;
    // a group of lanes per survivor, so that their row loads overlap; the same order of operations
    // as the query-by-query merge
    constexpr int kLpc = kRescoreLanes;
    const int sub = tid % kLpc;
#pragma unroll 1
    for (uint32_t c = (uint32_t)(tid / kLpc); c < n; c += (uint32_t)(nt / kLpc)) {
        const double s = rescore_row(a.lists, q, a.d, a.dtype, a.metric, rows[c], sub);
        if (sub == 0) keys[c] = ~ordered(a.metric == 0 ? s : -s);            // ascending key = best first
    }
    __syncthreads();
    const uint32_t want = min((uint32_t)k, n);
    if (tid == 0) sh[4] = 0;
    __syncthreads();
    auto key_at = [&](uint32_t i) { return keys[i]; };
    auto id_at = [&](uint32_t i) { return a.ids ? a.ids[rows[i]] : (int64_t)rows[i]; };
    auto emit = [&](uint32_t i) {
        uint32_t p = atomicAdd(&sh[4], 1u);
        if (p < 2 * kMaxKPrime) { f_key[p] = unordered(~keys[i]); f_id[p] = id_at(i); }
    };
    if (want > 0) {
        uint64_t mask, prefix; uint32_t need, group;
        block_radix_select<uint64_t>(key_at, n, want, hist, sh, mask, prefix, need, group);
        const bool take_group = need == group;
        for (uint32_t i = tid; i < n; i += nt) {
            uint64_t hi = keys[i] & mask;
            if (hi < prefix || (take_group && hi == prefix)) emit(i);
        }
        __syncthreads();
        if (!take_group) {
            long long last = -1;
            for (uint32_t it = 0; it < need; ++it) {
                if (tid == 0) best = ~0ull;
                __syncthreads();
                for (uint32_t i = tid; i < n; i += nt)
                    if ((keys[i] & mask) == prefix) { long long id = id_at(i); if (id > last) atomicMin(&best, (unsigned long long)id); }
                __syncthreads();
                unsigned long long b = best;
                if (b == ~0ull) break;
                last = (long long)b;
                for (uint32_t i = tid; i < n; i += nt)
                    if ((keys[i] & mask) == prefix && id_at(i) == last) emit(i);
                __syncthreads();
            }
        }
    }
    __syncthreads();
    const uint32_t tot = min(sh[4], (uint32_t)(2 * kMaxKPrime));
    if ((uint32_t)tid < tot) {
        double mk = f_key[tid]; int64_t mi = f_id[tid];
        uint32_t rank = 0;
        // eight others per pass, all read before any is compared, and no branches
#pragma unroll 1
        for (uint32_t j0 = 0; j0 < tot; j0 += 8) {
            double ok[8]; int64_t oi[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t j = min(j0 + u, tot - 1);
                ok[u] = f_key[j]; oi[u] = f_id[j];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool ahead = (ok[u] > mk) | ((ok[u] == mk) & (oi[u] < mi));
                rank += (uint32_t)(ahead & (j0 + u < tot));
            }
        }
        if (rank < (uint32_t)k) {
            a.out_ids[(size_t)qi * k + rank] = mi;
            a.out_dists[(size_t)qi * k + rank] = (float)(a.metric == 0 ? mk : -mk);
        }
    }
    for (uint32_t i = tot + tid; i < (uint32_t)k; i += nt) {
        a.out_ids[(size_t)qi * k + i] = -1;
        a.out_dists[(size_t)qi * k + i] = a.metric == 0 ? -INFINITY : INFINITY;
    }
}

// ---- launch sequence ---------------------------------------------------------------------------------------
int batched_group_q(int dtype) { return dtype == 0 ? kGroupQ32 : kGroupQ; }

size_t batched_scan_lds(int d, int dtype) {
    if (dtype == 0) return (size_t)kGroupQ32 * (d + kQPad32) * 4;
    return (size_t)kGroupQ * (d + kQPad) * 2 + (size_t)kBatchWaves * 32 * kStageLd * 2;
}

uint64_t batched_task_bound(const int64_t* off_host, int nlist, int nq, int dtype) {
    // every cluster may be probed, by every query
    uint64_t tiles = 0;
    for (int c = 0; c < nlist; ++c) tiles += (uint64_t)((off_host[c + 1] - off_host[c] + kTileRows - 1) / kTileRows);
    const uint64_t gq = (uint64_t)batched_group_q(dtype);
    return tiles * (((uint64_t)nq + gq - 1) / gq) + 1;
}

size_t batched_thr_part_floats(int nq) { return (size_t)nq * kSampleParts * kMaxKPrime; }

typedef void (*BatchedScanFn)(BatchedArgs);
static BatchedScanFn batched_scan_fn(int dtype, int metric) {
    if (dtype == 0) return metric == 0 ? batched_scan_f32_kernel<0> : batched_scan_f32_kernel<1>;
    if (dtype == 1) return metric == 0 ? batched_scan_kernel<F16, 0> : batched_scan_kernel<F16, 1>;
    return metric == 0 ? batched_scan_kernel<BF16, 0> : batched_scan_kernel<BF16, 1>;
}

int batched_resident_grid(int dtype, int metric, int d, int n_cu) {
    int per_cu = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)batched_scan_fn(dtype, metric), kBatchThreads,
                                                                batched_scan_lds(d, dtype));
    if (e != hipSuccess || per_cu < 1) per_cu = 1;
    if (per_cu > 4) per_cu = 4;
    return per_cu * n_cu;
}

// rounding of an fp32 sum made like the threshold sample's: terms per lane, six additions across
// the lanes, and for L2 the rounded difference and its square
float batched_sample_coef(int d, int dtype, int metric) {
    const int epl = dtype == 0 ? 4 : 8;
    const int chunks = d / epl;
    const int terms = epl * ((chunks + 63) / 64) + 6 + (metric != 0 ? 3 : 0);
    return 1.05f * (float)(terms + 2) * 0x1p-24f;
}

hipError_t launch_batched(const BatchedArgs& a, int grid, hipStream_t s, hipEvent_t scan_start, hipEvent_t scan_stop, bool with_merge) {
    const int pairs = a.nq * a.nprobe;
    if (a.dtype == 0) hipLaunchKernelGGL(thr_sample_kernel<F32>, dim3(a.nq, kSampleParts), dim3(256), (size_t)a.d * 4, s, a);
    else if (a.dtype == 1) hipLaunchKernelGGL(thr_sample_kernel<F16>, dim3(a.nq, kSampleParts), dim3(256), (size_t)a.d * 4, s, a);
    else hipLaunchKernelGGL(thr_sample_kernel<BF16>, dim3(a.nq, kSampleParts), dim3(256), (size_t)a.d * 4, s, a);
    hipLaunchKernelGGL(prep_queries_kernel, dim3(a.nq), dim3(64), 0, s, a);
    hipLaunchKernelGGL(zero_u32_kernel, dim3((a.nlist + 1 + 255) / 256), dim3(256), 0, s, a.list_count, a.nlist + 1);   // and the ticket behind them
    hipLaunchKernelGGL(count_pairs_kernel, dim3((pairs + 255) / 256), dim3(256), 0, s, a);
    hipLaunchKernelGGL(scan_lists_kernel, dim3(1), dim3(1024), 0, s, a);
    hipLaunchKernelGGL(fill_pairs_kernel, dim3((pairs + 255) / 256), dim3(256), 0, s, a);
    hipLaunchKernelGGL(make_tasks_kernel, dim3(min(a.nlist, 4096)), dim3(256), 0, s, a);
    const BatchedScanFn scan = batched_scan_fn(a.dtype, a.metric);
    IVF_LAUNCH(scan, dim3(grid), dim3(kBatchThreads), batched_scan_lds(a.d, a.dtype), s, scan_start, scan_stop, a);
    if (with_merge) hipLaunchKernelGGL(batched_merge_kernel, dim3(a.nq), dim3(kSelectThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace ivf
