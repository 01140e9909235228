// HIP kernels of the IVF search path for gfx950 (wave64): coarse scoring, top-nprobe
// selection, list scan with per-workgroup top-k', and the fp64 re-score + merge.
// The operations are those of TeleRAG (arxiv 2502.20969) App. B: coarse search over the
// centroids, fine search over the rows of the selected clusters, k nearest by a sort.
#include "ivf_device.h"

namespace ivf {
using namespace dev;

// =============================================================================================
// Coarse scoring (App. B, first step): scores[q][j] = d(x_q, c_j) for every centroid, in fp64.
// One wavefront per centroid row; the queries are staged in LDS and widened on use.
// HBM-bound on the nlist*d*4 bytes of the centroid matrix.
// =============================================================================================
constexpr int kCoarseQT = 4;   // queries sharing one pass over a centroid row

__global__ __launch_bounds__(256) void coarse_kernel(CoarseArgs a) {
    extern __shared__ float qd[];    // [kCoarseQT][d]
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int q0 = blockIdx.y * kCoarseQT;
    const int nqt = min(kCoarseQT, a.nq - q0);
    for (int i = threadIdx.x; i < kCoarseQT * a.d; i += blockDim.x) {
        int qq = i / a.d, t = i - qq * a.d;
        qd[i] = qq < nqt ? a.q[(size_t)(q0 + qq) * a.d + t] : 0.f;
    }
    __syncthreads();
    const int row = blockIdx.x * 4 + wave;
    if (row >= a.nlist) return;
    const float* c = a.centroids + (size_t)row * a.d;
    double acc[kCoarseQT];
#pragma unroll
    for (int qq = 0; qq < kCoarseQT; ++qq) acc[qq] = 0.0;
    if ((a.d & 3) == 0) {
        for (int t0 = lane * 4; t0 < a.d; t0 += 256) {
            float4 v = *(const float4*)(c + t0);
            const double cv[4] = {(double)v.x, (double)v.y, (double)v.z, (double)v.w};
#pragma unroll
            for (int qq = 0; qq < kCoarseQT; ++qq) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    double x = (double)qd[qq * a.d + t0 + e];
                    if (a.metric == 0) acc[qq] = fma(x, cv[e], acc[qq]);
                    else { double df = x - cv[e]; acc[qq] = fma(df, df, acc[qq]); }
                }
            }
        }
    } else {
        for (int t = lane; t < a.d; t += 64) {
            double cv = (double)c[t];
#pragma unroll
            for (int qq = 0; qq < kCoarseQT; ++qq) {
                double x = (double)qd[qq * a.d + t];
                if (a.metric == 0) acc[qq] = fma(x, cv, acc[qq]);
                else { double df = x - cv; acc[qq] = fma(df, df, acc[qq]); }
            }
        }
    }
#pragma unroll
    for (int qq = 0; qq < kCoarseQT; ++qq) {
        double s = wave_sum(acc[qq]);
        if (lane == 0 && qq < nqt) a.scores[(size_t)(q0 + qq) * a.nlist + row] = s;
    }
}

hipError_t launch_coarse(const CoarseArgs& a, hipStream_t s) {
    dim3 grid((a.nlist + 3) / 4, (a.nq + kCoarseQT - 1) / kCoarseQT);
    size_t lds = sizeof(float) * kCoarseQT * a.d;
    hipLaunchKernelGGL(coarse_kernel, grid, dim3(256), lds, s, a);
    return hipGetLastError();
}

// =============================================================================================
// Top-nprobe selection (App. B: the L nearest centroids), ordered nearest first with ties by
// smaller cluster index, plus the slot tables the scan walks.  One workgroup per query.
// =============================================================================================
__device__ __forceinline__ uint64_t coarse_key(double score, int metric) {
    uint64_t o = ordered(score);
    return metric == 0 ? ~o : o;       // ascending key = nearest first
}

__global__ __launch_bounds__(kSelectThreads) void select_kernel(SelectArgs a, uint32_t pad, int in_lds) {
    extern __shared__ unsigned char smem_raw[];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh[8];
    __shared__ uint32_t scan_buf[kSelectThreads / 64 + 1];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int qi = blockIdx.x;
    const double* sc = a.scores + (size_t)qi * a.nlist;
    uint64_t* keys; uint32_t* idx;
    if (in_lds) {
        keys = (uint64_t*)smem_raw;
        idx = (uint32_t*)(smem_raw + sizeof(uint64_t) * pad);
    } else {
        keys = a.sort_keys + (size_t)qi * pad;
        idx = a.sort_idx + (size_t)qi * pad;
    }
    const uint32_t nlist = a.nlist, nprobe = a.nprobe;

    if (nlist <= pad) {
        // small index: sort every centroid
        for (uint32_t i = tid; i < pad; i += nt) {
            keys[i] = i < nlist ? coarse_key(sc[i], a.metric) : ~0ull;
            idx[i] = i < nlist ? i : 0xFFFFFFFFu;
        }
        __syncthreads();
    } else {
        // large index: radix-select the nprobe best, then sort only those
        uint64_t mask, prefix; uint32_t need, group;
        auto key_at = [&](uint32_t i) { return coarse_key(sc[i], a.metric); };
        block_radix_select<uint64_t>(key_at, nlist, nprobe, hist, sh, mask, prefix, need, group);
        if (tid == 0) { sh[4] = 0; sh[5] = 0; }
        for (uint32_t i = tid; i < pad; i += nt) { keys[i] = ~0ull; idx[i] = 0xFFFFFFFFu; }
        __syncthreads();
        const bool take_group = need == group;
        for (uint32_t i = tid; i < nlist; i += nt) {
            uint64_t k = key_at(i);
            uint64_t hi = k & mask;
            if (hi < prefix || (take_group && hi == prefix)) {
                uint32_t p = atomicAdd(&sh[4], 1u);
                keys[p] = k; idx[p] = i;
            }
        }
        __syncthreads();
        if (!take_group) {
            // the boundary group holds fully equal scores: keep the `need` smallest indices.
            // Entries are visited in index order by one wavefront so the choice is ordered.
            if (tid < 64) {
                uint32_t taken = 0;
                for (uint32_t base = 0; base < nlist && taken < need; base += 64) {
                    uint32_t i = base + tid;
                    bool tie = i < nlist && (key_at(i) & mask) == prefix;
                    uint64_t b = __ballot(tie);
                    uint32_t rank = taken + __popcll(b & ((1ull << tid) - 1ull));
                    if (tie && rank < need) {
                        uint32_t p = sh[4] + rank;
                        keys[p] = key_at(i); idx[p] = i;
                    }
                    taken += __popcll(b);
                }
            }
            __syncthreads();
        }
    }
    block_bitonic_sort(keys, idx, pad);

    // slot tables: per selected cluster its placement and its share of the scan tasks
    const int64_t* off = a.off;
    int64_t* s_base = a.slots.base + (size_t)qi * nprobe;
    uint32_t* s_grow = a.slots.grow + (size_t)qi * nprobe;
    uint32_t* s_n = a.slots.nrows + (size_t)qi * nprobe;
    uint32_t* s_tp = a.slots.tprefix + (size_t)qi * (nprobe + 1);
    uint32_t carry = 0;
    for (uint32_t base = 0; base < nprobe; base += nt) {
        uint32_t i = base + tid;
        uint32_t tasks = 0;
        if (i < nprobe) {
            uint32_t c = idx[i];
            a.probe[(size_t)qi * nprobe + i] = (int32_t)c;
            int64_t lo = off[c];
            uint32_t n = (uint32_t)(off[c + 1] - lo);
            int64_t ro = a.res_off[c];
            s_base[i] = ro;
            s_grow[i] = (uint32_t)lo;
            s_n[i] = n;
            tasks = ro >= 0 ? (n + a.rows_per_task - 1) / a.rows_per_task : 0;
            if (a.rows_counter && ro >= 0) atomicAdd(a.rows_counter, (unsigned long long)n);
        }
        // block-wide exclusive scan of `tasks`
        uint32_t incl = tasks;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            uint32_t up = __shfl_up(incl, o);
            if ((tid & 63) >= o) incl += up;
        }
        if ((tid & 63) == 63) scan_buf[tid >> 6] = incl;
        __syncthreads();
        uint32_t wave_off = 0;
        for (int w = 0; w < (tid >> 6); ++w) wave_off += scan_buf[w];
        uint32_t total = 0;
        for (int w = 0; w < nt / 64; ++w) total += scan_buf[w];
        if (i < nprobe) s_tp[i] = carry + wave_off + incl - tasks;
        carry += total;
        __syncthreads();
    }
    if (tid == 0) s_tp[nprobe] = carry;
}

static uint32_t next_pow2(uint32_t v) { uint32_t p = 1; while (p < v) p <<= 1; return p; }

// power-of-two length of the select kernel's sort array for (nlist, nprobe)
uint32_t select_sort_pad(int nlist, int nprobe) {
    uint32_t full = next_pow2((uint32_t)nlist);
    return full <= (uint32_t)kSortLdsCap ? full : next_pow2((uint32_t)nprobe);
}

hipError_t launch_select(const SelectArgs& a, hipStream_t s) {
    uint32_t pad = select_sort_pad(a.nlist, a.nprobe);
    int in_lds = pad <= (uint32_t)kSortLdsCap;
    size_t lds = in_lds ? (size_t)pad * 12 : 0;
    hipLaunchKernelGGL(select_kernel, dim3(a.nq), dim3(kSelectThreads), lds, s, a, pad, in_lds);
    return hipGetLastError();
}

// =============================================================================================
// List scan (App. B, second step): d(x, y) for every row y of every selected, resident list,
// reduced in the kernel to the kprime best rows per workgroup.  HBM-bound: each row is read
// once with 16-byte loads; nothing but kprime pairs per workgroup is written.
//
// A row is covered by LPR lanes with SEG 16-byte loads each; a wavefront instruction covers
// 64/LPR rows; U such row groups are in flight per wavefront.  A task is U*64/LPR consecutive
// rows of one list.  The tasks of a query are split evenly over the grid; the four wavefronts
// of a workgroup take the tasks of its share in turn.
// =============================================================================================
struct SlotView {
    const int64_t* base; const uint32_t* grow; const uint32_t* nrows; const uint32_t* tp;
};

template <int U>
__device__ __forceinline__ float pick(const float (&a)[U], int u) {
    float r = a[0];
#pragma unroll
    for (int i = 1; i < U; ++i) r = (u == i) ? a[i] : r;
    return r;
}

// first slot whose task range contains t (tp is non-decreasing, tp[0] = 0, t < tp[nprobe])
__device__ __forceinline__ int find_slot(const uint32_t* tp, int nprobe, uint32_t t) {
    int lo = 0, hi = nprobe;      // invariant: tp[lo] <= t < tp[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (tp[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

template <int KL>
__device__ __forceinline__ void finish_workgroup(TopList<KL>& top, const ScanArgs& p, float* m_key,
                                                 uint32_t* m_row, int qi) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int kp = p.kprime;
    if (wave > 0) {
#pragma unroll
        for (int j = 0; j < KL; ++j) {
            int e = j * 64 + lane;
            if (e < kp) { m_key[(wave - 1) * kp + e] = top.key[j]; m_row[(wave - 1) * kp + e] = top.row[j]; }
        }
    }
    __syncthreads();
    if (wave == 0) {
        for (int w = 0; w < 3; ++w) {
            for (int i = 0; i < kp; ++i) {
                float ck = m_key[w * kp + i];
                uint32_t cr = m_row[w * kp + i];
                if (cr == kNoRow || ck < top.thr) break;     // lists are sorted: nothing further can enter
                top.insert(ck, cr, p.ids, kp);
            }
        }
        size_t o = ((size_t)qi * p.grid + blockIdx.x) * kp;
#pragma unroll
        for (int j = 0; j < KL; ++j) {
            int e = j * 64 + lane;
            if (e < kp) { p.part_key[o + e] = top.key[j]; p.part_row[o + e] = top.row[j]; }
        }
    }
}

// loads the slot table of query qi into LDS when it fits, else points at global memory
__device__ __forceinline__ SlotView stage_slots(const ScanArgs& p, int qi, unsigned char* smem, int in_lds) {
    const int np = p.nprobe;
    SlotView g{p.slots.base + (size_t)qi * np, p.slots.grow + (size_t)qi * np,
               p.slots.nrows + (size_t)qi * np, p.slots.tprefix + (size_t)qi * (np + 1)};
    if (!in_lds) return g;
    int64_t* l_base = (int64_t*)smem;
    uint32_t* l_grow = (uint32_t*)(smem + 8 * (size_t)np);
    uint32_t* l_n = l_grow + np;
    uint32_t* l_tp = l_n + np;
    for (int i = threadIdx.x; i < np; i += blockDim.x) {
        l_base[i] = g.base[i]; l_grow[i] = g.grow[i]; l_n[i] = g.nrows[i]; l_tp[i] = g.tp[i];
    }
    if (threadIdx.x == 0) l_tp[np] = g.tp[np];
    __syncthreads();
    return SlotView{l_base, l_grow, l_n, l_tp};
}

__host__ __device__ inline size_t scan_lds_bytes(int nprobe, int kprime, int in_lds, int d_floats) {
    size_t table = in_lds ? (size_t)nprobe * 20 + 8 : 0;
    table = (table + 7) & ~(size_t)7;
    return table + (size_t)3 * kprime * 8 + (size_t)d_floats * 4;
}

template <typename T, int LPR, int SEG, int U, int METRIC, int KL>
__global__ __launch_bounds__(kScanThreads) void scan_kernel(ScanArgs p, int in_lds) {
    constexpr int EPL = T::kPerLoad;
    constexpr int RPI = 64 / LPR;
    constexpr int RPT = U * RPI;
    extern __shared__ unsigned char smem[];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int sub = lane % LPR, rsel = lane / LPR;
    const int qi = blockIdx.y;
    const int np = p.nprobe;
    SlotView sv = stage_slots(p, qi, smem, in_lds);
    size_t table = in_lds ? (size_t)np * 20 + 8 : 0;
    table = (table + 7) & ~(size_t)7;
    float* m_key = (float*)(smem + table);
    uint32_t* m_row = (uint32_t*)(m_key + 3 * p.kprime);

    // this lane's slice of the query
    float qv[SEG][EPL];
    const float* q = p.q + (size_t)qi * p.d;
#pragma unroll
    for (int sg = 0; sg < SEG; ++sg) {
        int col = (sg * LPR + sub) * EPL;
#pragma unroll
        for (int e = 0; e < EPL; ++e) qv[sg][e] = col + e < p.d ? q[col + e] : 0.f;
    }

    TopList<KL> top;
    top.init();

    const uint32_t total = sv.tp[np];
    const uint32_t t_begin = (uint32_t)((uint64_t)total * blockIdx.x / gridDim.x);
    const uint32_t t_end = (uint32_t)((uint64_t)total * (blockIdx.x + 1) / gridDim.x);
    const size_t row_bytes = (size_t)p.d * T::kBytes;
    uint32_t t = t_begin + wave;
    int slot = t < t_end ? find_slot(sv.tp, np, t) : 0;
    for (; t < t_end; t += 4) {
        while (t >= sv.tp[slot + 1]) ++slot;
        const uint32_t n = sv.nrows[slot];
        const uint32_t r0 = (t - sv.tp[slot]) * RPT;
        const uint32_t nr = min((uint32_t)RPT, n - r0);
        const unsigned char* rows = (const unsigned char*)p.buf + ((size_t)sv.base[slot] + r0) * row_bytes;

        uint4 v[U][SEG];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t r = min((uint32_t)(u * RPI + rsel), nr - 1);   // rows past the end re-read the last one
            const unsigned char* rp = rows + (size_t)r * row_bytes;
#pragma unroll
            for (int sg = 0; sg < SEG; ++sg) {
                int col = (sg * LPR + sub) * EPL;
                if (col < p.d) v[u][sg] = *(const uint4*)(rp + (size_t)col * T::kBytes);
                else v[u][sg] = make_uint4(0, 0, 0, 0);
            }
        }
        float acc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float s = 0.f;
#pragma unroll
            for (int sg = 0; sg < SEG; ++sg) {
                float x[EPL];
                Unpack<T>::run(v[u][sg], x);
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    if (METRIC == 0) s = fmaf(qv[sg][e], x[e], s);
                    else { float df = qv[sg][e] - x[e]; s = fmaf(df, df, s); }
                }
            }
            s = group_sum<LPR>(s);
            acc[u] = METRIC == 0 ? s : -s;        // key: larger is nearer
        }
        // almost every row fails the threshold: one ballot decides whether to look closer
        bool any = false;
#pragma unroll
        for (int u = 0; u < U; ++u) any |= (uint32_t)(u * RPI + rsel) < nr && acc[u] >= top.thr;
        if (__ballot(any)) {
#pragma unroll 1
            for (int u = 0; u < U; ++u) {
                float au = pick<U>(acc, u);
#pragma unroll 1
                for (int j = 0; j < RPI; ++j) {
                    uint32_t r = u * RPI + j;
                    if (r >= nr) break;
                    float ck = read_lane(au, j * LPR);
                    if (ck >= top.thr) top.insert(ck, sv.grow[slot] + r0 + r, p.ids, p.kprime);
                }
            }
        }
    }
    finish_workgroup<KL>(top, p, m_key, m_row, qi);
}

// Fallback for any d and any row alignment: element-wise loads, query in LDS, 4 rows per task.
template <int METRIC, int KL>
__global__ __launch_bounds__(kScanThreads) void scan_generic_kernel(ScanArgs p, int in_lds) {
    constexpr int RPT = 4;
    extern __shared__ unsigned char smem[];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int qi = blockIdx.y;
    const int np = p.nprobe;
    SlotView sv = stage_slots(p, qi, smem, in_lds);
    size_t table = in_lds ? (size_t)np * 20 + 8 : 0;
    table = (table + 7) & ~(size_t)7;
    float* m_key = (float*)(smem + table);
    uint32_t* m_row = (uint32_t*)(m_key + 3 * p.kprime);
    float* ql = (float*)(m_row + 3 * p.kprime);
    for (int i = threadIdx.x; i < p.d; i += blockDim.x) ql[i] = p.q[(size_t)qi * p.d + i];
    __syncthreads();

    TopList<KL> top;
    top.init();
    const uint32_t total = sv.tp[np];
    const uint32_t t_begin = (uint32_t)((uint64_t)total * blockIdx.x / gridDim.x);
    const uint32_t t_end = (uint32_t)((uint64_t)total * (blockIdx.x + 1) / gridDim.x);
    uint32_t t = t_begin + wave;
    int slot = t < t_end ? find_slot(sv.tp, np, t) : 0;
    for (; t < t_end; t += 4) {
        while (t >= sv.tp[slot + 1]) ++slot;
        const uint32_t n = sv.nrows[slot];
        const uint32_t r0 = (t - sv.tp[slot]) * RPT;
        const uint32_t nr = min((uint32_t)RPT, n - r0);
        for (uint32_t r = 0; r < nr; ++r) {
            size_t e0 = ((size_t)sv.base[slot] + r0 + r) * p.d;
            float s = 0.f;
            for (int c = lane; c < p.d; c += 64) {
                float x;
                if (p.dtype == 0) x = ((const float*)p.buf)[e0 + c];
                else {
                    uint16_t b = ((const uint16_t*)p.buf)[e0 + c];
                    x = p.dtype == 1 ? (float)__builtin_bit_cast(_Float16, b) : __uint_as_float((uint32_t)b << 16);
                }
                if (METRIC == 0) s = fmaf(ql[c], x, s);
                else { float df = ql[c] - x; s = fmaf(df, df, s); }
            }
            s = group_sum<64>(s);
            float ck = read_lane(METRIC == 0 ? s : -s, 0);
            if (ck >= top.thr) top.insert(ck, sv.grow[slot] + r0 + r, p.ids, p.kprime);
        }
    }
    finish_workgroup<KL>(top, p, m_key, m_row, qi);
}

// ---- shape selection ---------------------------------------------------------------------
// (lanes per row, 16-byte segments per lane, row groups in flight), keyed by the number of
// 16-byte chunks in a row.  About 24 KB of loads are in flight per wavefront.
ScanShape pick_scan_shape(int d, int dtype) {
    const int esz = dtype == 0 ? 4 : 2;
    const size_t row_bytes = (size_t)d * esz;
    if (row_bytes % 16 != 0) return ScanShape{0, 0, 0, 4};
    const int chunks = (int)(row_bytes / 16);
    struct Opt { int lpr, seg, u; };
    static const Opt opts[] = {{16, 1, 16}, {32, 1, 16}, {64, 1, 16}, {32, 3, 8}, {64, 2, 8},
                               {64, 3, 8},  {64, 4, 6},  {64, 8, 3}};
    int best = -1, best_waste = 1 << 30;
    for (int i = 0; i < (int)(sizeof(opts) / sizeof(opts[0])); ++i) {
        int cap = opts[i].lpr * opts[i].seg;
        if (cap < chunks) continue;
        int waste = cap - chunks;
        if (waste < best_waste) { best = i; best_waste = waste; }
    }
    if (best < 0) return ScanShape{0, 0, 0, 4};
    return ScanShape{opts[best].lpr, opts[best].seg, opts[best].u, opts[best].u * (64 / opts[best].lpr)};
}

template <typename T, int LPR, int SEG, int U>
static void launch_scan_shape(const ScanArgs& a, dim3 grid, size_t lds, int in_lds, hipStream_t s) {
    const bool big = a.kprime > 64;
    if (a.metric == 0) {
        if (big) hipLaunchKernelGGL((scan_kernel<T, LPR, SEG, U, 0, 2>), grid, dim3(kScanThreads), lds, s, a, in_lds);
        else hipLaunchKernelGGL((scan_kernel<T, LPR, SEG, U, 0, 1>), grid, dim3(kScanThreads), lds, s, a, in_lds);
    } else {
        if (big) hipLaunchKernelGGL((scan_kernel<T, LPR, SEG, U, 1, 2>), grid, dim3(kScanThreads), lds, s, a, in_lds);
        else hipLaunchKernelGGL((scan_kernel<T, LPR, SEG, U, 1, 1>), grid, dim3(kScanThreads), lds, s, a, in_lds);
    }
}

template <typename T>
static bool launch_scan_dtype(const ScanArgs& a, dim3 grid, size_t lds, int in_lds, hipStream_t s) {
    const int l = a.shape.lanes_per_row, g = a.shape.segments;
#define IVF_SHAPE(L, G, UU) if (l == L && g == G) { launch_scan_shape<T, L, G, UU>(a, grid, lds, in_lds, s); return true; }
    IVF_SHAPE(16, 1, 16) IVF_SHAPE(32, 1, 16) IVF_SHAPE(64, 1, 16) IVF_SHAPE(32, 3, 8)
    IVF_SHAPE(64, 2, 8) IVF_SHAPE(64, 3, 8) IVF_SHAPE(64, 4, 6) IVF_SHAPE(64, 8, 3)
#undef IVF_SHAPE
    return false;
}

hipError_t launch_scan(const ScanArgs& a, hipStream_t s) {
    const int in_lds = a.nprobe <= kScanLdsSlots;
    dim3 grid(a.grid, a.nq);
    const bool generic = a.shape.lanes_per_row == 0;
    size_t lds = scan_lds_bytes(a.nprobe, a.kprime, in_lds, generic ? a.d : 0);
    if (generic) {
        const bool big = a.kprime > 64;
        if (a.metric == 0) {
            if (big) hipLaunchKernelGGL((scan_generic_kernel<0, 2>), grid, dim3(kScanThreads), lds, s, a, in_lds);
            else hipLaunchKernelGGL((scan_generic_kernel<0, 1>), grid, dim3(kScanThreads), lds, s, a, in_lds);
        } else {
            if (big) hipLaunchKernelGGL((scan_generic_kernel<1, 2>), grid, dim3(kScanThreads), lds, s, a, in_lds);
            else hipLaunchKernelGGL((scan_generic_kernel<1, 1>), grid, dim3(kScanThreads), lds, s, a, in_lds);
        }
        return hipGetLastError();
    }
    bool ok = false;
    if (a.dtype == 0) ok = launch_scan_dtype<F32>(a, grid, lds, in_lds, s);
    else if (a.dtype == 1) ok = launch_scan_dtype<F16>(a, grid, lds, in_lds, s);
    else ok = launch_scan_dtype<BF16>(a, grid, lds, in_lds, s);
    if (!ok) return hipErrorInvalidValue;
    return hipGetLastError();
}

// =============================================================================================
// Merge (App. B: "this involves sorting"; Sec. 4.1 step 4: results of the GPU and the host part
// are merged on the GPU).  One workgroup per query: picks the kprime best fp32 candidates of all
// workgroup lists, re-scores them in fp64 from the stored rows, adds the host's candidates
// (already fp64), orders everything by (score, id) and writes the k nearest.
// =============================================================================================
__global__ __launch_bounds__(kSelectThreads) void merge_kernel(MergeArgs a) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh[8];
    __shared__ uint32_t c_row[kMaxKPrime];
    __shared__ double f_key[2 * kMaxKPrime];
    __shared__ int64_t f_id[2 * kMaxKPrime];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = lane_id(), wave = tid >> 6;
    const int qi = blockIdx.x;
    const uint32_t n = (uint32_t)a.nparts * a.kprime;
    const float* pk = a.part_key + (size_t)qi * n;
    const uint32_t* pr = a.part_row + (size_t)qi * n;
    const uint32_t kp = a.kprime;

    // 1. the kprime best fp32 keys (ascending radix key = best first)
    uint32_t mask, prefix, need, group;
    auto key_at = [&](uint32_t i) { return ~ordered(pk[i]); };
    block_radix_select<uint32_t>(key_at, n, kp, hist, sh, mask, prefix, need, group);
    if (tid == 0) sh[4] = 0;
    __syncthreads();
    const bool take_group = need == group;
    for (uint32_t i = tid; i < n; i += nt) {
        uint32_t hi = key_at(i) & mask;
        if ((hi < prefix || (take_group && hi == prefix)) && pr[i] != kNoRow) {
            uint32_t p = atomicAdd(&sh[4], 1u);
            c_row[p] = pr[i];
        }
    }
    __syncthreads();
    if (!take_group) {
        // boundary group of bit-identical fp32 keys: keep the `need` smallest ids, one at a time
        __shared__ unsigned long long best;
        long long last = -1;
        for (uint32_t it = 0; it < need; ++it) {
            if (tid == 0) best = ~0ull;
            __syncthreads();
            for (uint32_t i = tid; i < n; i += nt) {
                if ((key_at(i) & mask) == prefix && pr[i] != kNoRow) {
                    long long id = a.ids ? a.ids[pr[i]] : (long long)pr[i];
                    if (id > last) atomicMin(&best, ((unsigned long long)id << 0));
                }
            }
            __syncthreads();
            unsigned long long b = best;
            if (b == ~0ull) break;
            last = (long long)b;
            for (uint32_t i = tid; i < n; i += nt) {
                if ((key_at(i) & mask) == prefix && pr[i] != kNoRow) {
                    long long id = a.ids ? a.ids[pr[i]] : (long long)pr[i];
                    if (id == last) { uint32_t p = atomicAdd(&sh[4], 1u); if (p < kMaxKPrime) c_row[p] = pr[i]; }
                }
            }
            __syncthreads();
        }
    }
    __syncthreads();
    const uint32_t m = min(sh[4], (uint32_t)kMaxKPrime);

    // 2. fp64 re-score, one wavefront per candidate
    const float* q = a.q + (size_t)qi * a.d;
    const int np = a.nprobe;
    const int64_t* s_base = a.slots.base + (size_t)qi * np;
    const uint32_t* s_grow = a.slots.grow + (size_t)qi * np;
    const uint32_t* s_n = a.slots.nrows + (size_t)qi * np;
    for (uint32_t c = wave; c < m; c += nt / 64) {
        const uint32_t row = c_row[c];
        size_t brow = row;
        if (!a.identity) {
            // find the slot whose global row range holds `row`
            long long found = -1;
            for (int s0 = 0; s0 < np && found < 0; s0 += 64) {
                int s = s0 + lane;
                bool hit = s < np && row >= s_grow[s] && row - s_grow[s] < s_n[s];
                uint64_t b = __ballot(hit);
                if (b) found = s0 + __ffsll((long long)b) - 1;
            }
            brow = (size_t)(s_base[found] + (int64_t)(row - s_grow[found]));
        }
        double acc = 0.0;
        const size_t e0 = brow * (size_t)a.d;
        for (int t = lane; t < a.d; t += 64) {
            double x = (double)q[t];
            double y = widen(a.buf, a.dtype, e0 + t);
            if (a.metric == 0) acc = fma(x, y, acc);
            else { double df = x - y; acc = fma(df, df, acc); }
        }
        acc = wave_sum(acc);
        if (lane == 0) {
            f_key[c] = a.metric == 0 ? acc : -acc;
            f_id[c] = a.ids ? a.ids[row] : (int64_t)row;
        }
    }
    // 3. host candidates
    uint32_t nh = 0;
    if (a.host_cand) {
        nh = min((uint32_t)a.host_count[qi], kp);
        for (uint32_t i = tid; i < nh; i += nt) {
            f_key[m + i] = a.host_cand[(size_t)qi * kp + i].key;
            f_id[m + i] = a.host_cand[(size_t)qi * kp + i].id;
        }
    }
    __syncthreads();
    // 4. rank by counting; nearest first, ties by smaller id
    const uint32_t tot = m + nh;
    const int k = a.k;
    if ((uint32_t)tid < tot) {
        double mk = f_key[tid]; int64_t mi = f_id[tid];
        uint32_t rank = 0;
        for (uint32_t j = 0; j < tot; ++j) {
            double ok = f_key[j]; int64_t oi = f_id[j];
            rank += (ok > mk) || (ok == mk && oi < mi);
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

hipError_t launch_merge(const MergeArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(merge_kernel, dim3(a.nq), dim3(kSelectThreads), 0, s, a);
    return hipGetLastError();
}

// =============================================================================================
// Layout build (the contiguous cluster-major region of Sec. "Implementation Details"): input
// rows scattered to their positions, one wavefront per row, 16 bytes per lane when rows allow.
// =============================================================================================
__global__ void scatter_rows_kernel(const unsigned char* src, unsigned char* dst, const int64_t* pos,
                                    int64_t n, size_t row_bytes) {
    const int lane = lane_id();
    int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t i = wave; i < n; i += nwaves) {
        const unsigned char* s = src + (size_t)i * row_bytes;
        unsigned char* d = dst + (size_t)pos[i] * row_bytes;
        if (row_bytes % 16 == 0) {
            for (size_t o = (size_t)lane * 16; o < row_bytes; o += 1024) *(uint4*)(d + o) = *(const uint4*)(s + o);
        } else {
            for (size_t o = lane; o < row_bytes; o += 64) d[o] = s[o];
        }
    }
}

hipError_t launch_scatter_rows(const void* src, void* dst, const int64_t* pos, int64_t n,
                               size_t row_bytes, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 3) / 4;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(scatter_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       (const unsigned char*)src, (unsigned char*)dst, pos, n, row_bytes);
    return hipGetLastError();
}

}  // namespace ivf
