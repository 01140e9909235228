// Prefetching scheduler (TeleRAG, arxiv 2502.20969, Sec. 4.2 "Scheduling optimization for
// prefetching"): the queries of a global batch are grouped into micro-batches by a greedy search on
// squared L2 distance, so that the queries of one micro-batch want largely the same clusters.
// Two kernels: all pairwise distances, then the greedy pick.
#include "ivf_device.h"

namespace ivf {
using namespace dev;

// D[i][j] = sum over t of (q[i][t] - q[j][t])^2 in fp64, added term by term in index order with
// separately rounded multiply and add: the greedy pick compares these values, and a fixed order
// of operations makes its decisions reproducible down to exact ties.
// One workgroup per 16 x 16 tile of pairs; slabs of 64 components go through LDS.
constexpr int kPairTile = 16, kPairSlab = 64;

__global__ __launch_bounds__(256) void pair_dist_kernel(const float* q, int B, int d, double* D) {
    __shared__ float sa[kPairTile][kPairSlab + 1];
    __shared__ float sb[kPairTile][kPairSlab + 1];
    const int tid = threadIdx.x;
    const int ti = tid / kPairTile, tj = tid % kPairTile;
    const int i0 = blockIdx.y * kPairTile, j0 = blockIdx.x * kPairTile;
    double acc = 0.0;
    for (int k0 = 0; k0 < d; k0 += kPairSlab) {
        for (int e = tid; e < kPairTile * kPairSlab; e += 256) {
            const int r = e / kPairSlab, t = e % kPairSlab;
            const bool in_k = k0 + t < d;
            sa[r][t] = (in_k && i0 + r < B) ? q[(size_t)(i0 + r) * d + k0 + t] : 0.f;
            sb[r][t] = (in_k && j0 + r < B) ? q[(size_t)(j0 + r) * d + k0 + t] : 0.f;
        }
        __syncthreads();
        const int kn = min(kPairSlab, d - k0);
        for (int t = 0; t < kn; ++t) {
            const double df = (double)sa[ti][t] - (double)sb[tj][t];
            acc = __dadd_rn(acc, __dmul_rn(df, df));
        }
        __syncthreads();
    }
    if (i0 + ti < B && j0 + tj < B) D[(size_t)(i0 + ti) * B + j0 + tj] = acc;
}

// Greedy pick, one workgroup.  While queries remain: the remaining query of lowest index seeds a
// micro-batch; the m - 1 remaining queries nearest to it follow, nearest first, equal distances by
// lower index.  A distance is non-negative, so its bit pattern orders like its value.
constexpr int kSchedThreads = 1024, kSchedPerThread = 4;      // up to 4096 queries

struct Pick { unsigned long long key; uint32_t idx; };
__device__ __forceinline__ Pick better(const Pick& a, const Pick& b) {
    return (b.key < a.key || (b.key == a.key && b.idx < a.idx)) ? b : a;
}

__global__ __launch_bounds__(kSchedThreads) void greedy_groups_kernel(const double* D, int B, int m, int32_t* order) {
    __shared__ unsigned char taken[kSchedThreads * kSchedPerThread];
    __shared__ unsigned long long w_key[kSchedThreads / 64];
    __shared__ uint32_t w_idx[kSchedThreads / 64];
    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
    for (int i = tid; i < kSchedThreads * kSchedPerThread; i += kSchedThreads) taken[i] = i < B ? 0 : 1;
    __syncthreads();
    int pos = 0, cursor = 0;
    while (pos < B) {
        // the seed: seeds only ever move up, so the search resumes where the last one stopped
        while (taken[cursor]) ++cursor;            // uniform: every thread walks the same flags
        const int seed = cursor;
        __syncthreads();                           // everyone has read the flags
        if (tid == 0) { taken[seed] = 1; order[pos] = seed; }
        ++pos;
        unsigned long long mine[kSchedPerThread];
#pragma unroll
        for (int r = 0; r < kSchedPerThread; ++r) {
            const int j = tid + r * kSchedThreads;
            mine[r] = j < B ? (unsigned long long)__double_as_longlong(D[(size_t)seed * B + j]) : ~0ull;
        }
        __syncthreads();
        for (int slot = 1; slot < m && pos < B; ++slot) {
            Pick p{~0ull, 0xFFFFFFFFu};
#pragma unroll
            for (int r = 0; r < kSchedPerThread; ++r) {
                const int j = tid + r * kSchedThreads;
                if (j < B && !taken[j]) p = better(p, Pick{mine[r], (uint32_t)j});
            }
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) {
                Pick other;
                other.key = ((unsigned long long)(uint32_t)__shfl_xor((int)(uint32_t)(p.key >> 32), o) << 32) |
                            (uint32_t)__shfl_xor((int)(uint32_t)p.key, o);
                other.idx = (uint32_t)__shfl_xor((int)p.idx, o);
                p = better(p, other);
            }
            if (lane == 0) { w_key[wave] = p.key; w_idx[wave] = p.idx; }
            __syncthreads();
            if (tid == 0) {
                Pick best{w_key[0], w_idx[0]};
                for (int w = 1; w < kSchedThreads / 64; ++w) best = better(best, Pick{w_key[w], w_idx[w]});
                taken[best.idx] = 1;
                order[pos] = (int32_t)best.idx;
            }
            ++pos;
            __syncthreads();
        }
    }
}

hipError_t launch_schedule(const float* q_dev, int B, int d, int m, double* dist, int32_t* order, hipStream_t s) {
    if (B < 1 || B > kSchedThreads * kSchedPerThread || d < 1 || m < 1) return hipErrorInvalidValue;
    const int tiles = (B + kPairTile - 1) / kPairTile;
    hipLaunchKernelGGL(pair_dist_kernel, dim3(tiles, tiles), dim3(256), 0, s, q_dev, B, d, dist);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(greedy_groups_kernel, dim3(1), dim3(kSchedThreads), 0, s, dist, B, m, order);
    return hipGetLastError();
}

}  // namespace ivf
