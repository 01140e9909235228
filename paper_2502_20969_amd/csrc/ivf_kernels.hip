// HIP kernels of the IVF search path for gfx950 (wave64): coarse scoring, top-nprobe
// selection, list scan with per-workgroup top-k', and the fp64 re-score + merge.
// The operations are those of TeleRAG (arxiv 2502.20969) App. B: coarse search over the
// centroids, fine search over the rows of the selected clusters, k nearest by a sort.
#include "ivf_device.h"
#include "../../include/ivf.h"
#include <hip/hip_ext.h>
#include <algorithm>

namespace ivf {
using namespace dev;

// =============================================================================================
// Coarse scoring (App. B, first step): scores[q][j] = d(x_q, c_j) for every centroid, in fp64
// (products of fp32 values are exact in fp64, so the selection below sees the same order as a
// plain fp64 loop up to the last bits of the sums).
//
// Few queries: one wavefront per centroid row, all loads of a row and of the query requested
// at once; HBM-bound on the nlist*d*4 bytes of the centroid matrix, in practice one memory
// latency.  A batch of queries: a dense contraction Q x C^T on the fp64 matrix cores.
// =============================================================================================
constexpr int kCoarseRowMax = 16;          // batches below this use the row kernel
constexpr int kSelectWaveSortMax = 4096;   // select: register sorting path up to this many clusters

__global__ __launch_bounds__(256) void coarse_rows_kernel(CoarseArgs a) {
    const int lane = lane_id(), wave = wave_id();
    const int row = blockIdx.x * 4 + wave;
    if (row >= a.nlist) return;
    const float* c = a.centroids + (size_t)row * a.d;
#pragma unroll 1
    for (int qi = 0; qi < a.nq; ++qi) {
        const float* q = a.q + (size_t)qi * a.d;
        double acc = 0.0;
        if ((a.d & 3) == 0) {
#pragma unroll 1
            for (int t0 = lane * 4; t0 < a.d; t0 += 1024) {
                float4 cv[4], qv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int t = min(t0 + u * 256, a.d - 4);
                    cv[u] = *(const float4*)(c + t);
                    qv[u] = *(const float4*)(q + t);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (t0 + u * 256 < a.d) {
                        const float ce[4] = {cv[u].x, cv[u].y, cv[u].z, cv[u].w};
                        const float qe[4] = {qv[u].x, qv[u].y, qv[u].z, qv[u].w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const double x = (double)qe[e], y = (double)ce[e];
                            if (a.metric == 0) acc = fma(x, y, acc);
                            else { const double df = x - y; acc = fma(df, df, acc); }
                        }
                    }
                }
            }
        } else {
            for (int t = lane; t < a.d; t += 64) {
                const double x = (double)q[t], y = (double)c[t];
                if (a.metric == 0) acc = fma(x, y, acc);
                else { const double df = x - y; acc = fma(df, df, acc); }
            }
        }
        const double s = wave_sum(acc);
        if (lane == 0) a.scores[(size_t)qi * a.nlist + row] = s;
    }
}

// Q x C^T with v_mfma_f64_16x16x4_f64.  Operand layout of the instruction: lane l supplies
// A[i = l % 16][k = l / 16] and B[k = l / 16][j = l % 16]; result register r of lane l is
// C[i = 4 r + l / 16][j = l % 16].  A workgroup of four wavefronts covers (WQ * 32) queries by
// ((4 / WQ) * 32) centroids, each wavefront 32 x 32 as 2 x 2 instruction tiles; fp32 operand
// slabs of 32 k-values go through LDS (rows padded by 4 floats: the 64 lanes of a fragment
// read then fall on 64 different (bank, half) positions) and are widened on use.  For the
// squared distance the norms are accumulated beside the products: |q - c|^2 = |q|^2 + |c|^2 - 2 q.c.
typedef double double4_t __attribute__((ext_vector_type(4)));
constexpr int kCoarseKT = 32, kCoarseLd = kCoarseKT + 4;

template <int WQ>
__global__ __launch_bounds__(256) void coarse_mfma_kernel(CoarseArgs a) {
    constexpr int WC = 4 / WQ, TQ = WQ * 32, TC = WC * 32;
    __shared__ float sq[TQ * kCoarseLd];
    __shared__ float sc[TC * kCoarseLd];
    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
    const int q0 = blockIdx.y * TQ, c0 = blockIdx.x * TC;
    const int wq = (wave % WQ) * 32, wc = (wave / WQ) * 32;      // this wavefront's corner in the tile
    const int fi = lane & 15, fk = lane >> 4;
    double4_t acc[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] = double4_t{0.0, 0.0, 0.0, 0.0};
    double nq2[2] = {0.0, 0.0}, nc2[2] = {0.0, 0.0};
#pragma unroll 1
    for (int k0 = 0; k0 < a.d; k0 += kCoarseKT) {
        // slabs: 8 float4 per row
        for (int i = tid; i < TQ * 8; i += 256) {
            const int r = i >> 3, k4 = (i & 7) * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (q0 + r < a.nq && k0 + k4 < a.d) v = *(const float4*)(a.q + (size_t)(q0 + r) * a.d + k0 + k4);
            *(float4*)&sq[r * kCoarseLd + k4] = v;
        }
        for (int i = tid; i < TC * 8; i += 256) {
            const int r = i >> 3, k4 = (i & 7) * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c0 + r < a.nlist && k0 + k4 < a.d) v = *(const float4*)(a.centroids + (size_t)(c0 + r) * a.d + k0 + k4);
            *(float4*)&sc[r * kCoarseLd + k4] = v;
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < kCoarseKT; ks += 4) {
            double fa[2], fb[2];
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                fa[x] = (double)sq[(wq + x * 16 + fi) * kCoarseLd + ks + fk];
                fb[x] = (double)sc[(wc + x * 16 + fi) * kCoarseLd + ks + fk];
                nq2[x] = fma(fa[x], fa[x], nq2[x]);
                nc2[x] = fma(fb[x], fb[x], nc2[x]);
            }
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y)
                    acc[x][y] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[x], fb[y], acc[x][y], 0, 0, 0);
        }
        __syncthreads();
    }
    // norms: sum over the four k-groups of lanes; then lane l holds the norm of row l % 16
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        nq2[x] += __shfl_xor(nq2[x], 16); nq2[x] += __shfl_xor(nq2[x], 32);
        nc2[x] += __shfl_xor(nc2[x], 16); nc2[x] += __shfl_xor(nc2[x], 32);
    }
#pragma unroll
    for (int x = 0; x < 2; ++x) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = 4 * r + fk;                      // row of result register r inside the 16 x 16 tile
            const double qn = __shfl(nq2[x], i);
            const int qi = q0 + wq + x * 16 + i;
#pragma unroll
            for (int y = 0; y < 2; ++y) {
                const int cj = c0 + wc + y * 16 + fi;
                const double dot = acc[x][y][r];
                const double s = a.metric == 0 ? dot : fma(-2.0, dot, qn + nc2[y]);
                if (qi < a.nq && cj < a.nlist) a.scores[(size_t)qi * a.nlist + cj] = s;
            }
        }
    }
}

hipError_t launch_coarse(const CoarseArgs& a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
    if (a.nq < kCoarseRowMax || (a.d & 3) != 0) {
        IVF_LAUNCH(coarse_rows_kernel, dim3((a.nlist + 3) / 4), dim3(256), 0, s, e0, e1, a);
    } else if (a.nq < 48) {
        IVF_LAUNCH(coarse_mfma_kernel<1>, dim3((a.nlist + 127) / 128, (a.nq + 31) / 32), dim3(256), 0, s, e0, e1, a);
    } else {
        IVF_LAUNCH(coarse_mfma_kernel<2>, dim3((a.nlist + 63) / 64, (a.nq + 63) / 64), dim3(256), 0, s, e0, e1, a);
    }
    return hipGetLastError();
}

// =============================================================================================
// Top-nprobe selection (App. B: the L nearest centroids), ordered nearest first with ties by
// smaller cluster index, plus the tables the scan walks: per selected cluster ("slot") its
// placement and rows, and per scan workgroup its share of the rows.  One workgroup per query.
// =============================================================================================
__device__ __forceinline__ uint64_t coarse_key(double score, int metric) {
    uint64_t o = ordered(score);
    return metric == 0 ? ~o : o;       // ascending key = nearest first
}

// Fills keys/idx (LDS or global, `pad` entries) with the nprobe best (key, index) pairs sorted
// ascending.  Inlined once per memory kind so that LDS accesses compile to LDS instructions.
__device__ __forceinline__ void select_sorted(const SelectArgs& a, const double* sc, uint64_t* keys,
                                              uint32_t* idx, uint32_t pad, uint32_t* hist, uint32_t* sh) {
    const int tid = threadIdx.x, nt = blockDim.x;
    const uint32_t nlist = a.nlist, nprobe = a.nprobe;
    if (nlist <= pad) {
        // every centroid fits the sort: no selection pass needed
        for (uint32_t i = tid; i < pad; i += nt) {
            keys[i] = i < nlist ? coarse_key(sc[i], a.metric) : ~0ull;
            idx[i] = i < nlist ? i : 0xFFFFFFFFu;
        }
        __syncthreads();
    } else {
        // radix-select the nprobe best, then sort only those
        uint64_t mask, prefix; uint32_t need, group;
        auto key_at = [&](uint32_t i) { return coarse_key(sc[i], a.metric); };
        block_radix_select<uint64_t>(key_at, nlist, nprobe, hist, sh, mask, prefix, need, group);
        if (tid == 0) sh[4] = 0;
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
}

// The nprobe nearest by a bucket cut (see block_bucket_cut) over the high halves of the keys: the
// clusters that pass the cut (the nprobe nearest and a few more) are pooled with their full keys
// and each counts the pooled clusters ahead of it by (key, index); the first nprobe take their
// places in idx.  Exact, with no sorting network.  Returns false (for the whole workgroup) when
// more clusters pass than the pool holds (masses of equal scores); idx is then untouched.
constexpr int kSelectPoolCap = 1024;
constexpr int kSelectCutMax = 512;          // largest nprobe this path takes
__device__ __forceinline__ bool select_by_cut(const SelectArgs& a, const double* sc, uint32_t* idx, uint64_t* pool_key,
                                              uint32_t* pool_idx, uint32_t* hist, uint32_t* red, uint32_t* sh) {
    const int tid = threadIdx.x, nt = blockDim.x;
    const uint32_t nlist = a.nlist, nprobe = a.nprobe;
    auto key_at = [&](uint32_t i) { return coarse_key(sc[i], a.metric); };
    // larger = nearer; never 0, so that every cluster counts
    auto near_at = [&](uint32_t i) -> uint32_t { const uint32_t v = (uint32_t)(~key_at(i) >> 32); return v ? v : 1u; };
    if (tid == 0) sh[4] = 0;
    const BucketCut bc = block_bucket_cut(near_at, nlist, nprobe, hist, red);
    if (bc.passing > (uint32_t)kSelectPoolCap) return false;
    for (uint32_t i = tid; i < nlist; i += nt) {
        if (bc.pass(near_at(i))) {
            const uint32_t p = atomicAdd(&sh[4], 1u);
            pool_key[p] = key_at(i); pool_idx[p] = i;
        }
    }
    __syncthreads();
    const uint32_t cnt = sh[4];
#pragma unroll 1
    for (uint32_t t = tid; t < cnt; t += nt) {
        const uint64_t mk = pool_key[t];
        const uint32_t mi = pool_idx[t];
        uint32_t rank = 0;
        // eight others per pass, all read before any is compared
#pragma unroll 1
        for (uint32_t j0 = 0; j0 < cnt; j0 += 8) {
            uint64_t ok[8]; uint32_t oi[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) { const uint32_t j = min(j0 + u, cnt - 1); ok[u] = pool_key[j]; oi[u] = pool_idx[j]; }
#pragma unroll
            for (int u = 0; u < 8; ++u) rank += (uint32_t)(((ok[u] < mk) | ((ok[u] == mk) & (oi[u] < mi))) & (j0 + u < cnt));
        }
        if (rank < nprobe) idx[rank] = mi;
    }
    __syncthreads();
    return true;
}

__global__ __launch_bounds__(kSelectThreads) void select_kernel(SelectArgs a, uint32_t pad, int in_lds,
                                                                int prefix_in_lds, int by_cut) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh[8];
    __shared__ uint32_t red[96];
    __shared__ uint32_t scan_buf[kSelectThreads / 64 + 1];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int qi = blockIdx.x;
    const double* sc = a.scores + (size_t)qi * a.nlist;
    const uint32_t nprobe = a.nprobe;
    const size_t sort_bytes = in_lds ? (size_t)pad * 12 : 0;
    uint32_t* idx;
    if (in_lds && nprobe <= 64 && a.nlist <= kSelectWaveSortMax) {
        // Few clusters wanted from a small index.  Each score is cut down to a packed candidate:
        // the top 40 bits of its descending key image, then the complement of the cluster index
        // (larger = nearer; equal prefixes by smaller index).  The candidates are dealt to 64 or
        // 128 groups (a thread's go to the group of its lane); the nprobe-th largest group maximum
        // is not above the nprobe-th largest candidate, so the nprobe nearest are among the
        // candidates that reach its prefix: about nprobe (1 + nprobe / 128) of them when the
        // groups are unrelated to the scores.  Those are pooled; up to 64 are ordered by one
        // sort of wavefront 0, more by counting.  The order of the prefixes is the order of the
        // scores wherever prefixes differ, so the result is exact unless two prefixes tie among
        // the selected clusters or across the cut; then the exact general path below redoes the
        // selection, as it does when the pool overflows.
        uint64_t* keys = (uint64_t*)smem_raw;
        idx = (uint32_t*)(smem_raw + sizeof(uint64_t) * pad);
        const int lane = lane_id(), wave = wave_id(), nw = nt >> 6;
        Cand* pool = (Cand*)(((uintptr_t)(smem_raw + sort_bytes + (size_t)(nprobe + 1) * 4) + 15) & ~(uintptr_t)15);   // [nt]
        Cand* sel = pool + nt;                                  // [65] the nprobe best and the one after, when counted
        uint32_t* gmax = (uint32_t*)(sel + 66);                 // [2 * nt] halves of every thread's best candidate
        if (tid == 0) { sh[4] = 0; sh[6] = 0; }
        if (tid < 65) sel[tid] = 0;
        auto packed = [&](int i, double s) {
            return (~coarse_key(s, a.metric) & ~0xFFFFFFull) | (uint64_t)(0xFFFFFFu - (uint32_t)i);
        };
        // the first four scores of a thread are requested together and stay in registers
        Cand c4[4];
        {
            double s4[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) { const int i = tid + j * nt; s4[j] = i < a.nlist ? sc[i] : 0.0; }
#pragma unroll
            for (int j = 0; j < 4; ++j) { const int i = tid + j * nt; c4[j] = i < a.nlist ? packed(i, s4[j]) : (Cand)0; }
        }
        Cand mine = max(max(c4[0], c4[1]), max(c4[2], c4[3]));
#pragma unroll 1
        for (int i = tid + 4 * nt; i < a.nlist; i += nt) mine = max(mine, packed(i, sc[i]));
        gmax[2 * tid] = (uint32_t)mine; gmax[2 * tid + 1] = (uint32_t)(mine >> 32);
        __syncthreads();
        // more than 32 wanted: 128 groups, sorted by two wavefronts, keep the pool small
        const int gw = nprobe > 32 ? 2 : 1;
        Cand sorted = 0;
        if (wave < gw) {
            Cand g = 0;
#pragma unroll 4
            for (int w = wave; w < nw; w += gw) {
                const Cand o = ((Cand)gmax[2 * (w * 64 + lane) + 1] << 32) | gmax[2 * (w * 64 + lane)];
                g = max(g, o);
            }
            sorted = bitonic_sort64<true>(g);                                  // largest first
            if (wave == 1) pool[lane] = sorted;
        }
        if (gw == 2) {
            __syncthreads();
            if (wave == 0) sorted = merge_best64<true>(sorted, pool[lane]);
        }
        if (wave == 0 && lane == (int)nprobe - 1) { gmax[0] = (uint32_t)(sorted >> 24); gmax[1] = (uint32_t)(sorted >> 56); }   // 0: all pass
        __syncthreads();
        const uint64_t cut = ((uint64_t)gmax[1] << 32) | gmax[0];              // 40-bit prefix
        {
            auto offer = [&](Cand c) {
                const bool ok = c != 0 && (c >> 24) >= cut;
                const uint64_t bal = __ballot(ok);
                if (bal) {
                    uint32_t base = 0;
                    if (lane == 0) base = atomicAdd(&sh[4], (uint32_t)__popcll(bal));
                    base = read_lane(base, 0);
                    const uint32_t pos = base + __popcll(bal & ((1ull << lane) - 1ull));
                    if (ok && pos < (uint32_t)nt) pool[pos] = c;
                }
            };
#pragma unroll
            for (int j = 0; j < 4; ++j) offer(c4[j]);
#pragma unroll 1
            for (int i0 = 4 * nt; i0 < a.nlist; i0 += nt) { const int i = i0 + tid; offer(i < a.nlist ? packed(i, sc[i]) : (Cand)0); }
        }
        __syncthreads();
        const uint32_t cnt = sh[4];
        Cand half = 0;                       // 65 .. 128 pooled: the sorted half of wavefronts 0 and 1
        Cand* run2 = (Cand*)gmax;            // the cut has been read: the area is free
        if (__builtin_expect(cnt > (uint32_t)nt, 0)) {
            if (tid == 0) sh[6] = 1;                                            // pool overflow: masses of equal prefixes
        } else if (__builtin_expect(cnt > 128, 0)) {
            // each pooled candidate counts those ahead of it; the first nprobe + 1 take their places
            const Cand me = (uint32_t)tid < cnt ? pool[tid] : (Cand)0;
            uint32_t rank = 0;
#pragma unroll 1
            for (uint32_t j0 = 0; j0 < cnt; j0 += 8) {
                Cand o[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) o[u] = pool[min(j0 + u, cnt - 1)];
#pragma unroll
                for (int u = 0; u < 8; ++u) rank += (uint32_t)((o[u] > me) & (j0 + u < cnt));
            }
            if ((uint32_t)tid < cnt && rank <= nprobe) sel[rank] = me;
        } else if (cnt > 64) {
            if (wave < 2) {
                half = bitonic_sort64<true>((uint32_t)tid < cnt ? pool[tid] : (Cand)0);
                if (wave == 1) run2[lane] = half;
            }
        }
        __syncthreads();
        if (wave == 0 && sh[6] == 0) {
            Cand best, after;
            if (cnt <= 64) {
                const Cand sorted = bitonic_sort64<true>((uint32_t)lane < cnt ? pool[lane] : (Cand)0);
                after = nprobe < 64 ? read_lane(sorted, (int)(nprobe & 63)) : (Cand)0;
                best = lane < (int)nprobe ? sorted : (Cand)0;
            } else if (cnt <= 128) {
                Cand dropped;
                const Cand merged = merge_best64<true>(half, run2[lane], dropped);
                after = nprobe < 64 ? read_lane(merged, (int)(nprobe & 63)) : wave_max(dropped);
                best = lane < (int)nprobe ? merged : (Cand)0;
            } else {
                best = lane < (int)nprobe ? sel[lane] : (Cand)0;
                after = sel[nprobe];
            }
            const int ns = __popcll(__ballot(best != 0));                     // a prefix of the lanes
            const uint64_t next = ((uint64_t)(uint32_t)__shfl_down((int)(uint32_t)(best >> 32), 1) << 32) |
                                  (uint32_t)__shfl_down((int)(uint32_t)best, 1);
            const bool adjacent = lane + 1 < ns && (best >> 24) == (next >> 24);
            const bool cut_tie = ns > 0 && after != 0 && (after >> 24) == (read_lane(best, max(ns - 1, 0)) >> 24);
            const bool redo = __ballot(adjacent) != 0 || cut_tie;
            if (lane == 0) sh[6] = redo;
            if (!redo && lane < (int)pad) idx[lane] = best != 0 ? 0xFFFFFFu - (uint32_t)(best & 0xFFFFFFull) : 0xFFFFFFFFu;
        }
        __syncthreads();
        if (__builtin_expect(sh[6] != 0, 0)) select_sorted(a, sc, keys, idx, pad, hist, sh);
    } else if (in_lds) {
        uint64_t* keys = (uint64_t*)smem_raw;
        idx = (uint32_t*)(smem_raw + sizeof(uint64_t) * pad);
        bool done = false;
        if (by_cut) {
            uint64_t* pool_key = (uint64_t*)(((uintptr_t)(smem_raw + sort_bytes + (size_t)(nprobe + 1) * 4) + 15) & ~(uintptr_t)15);
            done = select_by_cut(a, sc, idx, pool_key, (uint32_t*)(pool_key + kSelectPoolCap), hist, red, sh);
        }
        if (!done) {
            __syncthreads();
            select_sorted(a, sc, keys, idx, pad, hist, sh);
        }
    } else {
        uint64_t* keys = a.sort_keys + (size_t)qi * pad;
        idx = a.sort_idx + (size_t)qi * pad;
        select_sorted(a, sc, keys, idx, pad, hist, sh);
    }

    // slot tables: per selected cluster its placement and its rows
    const int64_t* off = a.off;
    int64_t* s_base = a.slots.base + (size_t)qi * nprobe;
    uint32_t* s_grow = a.slots.grow + (size_t)qi * nprobe;
    uint32_t* s_n = a.slots.nrows + (size_t)qi * nprobe;
    uint32_t* s_rp = a.slots.rprefix + (size_t)qi * (nprobe + 1);
    uint32_t* l_rp = (uint32_t*)(smem_raw + sort_bytes);     // LDS copy of the row prefix
    uint32_t carry = 0;
    // one selected cluster: its table entries; returns the rows it contributes to the scan
    auto fill_slot = [&](uint32_t i) -> uint32_t {
        uint32_t c = in_lds ? ((uint32_t*)(smem_raw + sizeof(uint64_t) * pad))[i] : idx[i];
        a.probe[(size_t)qi * nprobe + i] = (int32_t)c;
        int64_t lo = off[c];
        uint32_t n = (uint32_t)(off[c + 1] - lo);
        int64_t ro = a.res_off[c];
        s_base[i] = ro;
        s_grow[i] = (uint32_t)lo;
        s_n[i] = n;
        if (a.used && ro >= 0) a.used[c] = 1u;            // cache bookkeeping: resident and selected
        return ro >= 0 ? n : 0;
    };
    if (nprobe <= 64) {
        // the whole table fits one wavefront: prefix inside it, no LDS round trips
        if (wave_id() == 0) {
            const uint32_t i = (uint32_t)tid;
            const uint32_t rows = i < nprobe ? fill_slot(i) : 0;
            uint32_t incl = rows;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                uint32_t up = __shfl_up(incl, o);
                if (tid >= o) incl += up;
            }
            if (i < nprobe) {
                s_rp[i] = incl - rows;
                if (prefix_in_lds) l_rp[i] = incl - rows;
            }
            const uint32_t total = read_lane(incl, 63);
            if (tid == 0) {
                scan_buf[0] = total;
                s_rp[nprobe] = total;
                if (prefix_in_lds) l_rp[nprobe] = total;
                if (a.rows_counter) atomicAdd(a.rows_counter, (unsigned long long)total);
            }
        }
        __syncthreads();
        carry = scan_buf[0];
    } else {
        for (uint32_t base = 0; base < nprobe; base += nt) {
            uint32_t i = base + tid;
            uint32_t rows = i < nprobe ? fill_slot(i) : 0;
            // block-wide exclusive scan of `rows`
            uint32_t incl = rows;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                uint32_t up = __shfl_up(incl, o);
                if ((tid & 63) >= o) incl += up;
            }
            if ((tid & 63) == 63) scan_buf[tid >> 6] = incl;
            __syncthreads();
            uint32_t wave_off = 0, total = 0;
#pragma unroll
            for (int w = 0; w < kSelectThreads / 64; ++w) {        // all sums read at once
                const uint32_t v = w < nt / 64 ? scan_buf[w] : 0;
                total += v;
                wave_off += w < (tid >> 6) ? v : 0;
            }
            if (i < nprobe) {
                uint32_t ex = carry + wave_off + incl - rows;
                s_rp[i] = ex;
                if (prefix_in_lds) l_rp[i] = ex;
            }
            carry += total;
            __syncthreads();
        }
        if (tid == 0) {
            s_rp[nprobe] = carry;
            if (prefix_in_lds) l_rp[nprobe] = carry;
            if (a.rows_counter) atomicAdd(a.rows_counter, (unsigned long long)carry);
        }
        __syncthreads();
    }

    // workgroup shares: rows split evenly, each share starting inside some slot
    const uint32_t R = carry;
    const uint32_t per = R / (uint32_t)a.grid, extra = R % (uint32_t)a.grid;
    const uint32_t* rp = prefix_in_lds ? l_rp : s_rp;
    for (int b = tid; b < (nprobe > kLaneTableSlots ? a.grid : 0); b += nt) {   // few slots: the scan finds its share itself
        WgDesc ds;
        ds.r_begin = per * (uint32_t)b + min((uint32_t)b, extra);        // the first `extra` shares get one more row
        ds.r_end = per * (uint32_t)(b + 1) + min((uint32_t)(b + 1), extra);
        uint32_t slot = 0;
        if (ds.r_begin < ds.r_end) {
            uint32_t lo = 0, hi = nprobe;        // invariant: rp[lo] <= r_begin < rp[hi]
            while (hi - lo > 1) {
                uint32_t mid = (lo + hi) >> 1;
                if (rp[mid] <= ds.r_begin) lo = mid; else hi = mid;
            }
            slot = lo;
        }
        ds.slot = slot;
        ds.slot_rbegin = rp[slot];
        ds.slot_rend = rp[slot + 1];
        ds.slot_grow = s_grow[slot];
        ds.slot_base = s_base[slot];
        a.desc[(size_t)qi * a.grid + b] = ds;
    }
}

static uint32_t next_pow2(uint32_t v) { uint32_t p = 1; while (p < v) p <<= 1; return p; }

// power-of-two length of the select kernel's sort array for (nlist, nprobe)
uint32_t select_sort_pad(int nlist, int nprobe) {
    uint32_t full = next_pow2((uint32_t)nlist), part = next_pow2((uint32_t)nprobe);
    return part < full ? part : full;     // sort only the selected clusters when that is fewer
}

hipError_t launch_select(const SelectArgs& a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
    uint32_t pad = select_sort_pad(a.nlist, a.nprobe);
    int in_lds = pad <= (uint32_t)kSortLdsCap;
    int prefix_in_lds = a.nprobe <= kPrefixLdsCap;
    // a workgroup with one wavefront per SIMD issues fastest when there is little work per thread
    const int threads = a.nlist <= 1024 && a.grid <= 1024 ? 256 : kSelectThreads;
    size_t lds = (in_lds ? (size_t)pad * 12 : 0) + (prefix_in_lds ? (size_t)(a.nprobe + 1) * 4 : 0);
    const bool wave_sort = in_lds && a.nprobe <= 64 && a.nlist <= kSelectWaveSortMax;
    const int by_cut = in_lds && !wave_sort && a.nprobe <= kSelectCutMax;
    if (wave_sort) lds += 16 + (size_t)threads * 8 + 66 * 8 + (size_t)threads * 8;      // pool, the ranked few, the threads' best
    if (by_cut) lds += 16 + (size_t)kSelectPoolCap * 12;
    IVF_LAUNCH(select_kernel, dim3(a.nq), dim3(threads), lds, s, e0, e1, a, pad, in_lds, prefix_in_lds, by_cut);
    return hipGetLastError();
}

// =============================================================================================
// List scan (App. B, second step): d(x, y) for every row y of every selected, resident list,
// reduced in the kernel to the best rows each wavefront saw.  HBM-bound: each row is read once
// with 16-byte streaming loads; only candidate lists are written.
//
// A row is covered by LPR lanes with SEG 16-byte loads each, so one wavefront instruction
// covers 64/LPR rows; a batch is U such row groups; each wavefront has kScanBatches batches in
// flight (one: a compute unit's eight wavefronts overlap each other).  The resident rows of
// a query's clusters form one sequence.  With up to kLaneTableSlots selected clusters the
// sequence is cut into windows of one batch and wavefront w of all W takes the windows
// w, w + W, ...: every wavefront then reads the same mix of addresses.  With more clusters the
// sequence is split evenly over the workgroups (the select kernel wrote where each share begins)
// and inside a workgroup over its wavefronts.
//
// Every wavefront writes its own candidate list (kCandSlots per list, unordered, 0 = empty) and
// the list's best entry again into a dense array of heads: no LDS, no barrier.
// =============================================================================================
// Position of a wavefront in the row sequence of its query.
struct Cursor {
    uint32_t r, r_end;           // next row and end of the current range (a window, or the wavefront's share)
    uint32_t win, win_step;      // windows: start of the current one, distance to the next (0: one contiguous range)
    uint32_t total;              // rows in the sequence (windows only)
    uint32_t slot, s_rb, s_re;   // current slot and its row range
    uint32_t s_grow;
    int64_t s_base;
};

struct Batch {
    const unsigned char* rows;   // first row of the batch in the device buffer
    uint32_t nr;                 // rows in the batch (0: none left)
    uint32_t grow;               // global row of the first row
};

// With at most kLaneTableSlots selected clusters a wavefront keeps the query's slot table in its
// lanes: lane i holds the end of slot i in the row sequence, its first global row and its place
// in the device buffer.  Finding the slot of a row is then one ballot, and stepping to the next
// slot costs no memory access.
struct LaneTable {
    bool on;
    int nprobe;
    uint32_t end, grow;
    int64_t base;
    __device__ __forceinline__ void load(const ScanArgs& p, int qi) {
        on = p.nprobe <= kLaneTableSlots;
        nprobe = p.nprobe;
        end = 0; grow = 0; base = 0;
        const int lane = lane_id();
        if (on && lane < p.nprobe) {
            const size_t o = (size_t)qi * p.nprobe + lane;
            end = p.slots.rprefix[o + qi + 1];
            grow = p.slots.grow[o];
            base = p.slots.base[o];
        }
    }
    __device__ __forceinline__ uint32_t total() const { return read_lane(end, nprobe - 1); }
    // points the cursor at the slot that holds row c.r (c.r below the total)
    __device__ __forceinline__ void seek(Cursor& c) const {
        const int slot = __popcll(__ballot(lane_id() < nprobe && end <= c.r));     // ends are non-decreasing
        c.slot = (uint32_t)slot;
        c.s_rb = slot ? read_lane(end, slot - 1) : 0u;
        c.s_re = read_lane(end, slot);
        c.s_grow = read_lane(grow, slot);
        c.s_base = (int64_t)(((uint64_t)read_lane((uint32_t)((uint64_t)base >> 32), slot) << 32) | read_lane((uint32_t)base, slot));
    }
};

__device__ __forceinline__ Batch next_batch(Cursor& c, const ScanArgs& p, int qi, int rows_per_batch,
                                            size_t row_bytes, const LaneTable& tab) {
    Batch b{nullptr, 0, 0};
    if (c.r >= c.r_end) {
        if (c.win_step == 0) return b;
        if (c.total - c.win <= c.win_step) { c.win_step = 0; return b; }
        c.win += c.win_step;                 // the wavefront's next window
        c.r = c.win;
        c.r_end = c.total - c.win < (uint32_t)rows_per_batch ? c.total : c.win + (uint32_t)rows_per_batch;
    }
    if (tab.on) {
        if (c.r >= c.s_re) tab.seek(c);
    } else {
        while (c.r >= c.s_re) {      // step to the slot that holds row r (skips empty / absent lists)
            c.slot += 1;
            const size_t o = (size_t)qi * p.nprobe + c.slot;
            c.s_rb = c.s_re;
            c.s_re = p.slots.rprefix[o + qi + 1];
            c.s_grow = p.slots.grow[o];
            c.s_base = p.slots.base[o];
        }
    }
    const uint32_t in_slot = c.r - c.s_rb;
    b.nr = min((uint32_t)rows_per_batch, min(c.r_end, c.s_re) - c.r);      // a window that crosses into the next slot comes in two batches
    b.rows = (const unsigned char*)p.buf + ((size_t)c.s_base + in_slot) * row_bytes;
    b.grow = c.s_grow + in_slot;
    c.r += b.nr;
    return b;
}

__device__ __forceinline__ Cursor start_cursor(const ScanArgs& p, int qi, const LaneTable& tab, int rows_per_batch) {
    const int wave = wave_id();
    Cursor c;
    c.win = 0; c.win_step = 0; c.total = 0;
    if (tab.on) {
        const uint32_t R = tab.total();
        const uint32_t w = blockIdx.x * kScanWaves + (uint32_t)wave;
        c.total = R;
        c.win = w * (uint32_t)rows_per_batch;
        c.win_step = (uint32_t)p.grid * kScanWaves * (uint32_t)rows_per_batch;
        c.r = min(c.win, R);
        c.r_end = R - c.r < (uint32_t)rows_per_batch ? R : c.r + (uint32_t)rows_per_batch;
        c.slot = 0; c.s_rb = 0; c.s_re = 0; c.s_grow = 0; c.s_base = 0;
        if (c.r >= c.r_end) c.win_step = 0;        // beyond the last window: nothing to do
        return c;
    }
    const WgDesc ds = p.desc[(size_t)qi * p.grid + blockIdx.x];
    const uint32_t cnt = ds.r_end - ds.r_begin;
    c.r = ds.r_begin + (uint32_t)((uint64_t)cnt * wave / kScanWaves);
    c.r_end = ds.r_begin + (uint32_t)((uint64_t)cnt * (wave + 1) / kScanWaves);
    c.slot = ds.slot; c.s_rb = ds.slot_rbegin; c.s_re = ds.slot_rend;
    c.s_grow = ds.slot_grow; c.s_base = ds.slot_base;
    return c;
}

// What a wavefront leaves behind: its candidates as a list of 64 * KL entries (the sorted list when it has one,
// else the loose candidates as they stand) and the best of them as the list's head.
template <int KL>
__device__ __forceinline__ void write_wave_list(WaveTopK<KL, false>& top, const ScanArgs& p, int qi) {
    const int lane = lane_id();
    const size_t list = ((size_t)qi * p.grid + blockIdx.x) * kScanWaves + (size_t)wave_id();
    Cand* out = p.part + list * (size_t)(64 * KL);
    const bool has_list = read_lane(top.top[0], 0) != 0;
    Cand head;
    if (KL == 1 && !has_list) {
        const Cand c = lane < top.pcount ? top.pend : (Cand)0;
        out[lane] = c;
        head = wave_max(c);
    } else {
        top.flush(p.kprime);
#pragma unroll
        for (int j = 0; j < KL; ++j) {
            const int e = j * 64 + lane;
            out[e] = e < p.kprime ? top.top[j] : (Cand)0;
        }
        head = read_lane(top.top[0], 0);
    }
    if (lane == 0) p.heads[list] = head;
}

template <typename T, int LPR, int SEG, int U, int METRIC, int KL>
__global__ __launch_bounds__(kScanThreads) void scan_kernel(ScanArgs p) {
    constexpr int EPL = T::kPerLoad;
    constexpr int RPI = 64 / LPR;
    constexpr int RPB = U * RPI;
    const int lane = lane_id();
    const int sub = lane % LPR, rsel = lane / LPR;
    const int qi = blockIdx.y;
    const size_t row_bytes = (size_t)p.d * T::kBytes;

    // This lane's slice of the query (rows of this kernel are whole 16-byte chunks, so d is a
    // multiple of EPL).  It is requested right AFTER the tables: loads return in order, and the
    // tables decide where the rows are, so nothing should arrive before them; the query is needed
    // only when the first rows are there.  (Measured: query first 16.8 us, tables first 16.5,
    // query after the first rows 16.6 - 16.9.)
    float qv[SEG][EPL];
    const float* q = p.q + (size_t)qi * p.d;
    auto load_query = [&]() {
#pragma unroll
        for (int sg = 0; sg < SEG; ++sg) {
            const int col = (sg * LPR + sub) * EPL;
#pragma unroll
            for (int e = 0; e < EPL; e += 4) {
                float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
                if (col < p.d) t = *(const float4*)(q + col + e);
                qv[sg][e] = t.x; qv[sg][e + 1] = t.y; qv[sg][e + 2] = t.z; qv[sg][e + 3] = t.w;
            }
        }
    };

    LaneTable tab;
    tab.load(p, qi);
    load_query();
    Cursor cur = start_cursor(p, qi, tab, RPB);

    WaveTopK<KL, false> top;
    top.init();

    // `tie` receives the global row of batch row `lane` (lanes < RPB): equal keys come out by smaller row
    auto issue = [&](const Batch& b, uint4 (&v)[U][SEG], uint32_t& tie) {
        tie = b.grow + min((uint32_t)lane, b.nr - 1);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t r = min((uint32_t)(u * RPI + rsel), b.nr - 1);   // rows past the end re-read the last one
            const unsigned char* rp = b.rows + (size_t)r * row_bytes;
#pragma unroll
            for (int sg = 0; sg < SEG; ++sg) {
                int col = (sg * LPR + sub) * EPL;
                if (col < p.d) v[u][sg] = load_stream16(rp + (size_t)col * T::kBytes);
                else v[u][sg] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto consume = [&](const Batch& b, const uint4 (&v)[U][SEG], uint32_t tie) {
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
            s = group_total_last_lane<LPR>(s);
            acc[u] = METRIC == 0 ? s : -s;        // key: larger is nearer
        }
        // almost every row fails the threshold: one ballot decides whether to look closer
        bool any = false;
        const bool leader = sub == LPR - 1;
#pragma unroll
        for (int u = 0; u < U; ++u) any |= leader && (uint32_t)(u * RPI + rsel) < b.nr && acc[u] >= top.thr;
        if (__ballot(any)) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int j = 0; j < RPI; ++j) {
                    const uint32_t r = u * RPI + j;
                    const float ck = read_lane(acc[u], j * LPR + LPR - 1);
                    if (r < b.nr && ck >= top.thr) top.push(ck, read_lane(tie, (int)r));
                }
            }
            if (top.pcount > 64 - RPB) top.flush(p.kprime);   // room for a whole batch stays free
        }
    };

    // kScanBatches batches in flight: the oldest is consumed, its buffer takes the next one
    uint4 v[kScanBatches][U][SEG];
    uint32_t tie[kScanBatches];
    Batch bt[kScanBatches];
#pragma unroll
    for (int i = 0; i < kScanBatches; ++i) {
        tie[i] = 0;
        bt[i] = next_batch(cur, p, qi, RPB, row_bytes, tab);
        if (bt[i].nr) issue(bt[i], v[i], tie[i]);
    }
    bool more = true;
    while (more) {
#pragma unroll
        for (int i = 0; i < kScanBatches; ++i) {
            if (bt[i].nr == 0) { more = false; break; }     // batches arrive in order: an empty buffer ends the walk
            consume(bt[i], v[i], tie[i]);
            bt[i] = next_batch(cur, p, qi, RPB, row_bytes, tab);
            if (bt[i].nr) issue(bt[i], v[i], tie[i]);
        }
    }
    write_wave_list<KL>(top, p, qi);
}

// Fallback for any d and any row alignment: element-wise loads, query in LDS, 4 rows per batch.
template <int METRIC, int KL>
__global__ __launch_bounds__(kScanThreads) void scan_generic_kernel(ScanArgs p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = lane_id();
    const int qi = blockIdx.y;
    float* ql = (float*)smem;
    for (int i = threadIdx.x; i < p.d; i += blockDim.x) ql[i] = p.q[(size_t)qi * p.d + i];
    __syncthreads();
    const int esz = p.dtype == 0 ? 4 : 2;
    const size_t row_bytes = (size_t)p.d * esz;
    LaneTable tab;
    tab.load(p, qi);
    Cursor cur = start_cursor(p, qi, tab, 4);
    WaveTopK<KL, false> top;
    top.init();
    for (Batch b = next_batch(cur, p, qi, 4, row_bytes, tab); b.nr; b = next_batch(cur, p, qi, 4, row_bytes, tab)) {
        for (uint32_t r = 0; r < b.nr; ++r) {
            const unsigned char* rp = b.rows + (size_t)r * row_bytes;
            float s = 0.f;
            for (int c = lane; c < p.d; c += 64) {
                float x;
                if (p.dtype == 0) x = ((const float*)rp)[c];
                else {
                    uint16_t h = ((const uint16_t*)rp)[c];
                    x = p.dtype == 1 ? (float)__builtin_bit_cast(_Float16, h) : __uint_as_float((uint32_t)h << 16);
                }
                if (METRIC == 0) s = fmaf(ql[c], x, s);
                else { float df = ql[c] - x; s = fmaf(df, df, s); }
            }
            s = group_total_last_lane<64>(s);
            float ck = read_lane(METRIC == 0 ? s : -s, 63);
            if (ck >= top.thr) {
                top.push(ck, b.grow + r);
                if (top.pcount == 64) top.flush(p.kprime);
            }
        }
    }
    write_wave_list<KL>(top, p, qi);
}

// ---- shape selection ---------------------------------------------------------------------
// (lanes per row, 16-byte segments per lane, row groups per batch), keyed by the number of
// 16-byte chunks in a row.  A batch is about 6 KB and a wavefront has one in flight: with eight
// wavefronts per compute unit that keeps the memory path busy, and measured against two batches
// of 12 KB in flight it ends every scan about a microsecond earlier (shorter queues, a finer
// grain at the end).
struct ShapeOpt { int lpr, seg, u; };
static const ShapeOpt kShapes[] = {{16, 1, 6}, {32, 1, 6}, {64, 1, 6}, {32, 3, 2}, {64, 2, 3},
                                   {64, 3, 2}, {64, 4, 2}, {64, 8, 1}};

ScanShape pick_scan_shape(int d, int dtype) {
    const int esz = dtype == 0 ? 4 : 2;
    const size_t row_bytes = (size_t)d * esz;
    if (row_bytes % 16 != 0) return ScanShape{0, 0, 0, 4};
    const int chunks = (int)(row_bytes / 16);
    int best = -1, best_waste = 1 << 30;
    for (int i = 0; i < (int)(sizeof(kShapes) / sizeof(kShapes[0])); ++i) {
        int cap = kShapes[i].lpr * kShapes[i].seg;
        if (cap < chunks) continue;
        int waste = cap - chunks;
        if (waste < best_waste) { best = i; best_waste = waste; }
    }
    if (best < 0) return ScanShape{0, 0, 0, 4};
    return ScanShape{kShapes[best].lpr, kShapes[best].seg, kShapes[best].u,
                     kShapes[best].u * (64 / kShapes[best].lpr)};
}

typedef void (*ScanFn)(ScanArgs);

template <typename T, int LPR, int SEG, int U>
static ScanFn scan_fn_shape(int metric, bool big) {
    if (metric == 0) return big ? (ScanFn)scan_kernel<T, LPR, SEG, U, 0, 2> : (ScanFn)scan_kernel<T, LPR, SEG, U, 0, 1>;
    return big ? (ScanFn)scan_kernel<T, LPR, SEG, U, 1, 2> : (ScanFn)scan_kernel<T, LPR, SEG, U, 1, 1>;
}

template <typename T>
static ScanFn scan_fn_dtype(const ScanShape& sh, int metric, bool big) {
    const int l = sh.lanes_per_row, g = sh.segments;
#define IVF_SHAPE(L, G, UU) if (l == L && g == G) return scan_fn_shape<T, L, G, UU>(metric, big);
    IVF_SHAPE(16, 1, 6) IVF_SHAPE(32, 1, 6) IVF_SHAPE(64, 1, 6) IVF_SHAPE(32, 3, 2)
    IVF_SHAPE(64, 2, 3) IVF_SHAPE(64, 3, 2) IVF_SHAPE(64, 4, 2) IVF_SHAPE(64, 8, 1)
#undef IVF_SHAPE
    return nullptr;
}

static ScanFn scan_fn(const ScanShape& sh, int dtype, int metric, int kprime) {
    const bool big = kprime > 64;
    if (sh.lanes_per_row == 0) {
        if (metric == 0) return big ? (ScanFn)scan_generic_kernel<0, 2> : (ScanFn)scan_generic_kernel<0, 1>;
        return big ? (ScanFn)scan_generic_kernel<1, 2> : (ScanFn)scan_generic_kernel<1, 1>;
    }
    if (dtype == 0) return scan_fn_dtype<F32>(sh, metric, big);
    if (dtype == 1) return scan_fn_dtype<F16>(sh, metric, big);
    return scan_fn_dtype<BF16>(sh, metric, big);
}

static size_t scan_lds_bytes(const ScanShape& sh, int d) {
    return sh.lanes_per_row == 0 ? (size_t)d * 4 : 0;      // only the fallback kernel stages the query
}

float scan_error_coef(const ScanShape& shape, int d, int dtype, int metric) {
    // roundings on the longest path of one row's sum: the fused multiply-adds of a lane, then the tree over the lanes
    int terms;
    if (shape.lanes_per_row == 0) terms = (d + 63) / 64 + 6;
    else {
        int tree = 0;
        for (int l = shape.lanes_per_row; l > 1; l >>= 1) ++tree;
        terms = shape.segments * (dtype == 0 ? 4 : 8) + tree;
    }
    if (metric != 0) terms += 2;          // the difference is rounded before it is squared
    return 1.05f * (float)(terms + 2) * 0x1p-24f;
}

int scan_resident_grid(const ScanShape& shape, int dtype, int metric, int kprime, int d, int n_cu) {
    ScanFn fn = scan_fn(shape, dtype, metric, kprime);
    if (!fn) return n_cu;
    int per_cu = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)fn, kScanThreads,
                                                                scan_lds_bytes(shape, d));
    if (e != hipSuccess || per_cu < 1) per_cu = 1;
    if (per_cu > kScanMaxWgPerCu) per_cu = kScanMaxWgPerCu;
    return per_cu * n_cu;
}

hipError_t launch_scan(const ScanArgs& a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
    ScanFn fn = scan_fn(a.shape, a.dtype, a.metric, a.kprime);
    if (!fn) return hipErrorInvalidValue;
    dim3 grid(a.grid, a.nq);
    IVF_LAUNCH(fn, grid, dim3(kScanThreads), scan_lds_bytes(a.shape, a.d), s, e0, e1, a);
    return hipGetLastError();
}

// =============================================================================================
// Merge (App. B: "this involves sorting"; Sec. 4.1 step 4: results of the GPU and the host part
// are merged on the GPU).  One workgroup per query: finds the kprime best fp32 candidates of
// all workgroup lists, re-scores those rows in fp64 from the stored rows, adds the host's
// candidates (already fp64), orders everything by (score, id) and writes the k nearest.
// =============================================================================================
constexpr int kMergeCandCap = 4096;    // candidates the fast path can pool
constexpr int kMergeQlistCap = 1024;   // lists the fast path can visit
constexpr int kMergeFastThreads = 1024;

struct MergeLds {
    uint32_t gmax[kMergeFastThreads];      // fast path: the largest head key of every thread's share
    uint32_t hist[256];                    // general path: digit counts of the radix select
    uint32_t sh[8];
    Cand c_cand[kMaxKPrime];
    double f_key[2 * kMaxKPrime];
    int64_t f_id[2 * kMaxKPrime];
};

// The kprime best of `cnt` pooled candidates (cnt above 64) into L.c_cand, their number into
// L.sh[4].  The usual search pools fewer than 64 and never comes here.
__device__ __forceinline__ void rank_pool(Cand* pool, uint32_t cnt, int kp, MergeLds& L) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = lane_id(), wave = wave_id(), nw = nt >> 6;
    if (cnt <= (uint32_t)nt) {
        // each counts the candidates ahead of it (eight per pass, all read before any is
        // compared) and the first kprime take their places
        const Cand mine = (uint32_t)tid < cnt ? pool[tid] : (Cand)0;
        uint32_t rank = 0;
#pragma unroll 1
        for (uint32_t j0 = 0; j0 < cnt; j0 += 8) {
            Cand o[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) o[u] = pool[min(j0 + u, cnt - 1)];
#pragma unroll
            for (int u = 0; u < 8; ++u) rank += (uint32_t)((o[u] > mine) & (j0 + u < cnt));
        }
        if ((uint32_t)tid < cnt && rank < (uint32_t)kp) L.c_cand[rank] = mine;
        __syncthreads();
        if (tid == 0) L.sh[4] = min(cnt, (uint32_t)kp);
        __syncthreads();
        return;
    }
    // many: sort the pooled candidates in chunks of 64, merge the chunks
    const int nchunks = (int)((cnt + 63) / 64);
#pragma unroll 1
    for (int c = wave; c < nchunks; c += nw) {
        const uint32_t e = c * 64 + lane;
        pool[e] = bitonic_sort64<true>(e < cnt ? pool[e] : (Cand)0);
    }
    __syncthreads();
    if (wave == 0) {
        Cand top = pool[lane];
#pragma unroll 1
        for (int c = 1; c < nchunks; ++c) top = merge_best64<true>(top, pool[c * 64 + lane]);
        const bool ok = lane < kp && top != 0;          // valid entries form a prefix
        if (ok) L.c_cand[lane] = top;
        const uint32_t m = (uint32_t)__popcll(__ballot(ok));
        if (lane == 0) L.sh[4] = m;
    }
    __syncthreads();
}

// Fast path (kprime <= 64).  The scan left one unordered list of `slots` candidates per wavefront
// and each list's best entry in `heads` (0: empty list).  Candidates are distinct.  The heads are
// dealt to 64 groups (a thread's heads go to the group of its lane); the kprime-th largest group
// maximum T is not above the kprime-th largest head, so at least kprime candidates reach T and the
// kprime best overall are among those that do, in lists whose head does.  With heads spread at
// random over the groups, about kprime (1 + kprime / 128) heads reach T.  The passing entries of
// those lists are pooled; up to 64 are ordered by one sort of wavefront 0, more by rank_pool.
// Returns false (for the whole workgroup) when they did not fit `pool` (kMergeCandCap) or the
// lists did not fit `qlist` (kMergeQlistCap).
__device__ __forceinline__ bool gather_fast(const MergeArgs& a, const Cand* part, const Cand* heads, MergeLds& L,
                                            Cand* pool, uint32_t* qlist) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = lane_id(), wave = wave_id(), nw = nt >> 6;
    const int kp = a.kprime, np = a.nparts, slots = a.list_len;
    // 1. the cut, from the list heads (the first two heads of a thread stay in registers)
    if (tid == 0) { L.sh[4] = 0; L.sh[5] = 0; }
    const Cand h0 = tid < np ? heads[tid] : (Cand)0;
    const Cand h1 = tid + nt < np ? heads[tid + nt] : (Cand)0;
    auto head_at = [&](uint32_t l) -> Cand { return l == (uint32_t)tid ? h0 : (l == (uint32_t)(tid + nt) ? h1 : heads[l]); };
    uint32_t best = max((uint32_t)(h0 >> 32), (uint32_t)(h1 >> 32));
#pragma unroll 1
    for (int l = tid + 2 * nt; l < np; l += nt) best = max(best, (uint32_t)(heads[l] >> 32));
    L.gmax[wave * 64 + lane] = best;
    __syncthreads();
    if (wave == 0) {
        uint32_t g = 0;
#pragma unroll 4
        for (int w = 0; w < nw; ++w) g = max(g, L.gmax[w * 64 + lane]);
        const Cand sorted = bitonic_sort64<true>((Cand)g << 32);          // largest first
        if (lane == kp - 1) L.sh[6] = (uint32_t)(sorted >> 32);            // 0: fewer than kprime groups hold anything, all pass
    }
    __syncthreads();
    const uint32_t cut = L.sh[6];
    // 2. the lists whose head passes ...
#pragma unroll 1
    for (int l = tid; l < np; l += nt) {
        const Cand h = head_at((uint32_t)l);
        if (h != 0 && (uint32_t)(h >> 32) >= cut) {
            const uint32_t pos = atomicAdd(&L.sh[5], 1u);
            if (pos < (uint32_t)kMergeQlistCap) qlist[pos] = (uint32_t)l;
        }
    }
    __syncthreads();
    const int nql = (int)L.sh[5];
    if (nql > kMergeQlistCap) return false;
    // ... and their entries that pass: four entries per thread and pass, all requested before
    // the first is looked at
    const int total = nql * slots;
#pragma unroll 1
    for (int e0 = 0; e0 < total; e0 += 4 * nt) {
        Cand c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + u * nt + tid;
            c[u] = e < total ? part[(size_t)qlist[e / slots] * slots + e % slots] : (Cand)0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool ok = c[u] != 0 && (uint32_t)(c[u] >> 32) >= cut;
            const uint64_t b = __ballot(ok);
            if (b) {
                uint32_t base = 0;
                if (lane == 0) base = atomicAdd(&L.sh[4], (uint32_t)__popcll(b));
                base = read_lane(base, 0);
                const uint32_t pos = base + __popcll(b & ((1ull << lane) - 1ull));
                if (ok && pos < (uint32_t)kMergeCandCap) pool[pos] = c[u];
            }
        }
    }
    __syncthreads();
    const uint32_t cnt = L.sh[4];
    if (cnt > (uint32_t)kMergeCandCap) return false;
    if (__builtin_expect(cnt > 64, 0)) { rank_pool(pool, cnt, kp, L); return true; }
    // 3. at most 64 candidates: one sort
    if (wave == 0) {
        const Cand sorted = bitonic_sort64<true>((uint32_t)lane < cnt ? pool[lane] : (Cand)0);
        if ((uint32_t)lane < cnt && lane < kp) L.c_cand[lane] = sorted;
        if (lane == 0) L.sh[4] = min(cnt, (uint32_t)kp);
    }
    __syncthreads();
    return true;
}

// General path: radix select over all entries of all lists (candidates are distinct, so the
// selection ends with exactly kprime of them).
__device__ __forceinline__ void gather_radix(const MergeArgs& a, const Cand* part, MergeLds& L) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = lane_id();
    const uint32_t n = (uint32_t)a.nparts * (uint32_t)a.list_len, kp = a.kprime;
    auto key_at = [&](uint32_t i) { return ~part[i]; };      // ascending = best first; all ones = empty
    uint32_t my_valid = 0;
    for (uint32_t i = tid; i < n; i += nt) my_valid += part[i] != 0;
    if (tid == 0) { L.sh[4] = 0; L.sh[5] = 0; }
    __syncthreads();
#pragma unroll
    for (int m2 = 32; m2 >= 1; m2 >>= 1) my_valid += __shfl_xor(my_valid, m2);
    if (lane == 0) atomicAdd(&L.sh[5], my_valid);
    __syncthreads();
    const uint32_t n_valid = L.sh[5];
    if (n_valid <= kp) {
        for (uint32_t i = tid; i < n; i += nt)
            if (part[i] != 0) L.c_cand[atomicAdd(&L.sh[4], 1u)] = part[i];
        __syncthreads();
        return;
    }
    uint64_t mask, prefix; uint32_t need, group;
    block_radix_select<uint64_t>(key_at, n, kp, L.hist, L.sh, mask, prefix, need, group);
    // need == group here: distinct keys leave a boundary group of one
    for (uint32_t i = tid; i < n; i += nt) {
        const uint64_t key = key_at(i);
        if (key != ~0ull && (key & mask) <= prefix) {
            uint32_t p = atomicAdd(&L.sh[4], 1u);
            if (p < (uint32_t)kMaxKPrime) L.c_cand[p] = part[i];
        }
    }
    __syncthreads();
}

// Can a row that the scan or the gathering dropped still belong to the k nearest?  Everything
// dropped anywhere has an fp32 key of at most f_last, the key of the last candidate kept, so its
// exact score is at most f_last + E, E bounding the rounding of the fp32 accumulation:
//   inner product   |fl(sum) - sum| <= g |q| |y|        squared distance   |fl(sum) - sum| <= g sum
// with g = err_coef (a little above (terms + 2) 2^-24 for sums whose terms pass through at most
// `terms` roundings).  The k-th best exact score found, s_k, is a lower bound of the true one;
// the result is exact when s_k > f_last + E.
__device__ __forceinline__ bool result_is_safe(double s_k, float f_last, const MergeArgs& a, double qq) {
    // single precision is enough for the bound itself: it is rounded upwards
    const float e = a.metric == 0 ? a.err_coef * (sqrtf((float)qq) * 1.0001f) * a.row_norm_max * 1.0001f
                                  : a.err_coef * fabsf(f_last) * 1.0001f;
    return s_k > (double)f_last + (double)e;
}

__global__ __launch_bounds__(kSelectThreads) void merge_kernel(MergeArgs a, int fast) {
    extern __shared__ __align__(16) unsigned char m_dyn[];
    __shared__ MergeLds L;
    __shared__ double q_part[kSelectThreads / 64];
    __shared__ double s_kth;
    __shared__ uint32_t f_min;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int qi = blockIdx.x;
    const uint32_t n = (uint32_t)a.nparts * (uint32_t)a.list_len;
    const Cand* part = a.part + (size_t)qi * n;
    const uint32_t kp = a.kprime;
    const float* q = a.q + (size_t)qi * a.d;

    // |q|^2 for the error bound, summed while the heads travel
    {
        double s = 0.0;
        for (int t = tid; t < a.d; t += nt) { const double x = (double)q[t]; s = fma(x, x, s); }
        s = wave_sum(s);
        if (lane_id() == 0) q_part[wave_id()] = s;
        if (tid == 0) { f_min = 0xFFFFFFFFu; s_kth = -INFINITY; }
    }

    // 1. the kprime best fp32 candidates
    bool gathered = false;
    if (fast) {
        Cand* pool = (Cand*)m_dyn;
        gathered = gather_fast(a, part, a.heads + (size_t)qi * a.nparts, L, pool, (uint32_t*)(pool + kMergeCandCap));
    }
    if (__builtin_expect(!gathered, 0)) {
        __syncthreads();
        gather_radix(a, part, L);
    }
    const uint32_t m = min(L.sh[4], (uint32_t)kMaxKPrime);

    // 2. fp64 re-score: a group of kRescoreLanes lanes per candidate, nt / kRescoreLanes
    //    candidates at once.  The order of operations is fixed (see rescore_row), so a row has
    //    the same fp64 score whichever kernel, or the host, computes it.
    const int np = a.nprobe;
    constexpr int lpc = kRescoreLanes;
    const int sub = tid % lpc;
#pragma unroll 1
    for (uint32_t c = (uint32_t)(tid / lpc); c < m; c += (uint32_t)(nt / lpc)) {
        const Cand cand = L.c_cand[c];
        const uint32_t row = cand_tie(cand);
        const int64_t id = a.ids ? a.ids[row] : (int64_t)row;
        size_t brow = row;
        bool found_row = true;
        if (!a.identity) {
            // the slot whose global row range holds the row
            const int64_t* s_base = a.slots.base + (size_t)qi * np;
            const uint32_t* s_grow = a.slots.grow + (size_t)qi * np;
            const uint32_t* s_n = a.slots.nrows + (size_t)qi * np;
            int found = -1;
#pragma unroll 1
            for (int s = sub; s < np; s += lpc)
                if (row >= s_grow[s] && row - s_grow[s] < s_n[s]) found = s;
#pragma unroll 1
            for (int o = 1; o < lpc; o <<= 1) found = max(found, __shfl_xor(found, o));
            found_row = found >= 0;
            brow = found_row ? (size_t)(s_base[found] + (int64_t)(row - s_grow[found])) : 0;
        }
        const double s = rescore_row(a.buf, q, a.d, a.dtype, a.metric, brow, sub);
        if (sub == 0) {
            L.f_key[c] = !found_row ? -INFINITY : (a.metric == 0 ? s : -s);
            L.f_id[c] = id;
            atomicMin(&f_min, (uint32_t)(cand >> 32));        // key image of the last candidate kept
        }
    }
    // 3. host candidates
    uint32_t nh = 0;
    if (a.host_cand) {
        nh = min((uint32_t)a.host_count[qi], kp);
        for (uint32_t i = tid; i < nh; i += nt) {
            L.f_key[m + i] = a.host_cand[(size_t)qi * kp + i].key;
            L.f_id[m + i] = a.host_cand[(size_t)qi * kp + i].id;
        }
    }
    __syncthreads();
    // 4. rank by counting; nearest first, ties by smaller id
    const uint32_t tot = m + nh;
    const int k = a.k;
    if ((uint32_t)tid < tot) {
        double mk = L.f_key[tid]; int64_t mi = L.f_id[tid];
        uint32_t rank = 0;
        // eight others per pass, all read before any is compared, and no branches: a compare that
        // waits for its own LDS read every time costs more than the whole pass
#pragma unroll 1
        for (uint32_t j0 = 0; j0 < tot; j0 += 8) {
            double ok[8]; int64_t oi[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t j = min(j0 + u, tot - 1);
                ok[u] = L.f_key[j]; oi[u] = L.f_id[j];
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
        if (rank == (uint32_t)k - 1) s_kth = mk;
    }
    for (uint32_t i = tot + tid; i < (uint32_t)k; i += nt) {
        a.out_ids[(size_t)qi * k + i] = -1;
        a.out_dists[(size_t)qi * k + i] = a.metric == 0 ? -INFINITY : INFINITY;
    }
    __syncthreads();
    // 5. is the result proven?  Rows were dropped only if kprime candidates were kept (a wavefront
    //    drops nothing before it holds kprime, the gathering nothing before it has kprime).
    if (tid == 0) {
        uint32_t unsafe = 0;
        if (m == kp) {
            double qq = 0.0;
            for (int w = 0; w < nt / 64; ++w) qq += q_part[w];
            unsafe = result_is_safe(s_kth, unordered(f_min), a, qq) ? 0u : 1u;
        }
        if (a.redo_flag) {
            a.redo_flag[qi] = unsafe;
            if (unsafe) {
                a.redo_thr[qi] = s_kth;
                a.redo_ticket[qi] = 0u;
            }
        }
        if (a.host_flag) a.host_flag[qi] = unsafe;       // pinned: stored before the completion word below
        if (a.done) {
            __threadfence_system();
            __hip_atomic_store(a.done, a.done_value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

// =============================================================================================
// Exact second pass for a query whose first result could not be proven (merge_kernel's step 5):
// every selected resident row is scored in fp64, in the order of operations of the re-score.
// Only rows that reach the k-th best score found so far can belong to the result; each wavefront
// keeps the k best of those it meets, ordered by (score, id), in a small list in LDS (rows within
// the rounding error of the scan are few unless the data holds masses of equal rows, and then
// the lists still bound what is kept).  The workgroup that finishes last ranks the entries of all
// lists, together with the host's candidates, and rewrites the query's results.  Launched after
// every merge of the device path; all workgroups of a query whose result was proven leave at once.
// =============================================================================================
constexpr int kRedoThreads = 256;
constexpr int kRedoWaves = kRedoThreads / 64;
static_assert(kRedoWaves == kRedoListsPerWg, "the list buffers are sized by kRedoListsPerWg");

__global__ __launch_bounds__(kRedoThreads) void exact_redo_kernel(RedoArgs a) {
    __shared__ uint32_t s_last;
    __shared__ unsigned long long w_key[kRedoWaves][IVF_MAX_K];     // ascending-order image of the score; 0 = empty
    __shared__ long long w_id[kRedoWaves][IVF_MAX_K];
    const int qi = blockIdx.y;
    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
    if (a.redo_flag[qi] == 0) {
        if (a.done && blockIdx.x == 0 && tid == 0) {
            __threadfence_system();
            __hip_atomic_store(a.done, a.done_value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        return;
    }
    const int np = a.nprobe, k = a.k;
    const float* q = a.q + (size_t)qi * a.d;
    const uint32_t* rp = a.slots.rprefix + (size_t)qi * (np + 1);
    const int64_t* s_base = a.slots.base + (size_t)qi * np;
    const uint32_t* s_grow = a.slots.grow + (size_t)qi * np;
    const uint32_t R = rp[np];
    const double thr = a.redo_thr[qi];
    unsigned long long* mk = w_key[wave];
    long long* mi = w_id[wave];
    for (int i = lane; i < k; i += 64) { mk[i] = 0ull; mi[i] = 0; }
    int count = 0;                                   // entries in this wavefront's list (uniform)
    constexpr int lpc = kRescoreLanes;
    constexpr int gpw = 64 / lpc;                    // rows a wavefront scores at a time
    const int sub = lane % lpc;
    const uint32_t group = (uint32_t)((blockIdx.x * kRedoWaves + wave) * gpw + lane / lpc);
    const uint32_t ngroups = gridDim.x * kRedoWaves * gpw;
    const uint32_t rounds = (R + ngroups - 1) / ngroups;
#pragma unroll 1
    for (uint32_t it = 0; it < rounds; ++it) {
        const uint32_t r = it * ngroups + group;
        double key = -INFINITY;
        long long id = 0;
        if (r < R) {
            uint32_t lo = 0, hi = (uint32_t)np;            // rp[lo] <= r < rp[hi]
            while (hi - lo > 1) {
                const uint32_t mid = (lo + hi) >> 1;
                if (rp[mid] <= r) lo = mid; else hi = mid;
            }
            const uint32_t in_slot = r - rp[lo];
            const size_t brow = (size_t)(s_base[lo] + (int64_t)in_slot);
            const double s = rescore_row(a.buf, q, a.d, a.dtype, a.metric, brow, sub);
            key = a.metric == 0 ? s : -s;
            const uint32_t grow = s_grow[lo] + in_slot;
            id = a.ids ? (long long)a.ids[grow] : (long long)grow;
        }
        // the rows of this round that reach the threshold go into the list one after the other
        uint64_t want = __ballot(sub == 0 && r < R && key >= thr);
        while (want) {
            const int src = __ffsll((long long)want) - 1;
            want &= want - 1;
            const unsigned long long nk = ordered(__shfl(key, src));
            const long long nid = __shfl(id, src);
            // position: entries ahead of the new one (larger key, or equal key and smaller id)
            int ahead = 0;
            for (int i = lane; i < count; i += 64) ahead += (mk[i] > nk || (mk[i] == nk && mi[i] < nid)) ? 1 : 0;
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) ahead += __shfl_xor(ahead, m);
            if (ahead >= k) continue;                      // the list is full of better rows
            const int last = min(count, k - 1);            // entries ahead .. last-1 move down by one
            for (int base = ((last - 1) / 64) * 64; base >= 0 && last > ahead; base -= 64) {
                const int i = base + lane;
                const bool mv = i >= ahead && i < last;
                const unsigned long long tk = mv ? mk[i] : 0ull;
                const long long ti = mv ? mi[i] : 0;
                if (mv) { mk[i + 1] = tk; mi[i + 1] = ti; }    // a wavefront's LDS operations complete in order
            }
            if (lane == 0) { mk[ahead] = nk; mi[ahead] = nid; }
            count = min(count + 1, k);
        }
    }
    // every wavefront leaves its k slots (0 = empty) in the query's list
    {
        const size_t o = ((size_t)qi * gridDim.x * kRedoWaves + (size_t)blockIdx.x * kRedoWaves + wave) * (size_t)k;
        for (int i = lane; i < k; i += 64) {
            __hip_atomic_store(&a.list_key[o + i], i < count ? mk[i] : 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&a.list_id[o + i], mi[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
    if (tid == 0) {
        __threadfence();
        s_last = atomicAdd(&a.redo_ticket[qi], 1u) == gridDim.x - 1 ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    // the last workgroup: rank the entries of all lists and the host's candidates by (score, id)
    const uint32_t n = gridDim.x * kRedoWaves * (uint32_t)k;
    const unsigned long long* l_key = a.list_key + (size_t)qi * n;
    const long long* l_id = a.list_id + (size_t)qi * n;
    const uint32_t nh = a.host_cand ? min((uint32_t)a.host_count[qi], (uint32_t)a.kprime) : 0u;
    const uint32_t tot = n + nh;
    auto key_of = [&](uint32_t j) -> unsigned long long {
        if (j < n) return __hip_atomic_load(&l_key[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return (unsigned long long)ordered(a.host_cand[(size_t)qi * a.kprime + (j - n)].key);
    };
    auto id_of = [&](uint32_t j) -> long long {
        if (j < n) return __hip_atomic_load(&l_id[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return (long long)a.host_cand[(size_t)qi * a.kprime + (j - n)].id;
    };
#pragma unroll 1
    for (uint32_t e = tid; e < tot; e += kRedoThreads) {
        const unsigned long long ek = key_of(e);
        if (ek == 0ull) continue;
        const long long ei = id_of(e);
        uint32_t rank = 0;
#pragma unroll 1
        for (uint32_t j = 0; j < tot && rank < (uint32_t)k; ++j) {
            const unsigned long long ok = key_of(j);
            rank += (uint32_t)(ok > ek || (ok == ek && ok != 0ull && id_of(j) < ei));
        }
        if (rank < (uint32_t)k) {
            const double key = unordered((uint64_t)ek);
            a.out_ids[(size_t)qi * k + rank] = (int64_t)ei;
            a.out_dists[(size_t)qi * k + rank] = (float)(a.metric == 0 ? key : -key);
        }
    }
    if (a.done) {
        __syncthreads();
        if (tid == 0) {
            __threadfence_system();
            __hip_atomic_store(a.done, a.done_value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

hipError_t launch_redo(const RedoArgs& a, int grid, hipStream_t s) {
    if (a.done && a.nq != 1) return hipErrorInvalidValue;
    if (a.k > IVF_MAX_K) return hipErrorInvalidValue;
    hipLaunchKernelGGL(exact_redo_kernel, dim3(grid, a.nq), dim3(kRedoThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_merge(const MergeArgs& a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
    if (a.done && a.nq != 1) return hipErrorInvalidValue;
    const size_t n = (size_t)a.nparts * a.list_len;
    const int fast = a.kprime <= 64;
    const int threads = fast ? kMergeFastThreads : (n <= 8192 ? 256 : kSelectThreads);
    const size_t lds = fast ? (size_t)kMergeCandCap * 8 + (size_t)kMergeQlistCap * 4 : 0;
    IVF_LAUNCH(merge_kernel, dim3(a.nq), dim3(threads), lds, s, e0, e1, a, fast);
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

// =============================================================================================
// Consolidation of the prefetch buffer (Sec. 4.2 "Cache design"; appendix: the GPU memory is
// consolidated after each batch).  One launch carries out a group of moves that do not disturb
// each other (no destination of the group overlaps a source of the group): the moves are cut
// into chunks of kMoveChunk bytes and every workgroup copies chunks, 16 bytes per lane where the
// addresses allow.  HBM-bound: every byte moved is read once and written once.
// =============================================================================================
constexpr uint32_t kMoveChunk = 64u << 10;

__global__ __launch_bounds__(256) void gather_moves_kernel(unsigned char* buf, const MoveDesc* moves, int n_moves,
                                                           uint32_t n_chunks) {
    for (uint32_t ch = blockIdx.x; ch < n_chunks; ch += gridDim.x) {
        int lo = 0, hi = n_moves;                  // moves[lo].chunk0 <= ch < moves[hi].chunk0 (a sentinel past the end)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (moves[mid].chunk0 <= ch) lo = mid; else hi = mid;
        }
        const MoveDesc m = moves[lo];
        const uint64_t o = (uint64_t)(ch - m.chunk0) * kMoveChunk;
        const uint64_t len = min((uint64_t)kMoveChunk, m.bytes - o);
        const unsigned char* src = buf + m.from_byte + o;
        unsigned char* dst = buf + m.to_byte + o;
        if ((((uintptr_t)src | (uintptr_t)dst) & 15u) == 0) {
            const uint32_t vec = (uint32_t)(len / 16);
            // eight loads per lane in flight before the first store
#pragma unroll 1
            for (uint32_t i0 = 0; i0 < vec; i0 += 8 * 256) {
                uint4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const uint32_t i = i0 + u * 256 + threadIdx.x;
                    v[u] = load_stream16(src + (size_t)min(i, vec - 1) * 16);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const uint32_t i = i0 + u * 256 + threadIdx.x;
                    if (i < vec) store_stream16(dst + (size_t)i * 16, v[u]);
                }
            }
            for (uint64_t i = (uint64_t)vec * 16 + threadIdx.x; i < len; i += blockDim.x) dst[i] = src[i];
        } else {
            for (uint64_t i = threadIdx.x; i < len; i += blockDim.x) dst[i] = src[i];
        }
    }
}

uint32_t move_chunks(uint64_t bytes) { return (uint32_t)((bytes + kMoveChunk - 1) / kMoveChunk); }

hipError_t launch_gather_moves(void* buf, const MoveDesc* moves_dev, int n_moves, uint32_t n_chunks, int n_cu, hipStream_t s) {
    if (n_moves <= 0 || n_chunks == 0) return hipSuccess;
    const uint32_t grid = std::min<uint32_t>(n_chunks, (uint32_t)n_cu * 8u);
    hipLaunchKernelGGL(gather_moves_kernel, dim3(grid), dim3(256), 0, s, (unsigned char*)buf, moves_dev, n_moves, n_chunks);
    return hipGetLastError();
}

// =============================================================================================
// Queries handed over in host memory: a few KB that a kernel reads from the pinned buffer itself
// (one dispatch on the search stream) instead of a copy engine transfer set up by the runtime.
// =============================================================================================
__global__ void stage_query_kernel(const float* src, float* dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

hipError_t launch_stage_query(const float* src_pinned, float* dst, size_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    const size_t blocks = std::min<size_t>((n + 255) / 256, 64);
    hipLaunchKernelGGL(stage_query_kernel, dim3((unsigned)blocks), dim3(256), 0, s, src_pinned, dst, n);
    return hipGetLastError();
}

// =============================================================================================
// Cluster cache bookkeeping (Sec. 4.2 "Cache design"; appendix: hotness h <- h / d, + h_inc when
// the cluster was used in the round).  hot[c] < 0 marks a cluster that is not cached.
// Single precision, one correctly rounded division and one addition per cluster.
// =============================================================================================
// reset: the cache starts over (hotness and use marks are dropped) before the admission
__global__ void cache_admit_kernel(float* hot, uint32_t* used, const int64_t* res_off, int nlist, float h_init, int reset) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= nlist) return;
    if (reset) used[c] = 0u;
    float h = reset ? -1.f : hot[c];
    if (res_off[c] < 0) h = -1.f;
    else if (h < 0.f) h = h_init;            // fetched since the last call: cached from now on
    hot[c] = h;
}

__global__ void cache_round_kernel(float* hot, uint32_t* used, int nlist, float decay, float h_inc) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= nlist) return;
    float h = hot[c];
    if (h >= 0.f) {
        h = h / decay;
        if (used[c]) h = h + h_inc;
        hot[c] = h;
    }
    used[c] = 0u;
}

hipError_t launch_cache_admit(float* hot, uint32_t* used, const int64_t* res_off, int nlist, float h_init, int reset,
                              hipStream_t s) {
    hipLaunchKernelGGL(cache_admit_kernel, dim3((nlist + 255) / 256), dim3(256), 0, s, hot, used, res_off, nlist, h_init, reset);
    return hipGetLastError();
}
hipError_t launch_cache_round(float* hot, uint32_t* used, int nlist, float decay, float h_inc, hipStream_t s) {
    hipLaunchKernelGGL(cache_round_kernel, dim3((nlist + 255) / 256), dim3(256), 0, s, hot, used, nlist, decay, h_inc);
    return hipGetLastError();
}

}  // namespace ivf
