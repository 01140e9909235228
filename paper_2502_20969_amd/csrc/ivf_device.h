// Device-side building blocks for the IVF kernels (gfx950, wave64).
#pragma once
#include "ivf_internal.h"
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

// Launch with optional events that receive the kernel's own begin and end time; the plain launch
// is used when no events are asked for.
#define IVF_LAUNCH(kernel, grid, block, lds, stream, ev0, ev1, ...)                                \
    do {                                                                                            \
        if ((ev0) || (ev1)) hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, ev0, ev1, 0, __VA_ARGS__); \
        else hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                    \
    } while (0)

namespace ivf {
namespace dev {

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() {
    return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // uniform: kept in an SGPR
}

// ---- cross-lane sums ----------------------------------------------------------------------
// DPP controls (GFX9): quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E,
// row_half_mirror = 0x141, row_mirror = 0x140.  Applied in this order to a value each lane
// holds, every lane of a 16-lane row ends with the row's sum.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Sum over each aligned group of LANES lanes (16, 32 or 64); every lane of the group gets it.
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);
    if (LANES >= 32) v += __shfl_xor(v, 16);
    if (LANES >= 64) v += __shfl_xor(v, 32);
    return v;
}

// Same sum, but only the LAST lane of each group is guaranteed to hold it (cheaper: the two
// widest steps are DPP row broadcasts, row_bcast:15 = 0x142 into rows 1 and 3 and
// row_bcast:31 = 0x143 into rows 2 and 3, instead of LDS permutes).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move_rows(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
template <int LANES>
__device__ __forceinline__ float group_total_last_lane(float v) {
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);
    if (LANES >= 32) v += dpp_move_rows<0x142, 0xA>(v);
    if (LANES >= 64) v += dpp_move_rows<0x143, 0xC>(v);
    return v;
}

// 16-byte streaming load: the rows of a list are read once, so they should not displace
// the query, the tables or the centroids from the caches.
typedef unsigned int u4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
    u4_t t = __builtin_nontemporal_load((const u4_t*)p);
    return make_uint4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ void store_stream16(void* p, const uint4& v) {
    u4_t t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, (u4_t*)p);
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
    return v;
}

__device__ __forceinline__ float read_lane(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ uint32_t read_lane(uint32_t v, int lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}

// ---- stored element types -------------------------------------------------------------------
struct F32 { static constexpr int kBytes = 4; static constexpr int kPerLoad = 4; };
struct F16 { static constexpr int kBytes = 2; static constexpr int kPerLoad = 8; };
struct BF16 { static constexpr int kBytes = 2; static constexpr int kPerLoad = 8; };

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// Expands one 16-byte load into its float values.
template <typename T> struct Unpack;
template <> struct Unpack<F32> {
    __device__ static __forceinline__ void run(const uint4& v, float* out) {
        out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y);
        out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
    }
};
template <> struct Unpack<F16> {
    __device__ static __forceinline__ void run(const uint4& v, float* out) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            half2_t h = __builtin_bit_cast(half2_t, w[i]);
            out[2 * i] = (float)h.x;
            out[2 * i + 1] = (float)h.y;
        }
    }
};
template <> struct Unpack<BF16> {
    __device__ static __forceinline__ void run(const uint4& v, float* out) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};

// One stored element widened exactly to double (used by the fp64 re-score).
__device__ __forceinline__ double widen(const void* base, int dtype, size_t idx) {
    if (dtype == 0) return (double)((const float*)base)[idx];
    uint16_t b = ((const uint16_t*)base)[idx];
    if (dtype == 1) return (double)(float)__builtin_bit_cast(_Float16, b);
    return (double)__uint_as_float((uint32_t)b << 16);
}

// The fp64 re-score has one fixed order of operations, shared by the merge kernels and by the
// host's scan of the clusters that are not resident, so that identical rows get bit-identical
// scores wherever they are scored and equal scores are then ordered by id alone: kRescoreLanes
// accumulators; accumulator s takes the 16-byte chunks s, s + 32, ... of the row in that order
// (elements in memory order, one fused multiply-add each); the accumulators are added by a
// butterfly over the lane distances 1, 2, 4, 8, 16.  Rows that are not whole 16-byte chunks use
// the same scheme over single elements.
constexpr int kRescoreLanes = 32;

// Partial fp64 score of one stored row over the 16-byte chunks sub, sub + lpc, ... (lane `sub`
// of a group of `lpc` lanes); several loads are in flight at a time.
template <typename T>
__device__ __forceinline__ double rescore_partial(const unsigned char* row, const float* q, int d, int metric,
                                                  int sub, int lpc) {
    constexpr int EPL = T::kPerLoad;
    constexpr int U = EPL == 4 ? 6 : 4;        // 768 fp32 values over 32 lanes: one pass
    const int chunks = d / EPL;
    double acc = 0.0;
#pragma unroll 1
    for (int c0 = sub; c0 < chunks; c0 += lpc * U) {
        uint4 v[U];
        float qv[U][EPL];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = min(c0 + u * lpc, chunks - 1);
            v[u] = *(const uint4*)(row + (size_t)c * 16);
#pragma unroll
            for (int e = 0; e < EPL; e += 4) *(float4*)&qv[u][e] = *(const float4*)(q + (size_t)c * EPL + e);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (c0 + u * lpc < chunks) {
                float x[EPL];
                Unpack<T>::run(v[u], x);
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    const double qd = (double)qv[u][e], y = (double)x[e];
                    if (metric == 0) acc = fma(qd, y, acc);
                    else { const double df = qd - y; acc = fma(df, df, acc); }
                }
            }
        }
    }
    return acc;
}

// fp64 score of the stored row `brow` of the buffer for the query q, computed by a group of
// kRescoreLanes lanes (sub = lane in the group); every lane of the group gets the sum.  One fixed
// order of operations (rescore_partial, then a butterfly over the lane distances 1 .. 16).
__device__ __forceinline__ double rescore_row(const void* buf, const float* q, int d, int dtype, int metric,
                                              size_t brow, int sub) {
    constexpr int lpc = kRescoreLanes;
    const size_t row_bytes = (size_t)d * (dtype == 0 ? 4 : 2);
    const unsigned char* rp = (const unsigned char*)buf + brow * row_bytes;
    double s = 0.0;
    if (row_bytes % 16 == 0) {
        if (dtype == 0) s = rescore_partial<F32>(rp, q, d, metric, sub, lpc);
        else if (dtype == 1) s = rescore_partial<F16>(rp, q, d, metric, sub, lpc);
        else s = rescore_partial<BF16>(rp, q, d, metric, sub, lpc);
    } else {
        const size_t e0 = brow * (size_t)d;
#pragma unroll 1
        for (int t = sub; t < d; t += lpc) {
            const double x = (double)q[t], y = widen(buf, dtype, e0 + t);
            if (metric == 0) s = fma(x, y, s);
            else { const double df = x - y; s = fma(df, df, s); }
        }
    }
#pragma unroll 1
    for (int o = 1; o < lpc; o <<= 1) s += __shfl_xor(s, o);
    return s;
}

// ---- order-preserving integer keys ------------------------------------------------------------
// Unsigned keys whose ascending order is the ascending order of the floating value.
__device__ __forceinline__ uint32_t ordered(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ uint64_t ordered(double f) {
    uint64_t u = (uint64_t)__double_as_longlong(f);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ double unordered(uint64_t o) {       // inverse of ordered(double)
    uint64_t u = (o >> 63) ? (o & 0x7FFFFFFFFFFFFFFFull) : ~o;
    return __longlong_as_double((long long)u);
}

// ---- block-wide radix select -----------------------------------------------------------------
// Adds 1 to hist[digit] for every active lane; lanes of a wavefront that share a digit are
// combined into one LDS atomic for the first two distinct digits (keys that agree in their
// high bits would otherwise all hit the same counter one after the other).
__device__ __forceinline__ void hist_add(uint32_t* hist, uint32_t digit, bool active) {
#pragma unroll 1
    for (int round = 0; round < 2; ++round) {
        uint64_t act = __ballot(active);
        if (!act) return;
        int first = __ffsll((long long)act) - 1;
        uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)digit, first);
        uint64_t same = __ballot(active && digit == d0);
        if (lane_id() == first) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
        active = active && digit != d0;
    }
    if (active) atomicAdd(&hist[digit], 1u);
}

// Finds, among the valid keys key_at(i), i < n (smaller = better; the all-ones key marks an
// invalid entry and is ignored), the split that keeps the `want` smallest; want must not exceed
// the number of valid keys.  On return every thread holds: `mask` (the high bits decided),
// `prefix` (their value for the boundary group), `need` (how many keys of the boundary group,
// (key & mask) == prefix, are kept) and `group` (size of that group).  Keys with
// (key & mask) < prefix are all kept.  need == group unless the boundary group is a set of
// fully equal keys.  Digits above the highest bit in which the keys differ are skipped.
// hist: 256 words of LDS; sh: 8 words of LDS.  Must be called by all threads of the block.
template <typename KeyT, typename KeyAt>
__device__ void block_radix_select(KeyAt key_at, uint32_t n, uint32_t want, uint32_t* hist,
                                   uint32_t* sh, KeyT& mask, KeyT& prefix, uint32_t& need,
                                   uint32_t& group) {
    const int tid = threadIdx.x, nt = blockDim.x;
    constexpr KeyT kInvalid = ~(KeyT)0;
    // bits in which the valid keys differ, and how many valid keys there are
    KeyT all_or = 0, all_and = kInvalid;
    uint32_t cnt = 0;
    for (uint32_t i = tid; i < n; i += nt) {
        KeyT k = key_at(i);
        if (k != kInvalid) { all_or |= k; all_and &= k; ++cnt; }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        all_or |= __shfl_xor(all_or, m);
        all_and &= __shfl_xor(all_and, m);
        cnt += __shfl_xor(cnt, m);
    }
    KeyT* sk = (KeyT*)hist;                 // scratch use of hist before the first pass
    const int nw = nt >> 6;
    if ((tid & 63) == 0) { sk[2 * (tid >> 6)] = all_or; sk[2 * (tid >> 6) + 1] = all_and; }
    if ((tid & 63) == 0) sh[7] = 0;
    __syncthreads();
    if ((tid & 63) == 0) atomicAdd(&sh[7], cnt);
    all_or = 0; all_and = kInvalid;
    for (int w = 0; w < nw; ++w) { all_or |= sk[2 * w]; all_and &= sk[2 * w + 1]; }
    __syncthreads();
    const uint32_t n_valid = sh[7];
    const KeyT diff = all_or ^ all_and;
    mask = 0; prefix = 0; need = want; group = n_valid;
    int top_shift = (int)sizeof(KeyT) * 8 - 8;
    if (n_valid > 0) {
        // highest differing bit decides the first digit; everything above it is common
        int hb = diff == 0 ? -1 : (int)(sizeof(KeyT) * 8 - 1 - (sizeof(KeyT) == 8 ? __clzll((long long)diff) : __clz((int)diff)));
        int first_shift = hb < 0 ? -8 : (hb / 8) * 8;
        for (int sft = top_shift; sft > first_shift; sft -= 8) {
            mask |= (KeyT)255 << sft;
        }
        prefix = all_and & mask;
        top_shift = first_shift;
    }
    __syncthreads();
    for (int shift = top_shift; shift >= 0; shift -= 8) {
        if (need == group) break;
        for (int i = tid; i < 256; i += nt) hist[i] = 0;
        __syncthreads();
        for (uint32_t i0 = 0; i0 < n; i0 += nt) {
            uint32_t i = i0 + tid;
            KeyT k = i < n ? key_at(i) : kInvalid;
            bool act = k != kInvalid && (k & mask) == prefix;
            hist_add(hist, (uint32_t)(k >> shift) & 255u, act);
        }
        __syncthreads();
        if (tid < 64) {
            uint32_t c[4], s4 = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) { c[b] = hist[4 * tid + b]; s4 += c[b]; }
            uint32_t incl = s4;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                uint32_t up = __shfl_up(incl, o);
                if (tid >= o) incl += up;
            }
            uint32_t excl = incl - s4;
            if (excl < need && need <= incl) {
                uint32_t run = excl;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    if (run < need && need <= run + c[b]) {
                        sh[0] = 4 * tid + b; sh[1] = need - run; sh[2] = c[b];
                    }
                    run += c[b];
                }
            }
        }
        __syncthreads();
        prefix |= (KeyT)sh[0] << shift;
        mask |= (KeyT)255 << shift;
        need = sh[1];
        group = sh[2];
        __syncthreads();
    }
}

// ---- block-wide bucket cut ----------------------------------------------------------------------
// A coarse cut for "the `want` largest of n 32-bit values" in one pass over a 256-bucket
// histogram (three barriers; the sorting networks cost several times that in a kernel of one
// workgroup).  The bucket of a value is a monotone function of it over the range [lo, hi] of the
// values present; `cut` is the highest bucket such that at least `want` values fall into buckets
// >= cut.  Values below the range are not counted (they would all land on one counter); when
// fewer than `want` values lie in the range, everything passes.  Every one of the `want` largest
// values passes, and so does anything, also from outside the set, that is not smaller than one
// of them.
struct BucketCut {
    uint32_t lo;             // lower end of the range (0 when everything passes)
    float scale;
    uint32_t cut;
    uint32_t passing;        // values of the set that pass; all ones when everything passes (not counted then)
    __device__ __forceinline__ uint32_t bucket(uint32_t v) const {      // v >= lo
        const uint32_t b = (uint32_t)((float)(v - lo) * scale);
        return b > 255u ? 255u : b;
    }
    __device__ __forceinline__ bool pass(uint32_t v) const { return v >= lo && bucket(v) >= cut; }
};

// val_at(i), i < n: the values (0 = no value, ignored).  hist: 256 words of LDS; red: 96 words of
// LDS.  Must be called by all threads of the block (64 to 1024, a multiple of 64).
//
// The lower end of the range decides how fine the buckets are where it matters.  The threads
// are taken in 64 groups and every group folds its values into a maximum: when at least `want`
// groups hold a value, the smallest of those maxima has `want` values at or above it and is
// used as the lower end (values below it all fall into bucket 0); otherwise the smallest value
// is.  If the cut still lets more than about twice `want` values pass, the range is narrowed to
// the buckets from the cut upwards and the histogram is taken again (at most twice).
template <typename ValAt>
__device__ __forceinline__ BucketCut block_bucket_cut(ValAt val_at, uint32_t n, uint32_t want, uint32_t* hist, uint32_t* red) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = lane_id(), wave = wave_id();
    const int per_group = nt >> 6;                      // lanes per group: a power of two up to 16, inside one wavefront
    uint32_t lo = 0xFFFFFFFFu, hi = 0u;
    for (uint32_t i = tid; i < n; i += nt) {
        const uint32_t v = val_at(i);
        if (v) { lo = min(lo, v); hi = max(hi, v); }
    }
    uint32_t gmax = hi;
    for (int m = 1; m < per_group; m <<= 1) gmax = max(gmax, (uint32_t)__shfl_xor((int)gmax, m));
    if ((lane & (per_group - 1)) == 0) red[8 + tid / per_group] = gmax;        // red[8 .. 71]: the group maxima
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) lo = min(lo, (uint32_t)__shfl_xor((int)lo, m));
    if (lane == 0) red[72 + wave] = lo;                 // red[72 .. 87]: the wavefronts' smallest values
    for (int i = tid; i < 256; i += nt) hist[i] = 0;
    __syncthreads();
    {
        // all threads fold the 64 group maxima (lane l of every wavefront reads group l)
        const uint32_t g = red[8 + lane];
        uint32_t g_lo = g ? g : 0xFFFFFFFFu, g_hi = g;
        const uint32_t groups = (uint32_t)__popcll(__ballot(g != 0));
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            g_lo = min(g_lo, (uint32_t)__shfl_xor((int)g_lo, m));
            g_hi = max(g_hi, (uint32_t)__shfl_xor((int)g_hi, m));
        }
        uint32_t w_lo = lane < (nt >> 6) ? red[72 + lane] : 0xFFFFFFFFu;
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) w_lo = min(w_lo, (uint32_t)__shfl_xor((int)w_lo, m));
        w_lo = (uint32_t)__shfl((int)w_lo, 0);
        hi = g_hi;
        lo = groups >= want ? g_lo : w_lo;
    }
    BucketCut bc;
    bc.lo = lo;
    bc.scale = hi > lo ? 255.5f / (float)(hi - lo) : 0.f;
    bc.cut = 0; bc.passing = 0;
#pragma unroll 1
    for (int round = 0; round < 3; ++round) {
        for (uint32_t i = tid; i < n; i += nt) {
            const uint32_t v = val_at(i);
            if (v != 0 && v >= bc.lo) atomicAdd(&hist[bc.bucket(v)], 1u);
        }
        __syncthreads();
        if (wave == 0) {
            uint32_t c[4], s4 = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) { c[b] = hist[4 * lane + b]; s4 += c[b]; }
            uint32_t from_top = s4;                    // values in the buckets of this lane and of all higher lanes
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t dn = __shfl_down(from_top, o);
                if (lane + o < 64) from_top += dn;
            }
            const uint32_t above = from_top - s4;
            if (lane == 0 && from_top < want) { red[2] = 0xFFFFFFFFu; red[3] = 0xFFFFFFFFu; }
            if (above < want && want <= from_top) {
                uint32_t run = above;
#pragma unroll
                for (int b = 3; b >= 0; --b) {
                    if (run < want && want <= run + c[b]) { red[2] = (uint32_t)(4 * lane + b); red[3] = run + c[b]; }
                    run += c[b];
                }
            }
        }
        __syncthreads();
        bc.cut = red[2];
        bc.passing = red[3];
        if (bc.cut == 0xFFFFFFFFu) { bc.lo = 0u; bc.scale = 0.f; bc.cut = 0u; break; }      // fewer than `want` in the range: all pass
        if (round == 2 || bc.cut < 2 || bc.passing <= 2 * want + 16 || bc.scale == 0.f) break;
        // narrow the range to the buckets from one below the cut upwards (the edge is rounded down, so
        // nothing that passed is lost; what now falls below the range lands in bucket 0)
        const uint32_t edge = bc.lo + (uint32_t)((float)(bc.cut - 1) / bc.scale);
        bc.lo = min(max(edge, bc.lo), hi);
        bc.scale = hi > bc.lo ? 255.5f / (float)(hi - bc.lo) : 0.f;
        bc.cut = 0;
        for (int i = tid; i < 256; i += nt) hist[i] = 0;
        __syncthreads();                                // the histogram is clear, and red[2], red[3] were read, before the next round
    }
    return bc;
}

// ---- block-wide bitonic sort of (key, idx) pairs, ascending by key then idx --------------------
// n must be a power of two.  keys/idx may point to LDS or to global memory.
__device__ inline void block_bitonic_sort(uint64_t* keys, uint32_t* idx, uint32_t n) {
    const uint32_t tid = threadIdx.x, nt = blockDim.x;
    for (uint32_t size = 2; size <= n; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (uint32_t i = tid; i < n; i += nt) {
                uint32_t j = i ^ stride;
                if (j > i) {
                    uint64_t ki = keys[i], kj = keys[j];
                    uint32_t ii = idx[i], ij = idx[j];
                    bool i_after_j = ki > kj || (ki == kj && ii > ij);
                    bool ascending = (i & size) == 0;
                    if (i_after_j == ascending) {
                        keys[i] = kj; keys[j] = ki;
                        idx[i] = ij; idx[j] = ii;
                    }
                }
            }
            __syncthreads();
        }
    }
}

// ---- packed candidates --------------------------------------------------------------------------
// A candidate is one 64-bit word whose unsigned order is the result order: the order-preserving
// image of an fp32 key in the high half and the complement of a tie-break rank in the low half
// (rows: the rank of the row's id among all ids, so that equal keys come out by smaller id;
// clusters: see the select kernel).  Larger = comes first; 0 = empty (no finite or infinite key
// has a zero image).  One compare decides an exchange, which keeps the networks below short:
// a single-workgroup kernel runs each instruction once, so its time follows its code size.
typedef uint64_t Cand;
__device__ __forceinline__ float unordered(uint32_t o) {          // inverse of ordered(float)
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}
__device__ __forceinline__ Cand pack_cand(float key, uint32_t tie) {
    return ((uint64_t)ordered(key) << 32) | (uint64_t)(uint32_t)~tie;
}
__device__ __forceinline__ float cand_key(Cand c) { return unordered((uint32_t)(c >> 32)); }
__device__ __forceinline__ uint32_t cand_tie(Cand c) { return ~(uint32_t)c; }
__device__ __forceinline__ Cand read_lane(Cand v, int lane) {
    return ((uint64_t)read_lane((uint32_t)(v >> 32), lane) << 32) | read_lane((uint32_t)v, lane);
}

// ---- sorting networks over the 64 lanes of a wavefront --------------------------------------------
// Value held by lane (lane ^ STRIDE), with register-to-register moves only: DPP quad
// permutes (1, 2), row shifts (4), a row rotate (8), and the 16- and 32-lane swaps of gfx950.
template <int STRIDE>
__device__ __forceinline__ uint32_t xor_lane_u32(uint32_t v) {
    const int lane = lane_id();
    if (STRIDE == 1) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);
    if (STRIDE == 2) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);
    if (STRIDE == 4) {
        int up = __builtin_amdgcn_update_dpp(0, (int)v, 0x104, 0xF, 0xF, true);   // row_shl:4 = lane + 4
        int dn = __builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true);   // row_shr:4 = lane - 4
        return (uint32_t)((lane & 4) ? dn : up);
    }
    if (STRIDE == 8) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x128, 0xF, 0xF, true);  // row_ror:8
    if (STRIDE == 16) {
        auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);   // [0] = rows 0,0,2,2  [1] = rows 1,1,3,3
        return (lane & 16) ? r[0] : r[1];
    }
    auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);       // [0] = low half twice, [1] = high half twice
    return (lane & 32) ? r[0] : r[1];
}
// Value held by lane 63 - lane.
__device__ __forceinline__ uint32_t mirror_lane_u32(uint32_t v) {
    uint32_t m = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true);   // row_mirror = lane ^ 15
    return xor_lane_u32<32>(xor_lane_u32<16>(m));
}
template <int STRIDE>
__device__ __forceinline__ Cand xor_lane(Cand c) {
    return ((uint64_t)xor_lane_u32<STRIDE>((uint32_t)(c >> 32)) << 32) | xor_lane_u32<STRIDE>((uint32_t)c);
}
__device__ __forceinline__ Cand mirror(Cand c) {
    return ((uint64_t)mirror_lane_u32((uint32_t)(c >> 32)) << 32) | mirror_lane_u32((uint32_t)c);
}

// The largest candidate word held by any lane (0 when all are empty); every lane gets it.
__device__ __forceinline__ Cand wave_max(Cand c) {
    Cand o;
    o = xor_lane<1>(c); c = o > c ? o : c;
    o = xor_lane<2>(c); c = o > c ? o : c;
    o = xor_lane<4>(c); c = o > c ? o : c;
    o = xor_lane<8>(c); c = o > c ? o : c;
    o = xor_lane<16>(c); c = o > c ? o : c;
    o = xor_lane<32>(c); c = o > c ? o : c;
    return c;
}

// One compare-exchange step between lane and lane ^ STRIDE.  keep_first: this lane keeps the
// candidate that comes first (the larger word), else the other one.
template <int STRIDE>
__device__ __forceinline__ void cmp_exchange(Cand& c, bool keep_first) {
    Cand p = xor_lane<STRIDE>(c);
    if ((p > c) == keep_first) c = p;
}

// Sorts a bitonic sequence of 64 lane-held candidates into first-to-last order.
__device__ __forceinline__ Cand bitonic_merge64_inline(Cand c) {
    const int lane = lane_id();
    cmp_exchange<32>(c, (lane & 32) == 0);
    cmp_exchange<16>(c, (lane & 16) == 0);
    cmp_exchange<8>(c, (lane & 8) == 0);
    cmp_exchange<4>(c, (lane & 4) == 0);
    cmp_exchange<2>(c, (lane & 2) == 0);
    cmp_exchange<1>(c, (lane & 1) == 0);
    return c;
}
// Sorts 64 lane-held candidates first-to-last (bitonic sorting network over the lanes).
__device__ __forceinline__ Cand bitonic_sort64_inline(Cand c) {
    const int lane = lane_id();
#define IVF_STAGE(SIZE, STRIDE) cmp_exchange<STRIDE>(c, ((lane & STRIDE) == 0) == ((lane & SIZE) == 0));
    IVF_STAGE(2, 1)
    IVF_STAGE(4, 2) IVF_STAGE(4, 1)
    IVF_STAGE(8, 4) IVF_STAGE(8, 2) IVF_STAGE(8, 1)
    IVF_STAGE(16, 8) IVF_STAGE(16, 4) IVF_STAGE(16, 2) IVF_STAGE(16, 1)
    IVF_STAGE(32, 16) IVF_STAGE(32, 8) IVF_STAGE(32, 4) IVF_STAGE(32, 2) IVF_STAGE(32, 1)
    IVF_STAGE(64, 32) IVF_STAGE(64, 16) IVF_STAGE(64, 8) IVF_STAGE(64, 4) IVF_STAGE(64, 2) IVF_STAGE(64, 1)
#undef IVF_STAGE
    return c;
}
// Out-of-line copies: a kernel that sorts in several places then holds (and fetches) the
// network once.  CALL = true selects them; the streaming scan kernel keeps the inline form.
__device__ __attribute__((noinline)) Cand bitonic_merge64_call(Cand c) { return bitonic_merge64_inline(c); }
__device__ __attribute__((noinline)) Cand bitonic_sort64_call(Cand c) { return bitonic_sort64_inline(c); }
template <bool CALL> __device__ __forceinline__ Cand bitonic_merge64(Cand c) {
    if (CALL) return bitonic_merge64_call(c);
    return bitonic_merge64_inline(c);
}
template <bool CALL> __device__ __forceinline__ Cand bitonic_sort64(Cand c) {
    if (CALL) return bitonic_sort64_call(c);
    return bitonic_sort64_inline(c);
}

// The first 64 of (a u p), sorted; a and p sorted.  `dropped` receives this lane's loser.
template <bool CALL>
__device__ __forceinline__ Cand merge_best64(Cand a, Cand p, Cand& dropped) {
    Cand rev = mirror(p);
    const bool take = rev > a;
    dropped = take ? a : rev;
    return bitonic_merge64<CALL>(take ? rev : a);
}
template <bool CALL>
__device__ __forceinline__ Cand merge_best64(Cand a, Cand p) {
    Cand dropped;
    return merge_best64<CALL>(a, p, dropped);
}

// ---- wavefront-resident top-k ------------------------------------------------------------------
// The 64*KL best row candidates seen by a wavefront, best first: entry e lives in register
// e / 64 of lane e % 64.  New candidates wait in a 64-entry pending buffer (one per lane) and
// are folded in by a sort + bitonic merge when it fills up or on flush().
// `thr` is the key of entry kprime-1 of the sorted part: a key below it cannot matter.
template <int KL, bool CALL>
struct WaveTopK {
    Cand top[KL];
    Cand pend;
    int pcount;
    float thr;

    __device__ __forceinline__ void init() {
#pragma unroll
        for (int j = 0; j < KL; ++j) top[j] = 0;
        pend = 0; pcount = 0;
        thr = -INFINITY;
    }

    // Folds a sorted run of 64 candidates (one per lane) into the list.
    __device__ __forceinline__ void merge_run(Cand run, int kprime) {
        if (KL == 1) {
            top[0] = merge_best64<CALL>(top[0], run);
        } else {
            // the best 128 of (L0, L1, P) are L0 plus the best 64 of (L1 u P), re-split
            top[KL - 1] = merge_best64<CALL>(top[KL - 1], run);
            Cand rev = mirror(top[KL - 1]);
            const bool take = rev > top[0];
            Cand lo = take ? top[0] : rev;
            top[0] = bitonic_merge64<CALL>(take ? rev : top[0]);
            top[KL - 1] = bitonic_merge64<CALL>(lo);
        }
        const int last = kprime - 1;
        Cand e = 0;
#pragma unroll
        for (int j = 0; j < KL; ++j)
            if ((last >> 6) == j) e = read_lane(top[j], last & 63);
        thr = e ? cand_key(e) : -INFINITY;
    }
    // a run whose best entry is below the threshold cannot change the list
    __device__ __forceinline__ void merge_run_if_useful(Cand run, int kprime) {
        const Cand head = read_lane(run, 0);
        if (head != 0 && cand_key(head) >= thr) merge_run(run, kprime);
    }

    __device__ __forceinline__ void flush(int kprime) {
        if (pcount == 0) return;
        merge_run(bitonic_sort64<CALL>(pend), kprime);
        pend = 0; pcount = 0;
    }

    // Called by the whole wavefront with a uniform candidate; the caller flushes before the
    // pending buffer (64 entries) can overflow.
    __device__ __forceinline__ void push(float key, uint32_t tie) {
        if (lane_id() == pcount) pend = pack_cand(key, tie);
        ++pcount;
    }
};

}  // namespace dev
}  // namespace ivf
