// Device-side building blocks for the IVF kernels (gfx950, wave64).
#pragma once
#include "ivf_internal.h"
#include <hip/hip_runtime.h>

namespace ivf {
namespace dev {

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

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

// ---- block-wide radix select -----------------------------------------------------------------
// Finds, among n keys (key_at(i), smaller = better), the split that keeps the `want` smallest.
// On return every thread holds: `mask` (the high bits decided), `prefix` (their value for the
// boundary group), `need` (how many keys of the boundary group, (key & mask) == prefix, are
// kept) and `group` (size of that group).  Keys with (key & mask) < prefix are all kept.
// need == group unless the boundary group is a set of fully equal keys.
// hist: 256 words of LDS; sh: 4 words of LDS.  Must be called by all threads of the block.
template <typename KeyT, typename KeyAt>
__device__ void block_radix_select(KeyAt key_at, uint32_t n, uint32_t want, uint32_t* hist,
                                   uint32_t* sh, KeyT& mask, KeyT& prefix, uint32_t& need,
                                   uint32_t& group) {
    const int tid = threadIdx.x, nt = blockDim.x;
    mask = 0; prefix = 0; need = want; group = n;
    for (int shift = (int)sizeof(KeyT) * 8 - 8; shift >= 0; shift -= 8) {
        for (int i = tid; i < 256; i += nt) hist[i] = 0;
        __syncthreads();
        for (uint32_t i = tid; i < n; i += nt) {
            KeyT k = key_at(i);
            if ((k & mask) == prefix) atomicAdd(&hist[(uint32_t)(k >> shift) & 255u], 1u);
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
        if (need == group) break;
    }
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

// ---- wavefront-resident sorted candidate list ---------------------------------------------------
// The 64*KL best (key, row) pairs seen by a wavefront, best first: entry e lives in register
// e / 64 of lane e % 64.  Larger key is better; equal keys are ordered by smaller id.
// `thr` is the key of entry kprime-1: a candidate below it cannot enter the first kprime.
template <int KL>
struct TopList {
    float key[KL];
    uint32_t row[KL];
    float thr;

    __device__ __forceinline__ void init() {
#pragma unroll
        for (int j = 0; j < KL; ++j) { key[j] = -INFINITY; row[j] = kNoRow; }
        thr = -INFINITY;
    }

    __device__ static __forceinline__ int64_t id_of(uint32_t r, const int64_t* ids) {
        if (r == kNoRow) return INT64_MAX;
        return ids ? ids[r] : (int64_t)r;
    }

    // Called by the whole wavefront with a uniform candidate.
    __device__ __forceinline__ void insert(float ckey, uint32_t crow, const int64_t* ids, int kprime) {
        const int lane = lane_id();
        int pos = 0;
#pragma unroll
        for (int j = 0; j < KL; ++j) {
            bool before = key[j] > ckey;
            if (key[j] == ckey) before = id_of(row[j], ids) < id_of(crow, ids);
            pos += __popcll(__ballot(before));
        }
        if (pos >= 64 * KL) return;
#pragma unroll
        for (int j = KL - 1; j >= 0; --j) {
            float uk = __shfl_up(key[j], 1);
            uint32_t ur = __shfl_up(row[j], 1);
            if (j > 0) {
                float ck = read_lane(key[j - 1], 63);
                uint32_t cr = read_lane(row[j - 1], 63);
                if (lane == 0) { uk = ck; ur = cr; }
            }
            int e = j * 64 + lane;
            if (e == pos) { key[j] = ckey; row[j] = crow; }
            else if (e > pos) { key[j] = uk; row[j] = ur; }
        }
        const int last = kprime - 1;
#pragma unroll
        for (int j = 0; j < KL; ++j)
            if ((last >> 6) == j) thr = read_lane(key[j], last & 63);
    }
};

}  // namespace dev
}  // namespace ivf
