// Sorted 64-bit keys shared by the search kernels and the exhaustive search: the order-preserving key of a
// (relevance, id) pair, an LDS bitonic sort and a binary search.
#pragma once

#include "common.h"

namespace gmpgr {

// ---- order-preserving key: ascending uint64 == (score descending, id ascending) ----------
__device__ __forceinline__ uint64_t make_key(float score, int32_t id, uint32_t expanded) {
    uint32_t f = __float_as_uint(score);
    uint32_t asc = (f & 0x80000000u) ? ~f : (f | 0x80000000u);
    return ((uint64_t)(~asc) << 32) | ((uint64_t)(uint32_t)id << 1) | expanded;
}
__device__ __forceinline__ float key_score(uint64_t key) {
    uint32_t asc = ~(uint32_t)(key >> 32);
    uint32_t f = (asc & 0x80000000u) ? (asc ^ 0x80000000u) : ~asc;
    return __uint_as_float(f);
}
__device__ __forceinline__ int32_t key_id(uint64_t key) { return (int32_t)((uint32_t)key >> 1); }
__device__ __forceinline__ uint32_t key_expanded(uint64_t key) { return (uint32_t)key & 1u; }

// Ascending bitonic sort of keys[0..n) in LDS, n a power of two.  Thread t owns the t-th
// compare-exchange of every step (and t + BLOCK, ...): for strides up to 64 the 64 threads of a
// wave then touch one and the same 128-key segment step after step, so those steps need no
// workgroup barrier, only the wave's own program order (LDS executes a wave's operations in
// order); a barrier is needed around the steps with larger strides and at the end.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int BLK>
__device__ void bitonic_sort(uint64_t *keys, int n) {
    for (int k = 2; k <= n; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            const bool across_waves = j > 64;
            if (across_waves) __syncthreads();
            for (int t = threadIdx.x; t < (n >> 1); t += BLK) {
                // t-th compare-exchange of this step: indices i < ixj
                int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                int ixj = i | j;
                bool up = ((i & k) == 0);
                uint64_t a = keys[i], b = keys[ixj];
                if ((a > b) == up) {
                    keys[i] = b;
                    keys[ixj] = a;
                }
            }
            if (across_waves) __syncthreads();
            else wave_lds_fence();
        }
    }
    __syncthreads();
}

// First index of the ascending a[0..n) whose key is not below `key`.
__device__ __forceinline__ int lower_bound_keys(const uint64_t *a, int n, uint64_t key) {
    int lo = 0, hi = n;
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (a[mid] < key) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

}  // namespace gmpgr
