// Serendipity vector of the metric input (Eq. 5): users + sigma * h~, h~ ~ N(0, I), drawn on the device.
//
// The draw is a pure function of (seed, stream, element index e = q * d + c), so that it can be
// repeated anywhere:
//   Philox4x32-10 (Salmon et al., SC'11) with counter (block lo, block hi, stream lo, stream hi) and key
//   (seed lo, seed hi), block = e / 4; uniforms (x + 1/2) / 2^32; Box-Muller on the word pairs (0,1) and
//   (2,3): radius from the first word, angle from the second, cosine to the even element and sine to the
//   odd one; the sum is formed in fp64 and rounded fp64 -> fp32 (-> bf16, nearest even).
// One thread draws one block and writes its (up to) four elements; the whole array is Q*d elements, a few
// hundred KB for a batch of queries, so the kernel is bound by nothing but its launch.
#include "common.h"

namespace gmpgr {

struct Philox4 {
    uint32_t x[4];
};

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                 uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0, c1 = lo1, c2 = n2, c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Philox4{{c0, c1, c2, c3}};
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) return (uint16_t)(u >> 16);  // inf / nan unchanged
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// KIND: the library's dtype code of the array (ANN_F32, ANN_BF16, ANN_F16)
template <int KIND>
__global__ void __launch_bounds__(256)
users_add_noise_kernel(const void *__restrict__ users, void *__restrict__ out, int64_t n_elem, double sigma,
                       uint64_t seed, uint64_t stream_id) {
    const int64_t block = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t e0 = block * 4;
    if (e0 >= n_elem) return;
    const Philox4 r = philox4x32_10((uint32_t)block, (uint32_t)((uint64_t)block >> 32), (uint32_t)stream_id,
                                    (uint32_t)(stream_id >> 32), (uint32_t)seed, (uint32_t)(seed >> 32));
    double z[4];
#pragma unroll
    for (int a = 0; a < 4; a += 2) {
        const double ua = ((double)r.x[a] + 0.5) * (1.0 / 4294967296.0);
        const double ub = ((double)r.x[a + 1] + 0.5) * (1.0 / 4294967296.0);
        const double rad = sqrt(-2.0 * log(ua));
        const double ang = 6.283185307179586476925286766559 * ub;
        z[a] = rad * cos(ang);
        z[a + 1] = rad * sin(ang);
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int64_t e = e0 + t;
        if (e >= n_elem) break;
        if (KIND == ANN_BF16) {
            const float u = __uint_as_float((uint32_t)((const uint16_t *)users)[e] << 16);
            ((uint16_t *)out)[e] = f32_to_bf16_rne((float)((double)u + sigma * z[t]));
        } else if (KIND == ANN_F16) {
            const float u = (float)((const _Float16 *)users)[e];
            // fp64 -> fp32 -> binary16 as two roundings, like the bf16 branch (the empty statement keeps the compiler
            // from rounding the fp64 sum to binary16 in one step, which differs on the fp32 values that are ties)
            float f = (float)((double)u + sigma * z[t]);
            asm volatile("" : "+v"(f));
            ((_Float16 *)out)[e] = (_Float16)f;
        } else {
            ((float *)out)[e] = (float)((double)((const float *)users)[e] + sigma * z[t]);
        }
    }
}

int launch_users_add_noise(const void *users, void *out, int64_t n_elem, int dtype, double sigma, uint64_t seed,
                           uint64_t stream_id, hipStream_t stream) {
    if (n_elem == 0) return ANN_OK;
    const int64_t blocks4 = (n_elem + 3) / 4;
    const unsigned grid = (unsigned)((blocks4 + 255) / 256);
    auto fn = dtype == ANN_BF16  ? users_add_noise_kernel<ANN_BF16>
              : dtype == ANN_F16 ? users_add_noise_kernel<ANN_F16>
                                 : users_add_noise_kernel<ANN_F32>;
    hipLaunchKernelGGL(fn, dim3(grid), dim3(256), 0, stream, users, out, n_elem, sigma, seed, stream_id);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

}  // namespace gmpgr
