// Relevance metric of Sec. 3.1 (1), Eq. 5-8, on the vector ALUs (fp32 FMA).
//
// This is the path for fp32 metrics and the fallback for 16-bit metrics whose shape the MFMA
// kernels do not cover.  A workgroup takes one batch of T pairs from the dense pair list
// (the fixed-size batch of Algorithm 2), keeps the activations of the whole batch in LDS and
// walks the layers; a thread owns one pair and a strided set of output units, so a weight is
// read once per wave (all lanes of a wave share the output unit) and the activations are
// read from LDS with an odd row stride (no bank conflicts).
//
// Numerics, fp32 mode: x = concat(user, item) (Eq. 5); every layer is a sequential FMA chain
// over the inputs in index order (Eq. 7) carried in fp64 (the vector ALUs run fp64 at half the
// fp32 rate, and this mode is the reference-precision one), ReLU on hidden layers,
// relevance = sum_j w_j / (1 + exp(-z_j)) in fp64 (Eq. 8), rounded once to fp32.  Rank
// decisions therefore see the correctly rounded relevance, not fp32 summation noise.
// bf16 and fp16 modes: inputs and weights are widened to fp32, fp32 FMA chains with the bias
// added last, every hidden activation rounded to the 16-bit format (nearest even) after the ReLU;
// logits, sigmoid and the weighted sum in fp32 (the arithmetic of the MFMA kernels, on the plain ALUs).
#include "common.h"

namespace gmpgr {

constexpr int ALU_BLOCK = 256;

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t float_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) return (uint16_t)(u >> 16) | ((u & 0xffffu) ? 0x40 : 0);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// binary16 <-> fp32 through the hardware's conversions (nearest even, subnormals kept)
__device__ __forceinline__ float f16_bits_to_float(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
__device__ __forceinline__ uint16_t float_to_f16_rne(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

// KIND: the library's dtype code (ANN_F32, ANN_BF16, ANN_F16)
template <int KIND> struct Elem;
template <> struct Elem<ANN_F32> {
    using type = float;   // storage of items, users, weights
    using act = double;   // activations in LDS and accumulators
    static __device__ __forceinline__ float load(const float *p, size_t i) { return p[i]; }
    static __device__ __forceinline__ double fma(float w, double x, double acc) { return ::fma((double)w, x, acc); }
    static __device__ __forceinline__ double hidden(double a) { return a > 0.0 ? a : 0.0; }
    static __device__ __forceinline__ double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }
};
template <> struct Elem<ANN_BF16> {
    using type = uint16_t;
    using act = float;
    static __device__ __forceinline__ float load(const uint16_t *p, size_t i) { return bf16_bits_to_float(p[i]); }
    static __device__ __forceinline__ float fma(float w, float x, float acc) { return fmaf(w, x, acc); }
    static __device__ __forceinline__ float hidden(float a) {
        return bf16_bits_to_float(float_to_bf16_rne(fmaxf(a, 0.f)));
    }
    static __device__ __forceinline__ float sigmoid(float z) { return 1.0f / (1.0f + expf(-z)); }
};

template <> struct Elem<ANN_F16> {
    using type = uint16_t;
    using act = float;
    static __device__ __forceinline__ float load(const uint16_t *p, size_t i) { return f16_bits_to_float(p[i]); }
    static __device__ __forceinline__ float fma(float w, float x, float acc) { return fmaf(w, x, acc); }
    static __device__ __forceinline__ float hidden(float a) {
        return f16_bits_to_float(float_to_f16_rne(fmaxf(a, 0.f)));
    }
    static __device__ __forceinline__ float sigmoid(float z) { return 1.0f / (1.0f + expf(-z)); }
};

struct AluMlpParams {
    int32_t n_layers;
    int32_t dims[MAX_LAYERS + 1];
    int64_t w_off[MAX_LAYERS];
    int32_t b_off[MAX_LAYERS];
    int32_t d_user, d_item, J;
    float head_w[MAX_HEADS];
};

// act buffers: two ping-pong arrays of T rows with row stride `stride` floats (odd).
template <int KIND>
__global__ void __launch_bounds__(ALU_BLOCK)
mlp_alu_kernel(AluMlpParams P, const typename Elem<KIND>::type *__restrict__ emb, int64_t N,
               const typename Elem<KIND>::type *__restrict__ users, int32_t Q,
               const typename Elem<KIND>::type *__restrict__ W, const float *__restrict__ b,
               const int32_t *__restrict__ pair_q, const int32_t *__restrict__ pair_id,
               const int32_t *__restrict__ M_dev, int64_t M_max, float *__restrict__ scores, int T, int stride) {
    extern __shared__ __align__(16) unsigned char act_raw[];
    using E = Elem<KIND>;
    using A = typename E::act;
    A *act = (A *)act_raw;
    int64_t M = M_dev ? (int64_t)*M_dev : M_max;
    if (M > M_max) M = M_max;
    A *buf0 = act, *buf1 = act + (size_t)T * stride;
    const int r = threadIdx.x % T;       // pair inside the batch
    const int og = threadIdx.x / T;      // first output unit of this thread
    const int n_og = ALU_BLOCK / T;
    const int64_t n_tiles = (M + T - 1) / T;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t row = tile * T + r;
        const bool live = row < M;
        int32_t q = live ? pair_q[row] : -1;
        int32_t v = live ? pair_id[row] : -1;
        const bool ok = live && q >= 0 && q < Q && v >= 0 && (int64_t)v < N;
        // x = concat(user, item), Eq. 5
        for (int i = og; i < P.dims[0]; i += n_og) {
            A x = 0;
            if (ok) x = (i < P.d_user) ? E::load(users, (size_t)q * P.d_user + i)
                                       : E::load(emb, (size_t)v * P.d_item + (i - P.d_user));
            buf0[r * stride + i] = x;
        }
        __syncthreads();
        A *in = buf0, *out = buf1;
        for (int l = 0; l < P.n_layers; ++l) {
            const int n_in = P.dims[l], n_out = P.dims[l + 1];
            const bool last = (l == P.n_layers - 1);
            const typename E::type *Wl = W + P.w_off[l];
            const float *bl = b + P.b_off[l];
            const A *xin = in + r * stride;
            for (int o = og; o < n_out; o += n_og) {
                A acc = 0;
                const typename E::type *wrow = Wl + (size_t)o * n_in;
                for (int i = 0; i < n_in; ++i) acc = E::fma(E::load(wrow, i), xin[i], acc);
                acc += (A)bl[o];
                if (!last) acc = E::hidden(acc);
                out[r * stride + o] = acc;
            }
            __syncthreads();
            A *t = in;
            in = out;
            out = t;
        }
        if (og == 0 && live) {
            A s = 0;
            for (int j = 0; j < P.J; ++j) s += (A)P.head_w[j] * E::sigmoid(in[r * stride + j]);
            scores[row] = ok ? (float)s : __uint_as_float(0x7fc00000u);
        }
        __syncthreads();
    }
}

int launch_mlp_alu(const ann_graph *g, const ann_mlp *m, const void *queries, const int32_t *pair_q,
                   const int32_t *pair_id, const int32_t *M_dev, int64_t M_max, int32_t Q, float *scores,
                   int32_t tile_rows, hipStream_t stream) {
    if (M_max <= 0) return ANN_OK;
    AluMlpParams P;
    P.n_layers = m->n_layers;
    int maxw = 0;
    for (int l = 0; l <= m->n_layers; ++l) {
        P.dims[l] = m->dims[l];
        if (m->dims[l] > maxw) maxw = m->dims[l];
    }
    for (int l = 0; l < m->n_layers; ++l) {
        P.w_off[l] = m->w_off[l];
        P.b_off[l] = m->b_off[l];
    }
    P.d_user = m->d_user;
    P.d_item = m->d_item;
    P.J = m->J;
    for (int j = 0; j < m->J; ++j) P.head_w[j] = m->head_w[j];
    const int stride = maxw | 1;
    const bool half = (m->dtype != ANN_F32);  // a 16-bit metric: fp32 activations
    const size_t asz = half ? sizeof(float) : sizeof(double);
    // largest batch (pairs per workgroup) whose two activation buffers fit in 144 KB of LDS
    int T = 64;
    if (tile_rows > 0 && tile_rows < 64) {
        T = 1;
        while (T * 2 <= tile_rows) T *= 2;
    }
    // A small list (at most M_max pairs) is spread over more workgroups: fewer pairs per workgroup means more
    // threads per pair, i.e. fewer output units (sequential FMA chains) per thread.  A pair's arithmetic does
    // not depend on the batch it is in.
    if (tile_rows <= 0)
        while (T > 4 && (M_max + T - 1) / T < 512) T >>= 1;
    while (T > 1 && (size_t)2 * T * stride * asz > 144 * 1024) T >>= 1;
    size_t smem = (size_t)2 * T * stride * asz;
    if (smem > 144 * 1024) {
        set_error("layer width %d does not fit the ALU kernel", maxw);
        return ANN_ENOTIMPL;
    }
    const void *fn = m->dtype == ANN_BF16  ? (const void *)mlp_alu_kernel<ANN_BF16>
                     : m->dtype == ANN_F16 ? (const void *)mlp_alu_kernel<ANN_F16>
                                           : (const void *)mlp_alu_kernel<ANN_F32>;
    if (smem > 48 * 1024) {
        static std::atomic<uint32_t> raised[3];
        int rc = raise_lds_limit(fn, 144 * 1024, m->device, raised[m->dtype == ANN_BF16 ? 1 : m->dtype == ANN_F16 ? 2 : 0]);
        if (rc != ANN_OK) return rc;
    }
    int64_t tiles = (M_max + T - 1) / T;
    int grid = (int)(tiles < 4096 ? tiles : 4096);
    if (m->dtype == ANN_BF16)
        hipLaunchKernelGGL(mlp_alu_kernel<ANN_BF16>, dim3(grid), dim3(ALU_BLOCK), smem, stream, P,
                           (const uint16_t *)g->emb, g->N, (const uint16_t *)queries, Q,
                           (const uint16_t *)m->W_dev, m->b_dev, pair_q, pair_id, M_dev, M_max, scores, T, stride);
    else if (m->dtype == ANN_F16)
        hipLaunchKernelGGL(mlp_alu_kernel<ANN_F16>, dim3(grid), dim3(ALU_BLOCK), smem, stream, P,
                           (const uint16_t *)g->emb, g->N, (const uint16_t *)queries, Q,
                           (const uint16_t *)m->W_dev, m->b_dev, pair_q, pair_id, M_dev, M_max, scores, T, stride);
    else
        hipLaunchKernelGGL(mlp_alu_kernel<ANN_F32>, dim3(grid), dim3(ALU_BLOCK), smem, stream, P,
                           (const float *)g->emb, g->N, (const float *)queries, Q, (const float *)m->W_dev,
                           m->b_dev, pair_q, pair_id, M_dev, M_max, scores, T, stride);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

}  // namespace gmpgr
