// ann_score_pairs_noalloc: the relevance of an explicit pair list for callers that cannot allocate
// device memory (HIP graph capture, tight serving loops, harnesses that forbid it).
//
// ann_score_pairs keeps two things in a temporary it allocates and frees per call: the number of pairs,
// which the MFMA kernels read from device memory, and the per-query user term of the first layer
// (Q x H1 fp32).  Here both live in a fixed array that is part of the library's code object on every GPU
// it runs on.  Host code never uses the array's name as an address: the device address is looked up
// once per device with hipGetSymbolAddress and kept.
#include <mutex>

#include "common.h"

namespace gmpgr {

// 8 MiB of user terms (Q * H1 <= 2^21 floats: 4,096 queries of a 512-wide first layer) + the count block
// + the block one MFMA kernel pre-loads past the last row.
constexpr size_t SCRATCH_COUNT_BYTES = 256;
constexpr size_t SCRATCH_UPRE_FLOATS = (size_t)1 << 21;
constexpr size_t SCRATCH_BYTES = SCRATCH_COUNT_BYTES + (SCRATCH_UPRE_FLOATS + 32) * sizeof(float);

static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 32;
static std::mutex g_scratch_lock;
static unsigned char *g_scratch_ptr[MAX_DEVICES] = {};

// The array's address on the current device (each GPU holds its own copy); nullptr + error on failure.
static unsigned char *scratch_on_current_device(int *device_out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        set_error("no current device, or its index is beyond %d", MAX_DEVICES - 1);
        return nullptr;
    }
    *device_out = dev;
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_error("hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = (unsigned char *)p;
    }
    return g_scratch_ptr[dev];
}

// A kernel, not a memset or a copy: a caller may be recording the stream into a HIP graph.
__global__ void store_count_kernel(int32_t *dst, int32_t value) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *dst = value;
}

}  // namespace gmpgr

using namespace gmpgr;

extern "C" int ann_score_pairs_noalloc(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q,
                                       int64_t M, const int32_t *q_idx_dev, const int32_t *item_dev, float *out_dev,
                                       void *stream) {
    if (!g || !m) {
        set_error("null graph or metric handle");
        return ANN_EINVAL;
    }
    if (m->d_item != g->d || m->dtype != g->dtype) {
        set_error("metric (item width %d, dtype %d) does not match graph (%d, %d)", m->d_item, m->dtype, g->d,
                  g->dtype);
        return ANN_EINVAL;
    }
    if (M < 0 || M > 0x7fffffffll || Q < 1) {
        set_error("need 0 <= M < 2^31 and Q >= 1");
        return ANN_EINVAL;
    }
    if (M == 0) return ANN_OK;
    if (!queries_dev || !q_idx_dev || !item_dev || !out_dev) {
        set_error("queries_dev, q_idx_dev, item_dev and out_dev must not be null");
        return ANN_EINVAL;
    }
    hipStream_t s = (hipStream_t)stream;
    if (m->kernel != MLP_MFMA2)  // the plain ALU kernels take the count as an argument and need no user term
        return launch_mlp_alu(g, m, queries_dev, q_idx_dev, item_dev, nullptr, M, Q, out_dev, 0, s);
    const size_t need = (size_t)Q * (size_t)m->dims[1];
    if (need > SCRATCH_UPRE_FLOATS) {
        set_error("Q * first hidden width = %zu exceeds the %zu floats of the fixed scratch array "
                  "(use ann_score_pairs, which allocates)", need, SCRATCH_UPRE_FLOATS);
        return ANN_EINVAL;
    }
    int dev = -1;
    unsigned char *base = scratch_on_current_device(&dev);
    if (!base) return ANN_EDEVICE;
    if (dev != m->device) {
        set_error("the metric was loaded on device %d, the current device is %d", m->device, dev);
        return ANN_EINVAL;
    }
    int32_t *count = (int32_t *)base;
    float *upre = (float *)(base + SCRATCH_COUNT_BYTES);
    hipLaunchKernelGGL(store_count_kernel, dim3(1), dim3(64), 0, s, count, (int32_t)M);
    ANN_HIP_TRY(hipGetLastError());
    int rc = launch_user_pre(m, queries_dev, Q, upre, s);
    if (rc != ANN_OK) return rc;
    return launch_mlp_mfma(g, m, upre, q_idx_dev, item_dev, count, M, Q, out_dev, 0, s);
}
