// Shared declarations of the HIP library: handles, workspace plan, kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>
#include <stddef.h>

#include "../../include/gmpgr_ann.h"

namespace gmpgr {

constexpr int MAX_LAYERS = 8;
constexpr int MAX_WIDTH = 2048;
constexpr int MAX_HEADS = 8;
constexpr int MAX_WR = 4096;        // W*R candidates per query and round
constexpr int MAX_E = 1024;
constexpr uint32_t EMPTY_SLOT = 0xFFFFFFFFu;
constexpr uint64_t KEY_SENTINEL = 0xFFFFFFFFFFFFFFFFull;

void set_error(const char *fmt, ...);

#define ANN_HIP_TRY(expr)                                                                \
    do {                                                                                 \
        hipError_t _e = (expr);                                                          \
        if (_e != hipSuccess) {                                                          \
            gmpgr::set_error("%s failed: %s", #expr, hipGetErrorString(_e));             \
            return ANN_EDEVICE;                                                          \
        }                                                                                \
    } while (0)

// Raises a kernel's dynamic-LDS limit once per device: the runtime call is a host-side lookup that
// need not be repeated on every one of the hundreds of launches of a search.  `done` is the
// launcher's own bit mask of devices already served.
inline int raise_lds_limit(const void *fn, size_t bytes, int device, std::atomic<uint32_t> &done) {
    const bool tracked = device >= 0 && device < 32;
    if (tracked && ((done.load(std::memory_order_acquire) >> device) & 1u)) return ANN_OK;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) {
        set_error("hipFuncSetAttribute(dynamic LDS %zu) failed: %s", bytes, hipGetErrorString(e));
        return ANN_EDEVICE;
    }
    if (tracked) done.fetch_or(1u << device, std::memory_order_release);
    return ANN_OK;
}

// The logistic function of Eq. 8's heads for the 16- and 8-bit metrics: the hardware's base-2 exponential and
// reciprocal, each within one unit in the last place (5 instructions against about 25 for expf and an IEEE
// division; 0 and 1 at the ends of the range, never NaN for a finite argument).
__device__ __forceinline__ float sigmoid_hw(float z) {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}

}  // namespace gmpgr

struct ann_graph {
    const int32_t *adj;
    const void *emb;
    int64_t N;
    int32_t R, d, dtype;
    // locality order of the visited bitmap (ann_graph_set_locality): rank is the caller's [N] permutation,
    // adj_rank the library's own [N][R] table rank[adj]; both null = bits by id
    const int32_t *rank = nullptr;
    int32_t *adj_rank = nullptr;
};

// Which fused kernel serves the metric.
enum MlpKernel { MLP_ALU = 0, MLP_MFMA2 = 1 /* the bf16 MFMA kernels: one or two hidden layers */ };

struct ann_mlp {
    int32_t n_layers;
    int32_t dims[gmpgr::MAX_LAYERS + 1];
    int32_t d_user, d_item, dtype, J;
    int32_t kernel;        // MlpKernel
    // plain copies, layer l at w_off[l] (elements) in W_dev, b_off[l] in b_dev
    void *W_dev;           // fp32 or bf16, [out][in] row-major per layer
    float *b_dev;
    float *head_w_dev;
    int64_t w_off[gmpgr::MAX_LAYERS];
    int32_t b_off[gmpgr::MAX_LAYERS];
    float head_w[gmpgr::MAX_HEADS];
    // MFMA path: fragment-ordered bf16 copies (see mlp_mfma.hip)
    void *frag_dev;        // W1 item half, W2, W_last (padded to 32 rows), in fragment order
    int64_t frag_bytes;
    int device;
};

namespace gmpgr {

// Device workspace layout; every offset is in bytes from the workspace base, 256-aligned.
struct Plan {
    int32_t Q, E, W_max, L_max, k, C, R, max_iters_max, rounds_assumed;
    int32_t slots;          // survivors kept per query and round: max(W_max*R, E)
    int32_t hash_cap;       // per-query visited table entries (power of two)
    int32_t bitmap_words;   // > 0: the visited set is a bitmap of this many 32-bit words per query instead
    int64_t M_max;          // Q * slots
    int32_t H1;             // first hidden width (user-half pre-activations), 0 if unused
    size_t off_ctrl, off_state, off_pool, off_hash, off_cand, off_tag, off_counts, off_offsets,
        off_pair_q, off_pair_id, off_scores, off_upre, off_stats;
    size_t total;
};

// Control block at off_ctrl (device), 64 int32.
struct Ctrl {
    int32_t M;            // pairs in the current round
    int32_t n_active;     // queries not finished
    int32_t next_query;   // continuous batching: queries admitted so far (a closed batch may overshoot its total)
    int32_t avail;        // open stream: queries that have arrived so far
    int32_t pad[12];
};

// Per-query state at off_state.
struct alignas(16) QState {
    int32_t t;            // rounds done
    int32_t done;         // bit 0 = finished, bit 1 = stopped because its visited table was full
    int32_t n_list;       // entries in the list
    int32_t n_visited;    // ids in the visited table = pairs scored for this query
    int32_t W, L, cap;    // this query's parameters
    int32_t n_expanded;   // nodes whose neighbours were fetched
    int32_t first_open;   // every list rank below this one has been expanded (a lower bound of the first open rank)
    int32_t pad[3];
};
static_assert(sizeof(QState) == 48, "QState is read and written as three 16-byte pieces");

bool make_plan(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t E, int32_t W_max,
               int32_t L_max, int32_t k, int32_t max_iters_max, Plan *p);

struct SearchArgs {
    const ann_graph *g;
    const ann_mlp *m;
    const void *queries;
    const int32_t *entries;
    const int32_t *W_q, *L_q, *cap_q;  // null = uniform
    int32_t W, L, cap;
    char *ws;
    Plan plan;
    int32_t *out_ids;
    float *out_scores;
    hipStream_t stream;
    bool keep_stats = false;  // counters continue from an earlier search on this workspace
    // continuous batching: Q_total queries share plan.Q slots
    int32_t Q_total = 0;          // 0 = every query owns a slot; -1 = open stream (queries keep arriving)
    int32_t Q_rows = 0;           // open stream: rows of the caller's query arrays
    int32_t *slot_query = nullptr;  // [plan.Q] query served by each slot, -1 = idle
    float *upre_all = nullptr;    // [Q_total][H1] user terms of all queries (MFMA path)
    // paper-literal variant: one walker per seed, plan.max_iters_max hops (see round_kernel)
    bool walkers = false;
    // progress word in pinned host memory, written by the packing step of every round (null = none):
    // mail_tag | (rounds packed << 1) | finished
    uint64_t *mailbox = nullptr;
    uint64_t mail_tag = 0;
    int32_t round_index = 0;
};

// search_kernels.hip
int launch_init(const SearchArgs &a);
int launch_scan_compact(const SearchArgs &a);
int launch_round(const SearchArgs &a);
int launch_emit(const SearchArgs &a);
int launch_stream_reset(const SearchArgs &a);
int launch_admit(const SearchArgs &a);
int launch_stream_publish(const SearchArgs &a, int avail);

// noise.hip: out = users + sigma * N(0, I), element-indexed counter-based draw (Eq. 5)
int launch_users_add_noise(const void *users, void *out, int64_t n_elem, int dtype, double sigma, uint64_t seed,
                           uint64_t stream_id, hipStream_t stream);

// mlp_mfma_f8.hip: the 8-bit (e4m3) metric
bool f8_supported(const int32_t *dims, int32_t n_layers, int32_t d_user);
int build_f8_fragments(ann_mlp *m, const void *const *W_host, hipStream_t stream);
int launch_mlp_mfma_f8(const ann_graph *g, const ann_mlp *m, const float *upre, const int32_t *pair_q,
                       const int32_t *pair_id, const int32_t *M_dev, int64_t M_max, int32_t Q, float *scores,
                       hipStream_t stream);
int launch_quantize_e4m3(const void *in, int dtype, int64_t n, float scale, uint8_t *out, hipStream_t stream);

// mlp_alu.hip / mlp_mfma.hip: score `*M_dev` (<= M_max) pairs; M_dev is read on the device.
int launch_mlp_alu(const ann_graph *g, const ann_mlp *m, const void *queries, const int32_t *pair_q,
                   const int32_t *pair_id, const int32_t *M_dev, int64_t M_max, int32_t Q, float *scores,
                   int32_t tile_rows, hipStream_t stream);
int launch_user_pre(const ann_mlp *m, const void *queries, int32_t Q, float *upre, hipStream_t stream);
int launch_mlp_mfma(const ann_graph *g, const ann_mlp *m, const float *upre, const int32_t *pair_q,
                    const int32_t *pair_id, const int32_t *M_dev, int64_t M_max, int32_t Q, float *scores,
                    int32_t tile_rows, hipStream_t stream);
bool mfma_supported(const int32_t *dims, int32_t n_layers, int32_t d_user, int32_t dtype);
// mlp_mfma_stream.hip: the hand-scheduled kernel for item width 128, hidden 512 x 256
bool mfma_stream_supported(int D, int H1, int H2);
int build_stream_fragments(ann_mlp *m, const void *const *W_host, hipStream_t stream);
int launch_mlp_mfma_stream(const ann_graph *g, const ann_mlp *m, const float *upre, const int32_t *pair_q,
                           const int32_t *pair_id, const int32_t *M_dev, int64_t M_max, int32_t Q, float *scores,
                           hipStream_t stream);
int build_mfma_fragments(ann_mlp *m, const void *const *W_host, hipStream_t stream);

}  // namespace gmpgr
