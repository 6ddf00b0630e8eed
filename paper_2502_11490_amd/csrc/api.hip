// C ABI of the library (include/gmpgr_ann.h): argument checks, handles, workspace plan and
// the host side of the round loop.  Every step of the search runs in the kernels of
// search_kernels.hip, mlp_alu.hip and mlp_mfma.hip; nothing here computes a score or a rank.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <chrono>
#include <mutex>
#include <sched.h>
#include <new>
#include <vector>

#include "common.h"

namespace gmpgr {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
static inline int next_pow2(int64_t x) {
    int64_t p = 1;
    while (p < x) p <<= 1;
    return (int)p;
}

constexpr size_t STATS_OFFSET = 256;  // bytes from the workspace base: int64[8] counters

bool make_plan(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t E, int32_t W_max, int32_t L_max,
               int32_t k, int32_t max_iters_max, Plan *p) {
    if (!g || !m) {
        set_error("null graph or metric handle");
        return false;
    }
    if (Q < 0 || E < 1 || W_max < 1 || L_max < 1 || k < 1 || max_iters_max < 0) {
        set_error("need Q >= 0, E >= 1, W >= 1, L >= 1, k >= 1, max_iters >= 0 (got Q=%d E=%d W=%d L=%d k=%d iters=%d)",
                  Q, E, W_max, L_max, k, max_iters_max);
        return false;
    }
    if (m->d_item != g->d) {
        set_error("metric expects item width %d, graph has %d", m->d_item, g->d);
        return false;
    }
    if (m->dtype != g->dtype) {
        set_error("metric dtype %d differs from graph dtype %d", m->dtype, g->dtype);
        return false;
    }
    if ((int64_t)W_max * g->R > MAX_WR || E > MAX_E) {
        set_error("W*R = %lld exceeds %d or E = %d exceeds %d", (long long)W_max * g->R, MAX_WR, E, MAX_E);
        return false;
    }
    p->Q = Q;
    p->E = E;
    p->W_max = W_max;
    p->L_max = L_max;
    p->k = k;
    p->R = g->R;
    p->max_iters_max = max_iters_max;
    p->C = L_max > k ? L_max : k;
    p->slots = W_max * g->R > E ? W_max * g->R : E;
    if ((int64_t)Q * p->C > (1ll << 40)) {
        set_error("Q * max(L,k) = %lld list entries is beyond any workspace", (long long)Q * p->C);
        return false;
    }
    // ids one query can score: seeds + rounds * W * R with a cap; without one, (2*L + 32*W) * R ids are
    // assumed (twice the expansions a list of L entries needs, plus slack for short lists)
    int64_t rounds = max_iters_max > 0 ? max_iters_max : 2 * (int64_t)((L_max + W_max - 1) / W_max) + 32;
    p->rounds_assumed = (int32_t)(rounds > 0x7fffffff ? 0x7fffffff : rounds);
    int64_t visited = (int64_t)E + rounds * W_max * g->R;
    if (visited > g->N) visited = g->N;
    int64_t cap = 2 * (visited + (int64_t)W_max * g->R);
    if (cap > (1ll << 30)) {
        set_error("visited table of %lld entries per query is too large", (long long)cap);
        return false;
    }
    p->hash_cap = next_pow2(cap < 64 ? 64 : cap);
    // one bit per item is the smaller visited set once the table outgrows N / 8 bytes (long lists): all probes
    // of a batch then fall into a far smaller address range, and seeding has far less to clear
    // (measured: already faster at 1.2 x the table's size; taken up to twice its size, for tables of a megabyte or
    // more: a small table is cheaper to clear than a bitmap of all items).  GMPGR_VISITED_SET =
    // "bitmap" / "hash" overrides the rule, for measurements and for tests of either form at any size.
    const int64_t words = ((g->N + 31) / 32 + 63) & ~63ll;
    bool bitmap = p->hash_cap >= (1 << 18) && words <= 2 * (int64_t)p->hash_cap;
    if (const char *force = getenv("GMPGR_VISITED_SET")) {
        if (!strcmp(force, "bitmap")) bitmap = true;
        if (!strcmp(force, "hash")) bitmap = false;
    }
    p->bitmap_words = bitmap ? (int32_t)words : 0;
    p->M_max = (int64_t)Q * p->slots;
    if (p->M_max > 0x7fffffffll) {
        set_error("Q * max(W*R,E) = %lld pairs per round exceeds 2^31", (long long)p->M_max);
        return false;
    }
    p->H1 = (m->kernel == MLP_MFMA2) ? m->dims[1] : 0;
    size_t o = 0;
    p->off_ctrl = o;
    o += STATS_OFFSET;
    p->off_stats = o;
    o += 256;
    p->off_state = o;
    o = align256(o + (size_t)Q * sizeof(QState));
    p->off_pool = o;
    o = align256(o + (size_t)Q * p->C * 8);
    p->off_hash = o;
    o = align256(o + (size_t)Q * (size_t)(p->bitmap_words > 0 ? p->bitmap_words : p->hash_cap) * 4);
    p->off_cand = o;
    o = align256(o + (size_t)Q * p->slots * 4);
    p->off_tag = o;  // which parent (or seed) produced each survivor
    o = align256(o + (size_t)Q * p->slots * 2);
    p->off_counts = o;
    o = align256(o + (size_t)Q * 4);
    p->off_offsets = o;
    o = align256(o + (size_t)Q * 4);
    p->off_pair_q = o;
    o = align256(o + (size_t)p->M_max * 4);
    p->off_pair_id = o;
    o = align256(o + (size_t)p->M_max * 4);
    p->off_scores = o;
    o = align256(o + (size_t)p->M_max * 4);
    p->off_upre = o;
    o = align256(o + ((size_t)Q * p->H1 + 32) * 4);  // +32: the MFMA kernel pre-loads one block past a row
    p->total = o;
    return true;
}

// "Has every query converged": the packing step of every round stores one progress word to pinned
// host memory (search tag, rounds packed so far, a finished bit).  The enqueuing thread reads it
// between launches: it stops when the finished bit is up and otherwise only makes sure that it is not
// more than AHEAD rounds in front of the device, so the stream never runs dry and no copy or
// synchronisation is put between the kernels.  A round enqueued after the batch has finished is
// three launches that find nothing to do.  "Finished" never reverts, so a late look is safe.
// One word per host thread; the tag tells a search's word from an older search's.  A thread's 64 pinned
// bytes are never freed: a destructor at thread exit could run after the runtime has shut down.
// Longest time an uncapped search waits for the next progress report of its kernels while the stream stays busy
// (seconds, 0 = no limit); see ann_set_progress_timeout.
static std::atomic<double> g_wait_limit_s{600.0};

struct Mailbox {
    static constexpr int AHEAD = 4;
    volatile uint64_t *host = nullptr;
    uint64_t *dev = nullptr;
    uint64_t seq = 0;
    bool ok = false;
    bool init() {
        if (ok) return true;
        void *h = nullptr, *d = nullptr;
        if (hipHostMalloc(&h, 64, hipHostMallocPortable | hipHostMallocMapped | hipHostMallocCoherent) != hipSuccess) return false;
        if (hipHostGetDevicePointer(&d, h, 0) != hipSuccess) {
            (void)hipHostFree(h);
            return false;
        }
        host = (volatile uint64_t *)h;
        dev = (uint64_t *)d;
        host[0] = 0;
        host[1] = 0;
        ok = true;
        return true;
    }
    void release() {  // only for a word that belongs to an object with an explicit end of life
        if (ok) (void)hipHostFree((void *)host);
        ok = false;
        host = nullptr;
        dev = nullptr;
    }
    uint64_t new_tag() {
        seq = (seq + 1) & 0xFFFFFFull;
        if (seq == 0) seq = 1;
        return seq << 40;
    }
    // Before enqueuing round `i` (0-based): 1 = the search has finished, 0 = go on, -1 = the stream reports an
    // error, or has run everything enqueued so far without the progress the kernels would have reported.
    // A wait that lasts (20 ms without the word it needs, again every 20 ms) asks the stream: a search enqueued
    // behind long work of the caller's waits as long as that takes, and a failed device ends the wait.  Rounds
    // take microseconds, so a running search never asks (a stream query is not free: asked every few thousand
    // spins it cost the small configurations, whose host thread mostly waits here, 0.4 ms per search).
    // *seen_rounds (if given): the number of rounds the device had packed in the word the answer came from.
    int gate(uint64_t tag, int64_t i, hipStream_t stream, int64_t *seen_rounds = nullptr) const {
        auto enough = [&](uint64_t w) {
            if ((w >> 40) != (tag >> 40)) return i <= AHEAD ? 0 : -2;  // nothing reported yet
            if (seen_rounds) *seen_rounds = (int64_t)((w & 0xFFFFFFFFFFull) >> 1);
            if (w & 1ull) return 1;
            return (int64_t)((w & 0xFFFFFFFFFFull) >> 1) + AHEAD >= i ? 0 : -2;
        };
        if (seen_rounds) *seen_rounds = 0;
        const auto start = std::chrono::steady_clock::now();
        auto last = start;
        uint64_t seen = *host;
        for (int spin = 0;; ++spin) {
            const uint64_t w = *host;
            int r = enough(w);
            if (r != -2) return r;
            if (spin > 4096) sched_yield();  // a long wait: let another thread have the core between looks
            if ((spin & 1023) == 1023) {
                const auto now = std::chrono::steady_clock::now();
                if (w != seen) {  // the device is making progress: the limit below counts from the last report
                    seen = w;
                    last = now;
                    continue;
                }
                if (now - last <= std::chrono::milliseconds(20)) continue;
                const hipError_t e = hipStreamQuery(stream);
                if (e == hipErrorNotReady) {
                    const double limit = g_wait_limit_s.load(std::memory_order_relaxed);
                    if (limit > 0 && std::chrono::duration<double>(now - last).count() > limit) return -3;
                    continue;
                }
                if (e != hipSuccess) return -1;
                r = enough(*host);  // the stream is idle: every packing kernel enqueued so far has reported
                return r != -2 ? r : -1;
            }
        }
    }
};

static Mailbox *mailbox() {
    static thread_local Mailbox box;
    return box.init() ? &box : nullptr;
}

// Optional stage timing (ann_profile_enable): every kernel launch of a stage is bracketed by two
// HIP events on the search's stream; ann_profile_read sums the elapsed times.
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> events;  // pairs: 2*i = start, 2*i+1 = stop
    std::vector<int> stage;
    size_t used = 0;
    hipEvent_t *next(int st) {
        if (used == stage.size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess) return nullptr;
            if (hipEventCreate(&b) != hipSuccess) {
                (void)hipEventDestroy(a);
                return nullptr;
            }
            events.push_back(a);
            events.push_back(b);
            stage.push_back(st);
        }
        stage[used] = st;
        return &events[2 * used++];
    }
};
static thread_local Profiler g_prof;

struct StageTimer {
    hipEvent_t *ev = nullptr;
    hipStream_t s;
    StageTimer(int stage, hipStream_t stream) : s(stream) {
        if (g_prof.on) {
            ev = g_prof.next(stage);
            if (ev) (void)hipEventRecord(ev[0], s);
        }
    }
    ~StageTimer() {
        if (ev) (void)hipEventRecord(ev[1], s);
    }
};

static int score_batch(const SearchArgs &a) {
    StageTimer timer(ANN_STAGE_SCORE, a.stream);
    const Plan &p = a.plan;
    const int32_t *M_dev = &((const Ctrl *)(a.ws + p.off_ctrl))->M;
    // pair_q names user vectors: slots and queries coincide unless queries stream through the slots
    const int32_t n_users = a.Q_total > 0 ? a.Q_total : a.Q_total < 0 ? a.Q_rows : p.Q;
    const float *upre = a.upre_all ? a.upre_all : (const float *)(a.ws + p.off_upre);
    if (a.m->kernel == MLP_MFMA2)
        return launch_mlp_mfma(a.g, a.m, upre, (const int32_t *)(a.ws + p.off_pair_q),
                               (const int32_t *)(a.ws + p.off_pair_id), M_dev, p.M_max, n_users,
                               (float *)(a.ws + p.off_scores), 0, a.stream);
    return launch_mlp_alu(a.g, a.m, a.queries, (const int32_t *)(a.ws + p.off_pair_q),
                          (const int32_t *)(a.ws + p.off_pair_id), M_dev, p.M_max, n_users,
                          (float *)(a.ws + p.off_scores), 0, a.stream);
}

static int run_search(SearchArgs &a) {
    const Plan &p = a.plan;
    int rc;
    if (p.Q == 0) return ANN_OK;
    if (a.m->kernel == MLP_MFMA2)
        if ((rc = launch_user_pre(a.m, a.queries, p.Q, (float *)(a.ws + p.off_upre), a.stream)) != ANN_OK) return rc;
    {
        StageTimer timer(ANN_STAGE_ROUND, a.stream);
        if ((rc = launch_init(a)) != ANN_OK) return rc;
    }
    const bool capped = p.max_iters_max > 0;
    Mailbox *box = nullptr;
    if (!capped) {
        box = mailbox();
        if (!box) {
            set_error("pinned host allocation failed");
            return ANN_ENOMEM;
        }
        a.mailbox = box->dev;
        a.mail_tag = box->new_tag();
    }
    bool overflow_seen = false;
    // a query expands only ids it has scored, so it cannot run more rounds than its visited
    // table holds ids: the loop is bounded even if no query ever reported convergence
    const int64_t round_limit = capped ? (int64_t)p.max_iters_max
                                       : (p.bitmap_words > 0 ? a.g->N : (int64_t)p.hash_cap / 2) + 1;
    for (int64_t i = 0; i <= round_limit; ++i) {
        if (box) {  // no query is running: nothing left to score or merge
            const int g = box->gate(a.mail_tag, i, a.stream);
            if (g > 0) break;
            if (g < 0) {
                set_error(g == -3 ? "no progress report from the search's kernels within the time limit (ann_set_progress_timeout)"
                                  : "the stream failed or ran dry without the search's progress report");
                return ANN_EDEVICE;
            }
        }
        a.round_index = (int32_t)i;
        {
            StageTimer timer(ANN_STAGE_PACK, a.stream);
            if ((rc = launch_scan_compact(a)) != ANN_OK) return rc;
        }
        if ((rc = score_batch(a)) != ANN_OK) return rc;
        {
            StageTimer timer(ANN_STAGE_ROUND, a.stream);
            if ((rc = launch_round(a)) != ANN_OK) return rc;
        }
    }
    if ((rc = launch_emit(a)) != ANN_OK) return rc;
    if (!capped) {
        int64_t stats[8];
        ANN_HIP_TRY(hipMemcpyAsync(stats, a.ws + p.off_stats, sizeof(stats), hipMemcpyDeviceToHost, a.stream));
        ANN_HIP_TRY(hipStreamSynchronize(a.stream));
        overflow_seen = stats[3] > 0;
        if (overflow_seen) {
            set_error("%lld queries filled their visited table (sized for %d rounds) and stopped early",
                      (long long)stats[3], p.rounds_assumed);
            return ANN_EWORKSPACE;
        }
    }
    return ANN_OK;
}

// Continuous batching: a.Q_total queries stream through a.plan.Q slots.  Every round starts with
// the admission kernel (finished slots write their result and take the next waiting query); the
// host learns every few rounds whether anything is still running or waiting.
static int run_stream(SearchArgs &a) {
    const Plan &p = a.plan;
    int rc;
    if (a.Q_total == 0 || p.Q == 0) return ANN_OK;
    if (a.m->kernel == MLP_MFMA2)
        if ((rc = launch_user_pre(a.m, a.queries, a.Q_total, a.upre_all, a.stream)) != ANN_OK) return rc;
    if ((rc = launch_stream_reset(a)) != ANN_OK) return rc;
    Mailbox *box = mailbox();
    if (!box) {
        set_error("pinned host allocation failed");
        return ANN_ENOMEM;
    }
    a.mailbox = box->dev;
    a.mail_tag = box->new_tag();
    // every query ends within hash_cap / 2 + 1 rounds of its admission, and at least one slot is
    // re-used per ceil(Q_total / Q) turn-overs: a generous bound that only guards against a bug
    const int64_t per_query = p.max_iters_max > 0 ? (int64_t)p.max_iters_max + 2
                                                  : (p.bitmap_words > 0 ? a.g->N : (int64_t)p.hash_cap / 2) + 3;
    const int64_t round_limit = per_query * (((int64_t)a.Q_total + p.Q - 1) / p.Q + 1);
    for (int64_t i = 0; i <= round_limit; ++i) {
        {   // nothing running after an admission step, and nothing left to admit: every result is written
            const int g = box->gate(a.mail_tag, i, a.stream);
            if (g > 0) break;
            if (g < 0) {
                set_error(g == -3 ? "no progress report from the search's kernels within the time limit (ann_set_progress_timeout)"
                                  : "the stream failed or ran dry without the search's progress report");
                return ANN_EDEVICE;
            }
        }
        a.round_index = (int32_t)i;
        {
            StageTimer timer(ANN_STAGE_ROUND, a.stream);
            if ((rc = launch_admit(a)) != ANN_OK) return rc;
        }
        {
            StageTimer timer(ANN_STAGE_PACK, a.stream);
            if ((rc = launch_scan_compact(a)) != ANN_OK) return rc;
        }
        if ((rc = score_batch(a)) != ANN_OK) return rc;
        {
            StageTimer timer(ANN_STAGE_ROUND, a.stream);
            if ((rc = launch_round(a)) != ANN_OK) return rc;
        }
    }
    int64_t stats[8];
    ANN_HIP_TRY(hipMemcpyAsync(stats, a.ws + p.off_stats, sizeof(stats), hipMemcpyDeviceToHost, a.stream));
    ANN_HIP_TRY(hipStreamSynchronize(a.stream));
    if (stats[3] > 0) {
        set_error("%lld queries filled their visited table (sized for %d rounds) and stopped early",
                  (long long)stats[3], p.rounds_assumed);
        return ANN_EWORKSPACE;
    }
    return ANN_OK;
}

}  // namespace gmpgr

using namespace gmpgr;

extern "C" {

const char *ann_last_error(void) { return g_err; }

__global__ void validate_adj_kernel(const int32_t *adj, int64_t n, int64_t N, int *bad) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t step = (int64_t)gridDim.x * blockDim.x;
    int found = 0;
    for (; i < n; i += step)
        if ((int64_t)adj[i] >= N) found = 1;
    if (found) atomicOr(bad, 1);
}

int ann_graph_load(const int32_t *adj_dev, const void *emb_dev, int64_t N, int32_t R, int32_t d, int32_t dtype,
                   uint32_t flags, void *stream, ann_graph **out) {
    if (!out) {
        set_error("out is null");
        return ANN_EINVAL;
    }
    *out = nullptr;
    if (!adj_dev || !emb_dev) {
        set_error("adj_dev and emb_dev must not be null");
        return ANN_EINVAL;
    }
    if (N < 1 || N >= (1ll << 31) || R < 1 || R > 64 || d < 1 || d > 1024) {
        set_error("need 1 <= N < 2^31, 1 <= R <= 64, 1 <= d <= 1024 (got N=%lld R=%d d=%d)", (long long)N, R, d);
        return ANN_EINVAL;
    }
    if (dtype != ANN_F32 && dtype != ANN_BF16 && dtype != ANN_F8 && dtype != ANN_F16) {
        set_error("dtype must be ANN_F32, ANN_BF16, ANN_F16 or ANN_F8");
        return ANN_EINVAL;
    }
    if (dtype == ANN_F8 && (((uintptr_t)emb_dev & 15) || (d & 15))) {
        set_error("an 8-bit item table needs a 16-byte aligned base and a width that is a multiple of 16");
        return ANN_EINVAL;
    }
    if (((uintptr_t)adj_dev & 3) || ((uintptr_t)emb_dev & 3)) {
        set_error("adj_dev and emb_dev must be 4-byte aligned");
        return ANN_EINVAL;
    }
    if (flags & ANN_VALIDATE) {
        int *bad = nullptr;
        hipStream_t s = (hipStream_t)stream;
        ANN_HIP_TRY(hipMalloc((void **)&bad, sizeof(int)));
        hipError_t e = hipMemsetAsync(bad, 0, sizeof(int), s);
        int h = 0;
        if (e == hipSuccess) {
            hipLaunchKernelGGL(validate_adj_kernel, dim3(2048), dim3(256), 0, s, adj_dev, N * R, N, bad);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipMemcpyAsync(&h, bad, sizeof(int), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        (void)hipFree(bad);
        if (e != hipSuccess) {
            set_error("adjacency validation failed: %s", hipGetErrorString(e));
            return ANN_EDEVICE;
        }
        if (h) {
            set_error("adjacency holds an id >= N");
            return ANN_EINVAL;
        }
    }
    ann_graph *g = new (std::nothrow) ann_graph;
    if (!g) {
        set_error("out of host memory");
        return ANN_ENOMEM;
    }
    g->adj = adj_dev;
    g->emb = emb_dev;
    g->N = N;
    g->R = R;
    g->d = d;
    g->dtype = dtype;
    *out = g;
    return ANN_OK;
}

void ann_graph_free(ann_graph *g) {
    if (g && g->adj_rank) (void)hipFree(g->adj_rank);
    delete g;
}

// rank must be a permutation of 0 .. N-1: every value in range, none twice (seen: one bit per value)
__global__ void check_rank_kernel(const int32_t *rank, int64_t N, uint32_t *seen, int *bad) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    int found = 0;
    for (; i < N; i += step) {
        const int32_t r = rank[i];
        if (r < 0 || (int64_t)r >= N) found |= 1;
        else if (atomicOr(&seen[(uint32_t)r >> 5], 1u << (r & 31)) & (1u << (r & 31))) found |= 2;
    }
    if (found) atomicOr(bad, found);
}

// adj_rank[e] = rank[adj[e]] (-1 where the adjacency holds no valid id)
__global__ void fill_adj_rank_kernel(const int32_t *adj, const int32_t *rank, int64_t n, int64_t N, int32_t *adj_rank) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += step) {
        const int32_t v = adj[i];
        adj_rank[i] = (v >= 0 && (int64_t)v < N) ? rank[v] : -1;
    }
}

int ann_search_visited_set_is_bitmap(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t E, int32_t W_max,
                                     int32_t L_max, int32_t k, int32_t max_iters_max) {
    Plan p;
    if (!make_plan(g, m, Q, E, W_max, L_max, k, max_iters_max, &p)) return ANN_EINVAL;
    return p.bitmap_words > 0 ? 1 : 0;
}

int ann_graph_set_locality(ann_graph *g, const int32_t *rank_dev, void *stream) {
    if (!g) {
        set_error("null graph handle");
        return ANN_EINVAL;
    }
    if (g->adj_rank) (void)hipFree(g->adj_rank);
    g->adj_rank = nullptr;
    g->rank = nullptr;
    if (!rank_dev) return ANN_OK;  // back to bits by id
    hipStream_t s = (hipStream_t)stream;
    const size_t seen_bytes = (size_t)((g->N + 31) / 32) * 4;
    char *tmp = nullptr;
    if (hipMalloc((void **)&tmp, 256 + seen_bytes) != hipSuccess) {
        set_error("device allocation of %zu bytes failed", 256 + seen_bytes);
        return ANN_ENOMEM;
    }
    int32_t *table = nullptr;
    const size_t table_bytes = (size_t)g->N * g->R * sizeof(int32_t);
    if (hipMalloc((void **)&table, table_bytes) != hipSuccess) {
        (void)hipFree(tmp);
        set_error("device allocation of %zu bytes failed", table_bytes);
        return ANN_ENOMEM;
    }
    int h = 0;
    hipError_t e = hipMemsetAsync(tmp, 0, 256 + seen_bytes, s);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(check_rank_kernel, dim3(2048), dim3(256), 0, s, rank_dev, g->N, (uint32_t *)(tmp + 256), (int *)tmp);
        hipLaunchKernelGGL(fill_adj_rank_kernel, dim3(4096), dim3(256), 0, s, g->adj, rank_dev, g->N * g->R, g->N, table);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(&h, tmp, sizeof(int), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(tmp);
    if (e != hipSuccess || h) {
        (void)hipFree(table);
        if (e != hipSuccess) {
            set_error("building the locality table failed: %s", hipGetErrorString(e));
            return ANN_EDEVICE;
        }
        set_error("rank_dev is not a permutation of 0 .. N-1 (%s)", (h & 1) ? "a value is out of range" : "a value occurs twice");
        return ANN_EINVAL;
    }
    g->rank = rank_dev;
    g->adj_rank = table;
    return ANN_OK;
}

int ann_mlp_load(int32_t n_layers, const int32_t *dims_host, const void *const *W_host, const float *const *b_host,
                 const float *head_w_host, int32_t d_user, int32_t dtype, uint32_t flags, void *stream,
                 ann_mlp **out) {
    if (!out) {
        set_error("out is null");
        return ANN_EINVAL;
    }
    *out = nullptr;
    if (!dims_host || !W_host || !b_host || !head_w_host) {
        set_error("dims_host, W_host, b_host and head_w_host must not be null");
        return ANN_EINVAL;
    }
    if (n_layers < 1 || n_layers > MAX_LAYERS) {
        set_error("need 1 <= n_layers <= %d", MAX_LAYERS);
        return ANN_EINVAL;
    }
    if (dtype != ANN_F32 && dtype != ANN_BF16 && dtype != ANN_F8 && dtype != ANN_F16) {
        set_error("dtype must be ANN_F32, ANN_BF16, ANN_F16 or ANN_F8");
        return ANN_EINVAL;
    }
    if (dtype == ANN_F8 && !f8_supported(dims_host, n_layers, d_user)) {
        set_error("the 8-bit metric is built for 64-wide items with hidden widths 256, 128 and 128-wide items with 512, 256");
        return ANN_ENOTIMPL;
    }
    for (int l = 0; l <= n_layers; ++l)
        if (dims_host[l] < 1 || dims_host[l] > MAX_WIDTH) {
            set_error("layer width %d out of [1, %d]", dims_host[l], MAX_WIDTH);
            return ANN_EINVAL;
        }
    const int J = dims_host[n_layers];
    if (J > MAX_HEADS) {
        set_error("at most %d heads", MAX_HEADS);
        return ANN_EINVAL;
    }
    if (d_user < 1 || d_user >= dims_host[0]) {
        set_error("need 1 <= d_user < dims[0]");
        return ANN_EINVAL;
    }
    for (int l = 0; l < n_layers; ++l)
        if (!W_host[l] || !b_host[l]) {
            set_error("layer %d has a null weight or bias array", l);
            return ANN_EINVAL;
        }
    hipStream_t s = (hipStream_t)stream;
    ann_mlp *m = new (std::nothrow) ann_mlp;
    if (!m) {
        set_error("out of host memory");
        return ANN_ENOMEM;
    }
    memset(m, 0, sizeof(*m));
    m->n_layers = n_layers;
    for (int l = 0; l <= n_layers; ++l) m->dims[l] = dims_host[l];
    m->d_user = d_user;
    m->d_item = dims_host[0] - d_user;
    m->dtype = dtype;
    m->J = J;
    for (int j = 0; j < J; ++j) m->head_w[j] = head_w_host[j];
    if (hipGetDevice(&m->device) != hipSuccess) m->device = 0;
    const size_t es = dtype == ANN_F32 ? 4 : 2;  // the 8-bit metric takes bf16 weights and quantises them itself
    int64_t wtot = 0;
    int32_t btot = 0;
    for (int l = 0; l < n_layers; ++l) {
        m->w_off[l] = wtot;
        m->b_off[l] = btot;
        wtot += (int64_t)dims_host[l] * dims_host[l + 1];
        wtot = (wtot + 63) & ~63ll;  // keep every layer 128-byte aligned
        btot += (dims_host[l + 1] + 63) & ~63;
    }
    std::vector<unsigned char> wbuf((size_t)wtot * es, 0);
    std::vector<float> bbuf((size_t)btot, 0.f);
    for (int l = 0; l < n_layers; ++l) {
        memcpy(wbuf.data() + (size_t)m->w_off[l] * es, W_host[l], (size_t)dims_host[l] * dims_host[l + 1] * es);
        memcpy(bbuf.data() + m->b_off[l], b_host[l], (size_t)dims_host[l + 1] * sizeof(float));
    }
    if (dtype == ANN_F8)  // the 8-bit kernel holds the second hidden layer at 16 x its value (see mlp_mfma_f8.hip)
        for (int i = 0; i < dims_host[2]; ++i) bbuf[(size_t)m->b_off[1] + i] *= 16.f;
    int rc = ANN_OK;
    auto fail = [&](int code) {
        ann_mlp_free(m);
        return code;
    };
    if (hipMalloc(&m->W_dev, wbuf.size()) != hipSuccess || hipMalloc((void **)&m->b_dev, bbuf.size() * 4) != hipSuccess ||
        hipMalloc((void **)&m->head_w_dev, MAX_HEADS * 4) != hipSuccess) {
        set_error("device allocation for the metric failed");
        return fail(ANN_ENOMEM);
    }
    if (hipMemcpyAsync(m->W_dev, wbuf.data(), wbuf.size(), hipMemcpyHostToDevice, s) != hipSuccess ||
        hipMemcpyAsync(m->b_dev, bbuf.data(), bbuf.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
        hipMemcpyAsync(m->head_w_dev, m->head_w, MAX_HEADS * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) {
        set_error("copy of the metric to the device failed");
        return fail(ANN_EDEVICE);
    }
    m->kernel = MLP_ALU;
    if (dtype == ANN_F8) {
        rc = build_f8_fragments(m, W_host, s);
        if (rc != ANN_OK) return fail(rc);
        m->kernel = MLP_MFMA2;
    } else if (!(flags & ANN_MLP_GENERIC) && mfma_supported(m->dims, n_layers, d_user, dtype)) {
        rc = build_mfma_fragments(m, W_host, s);
        if (rc != ANN_OK) return fail(rc);
        m->kernel = MLP_MFMA2;
    }
    *out = m;
    return ANN_OK;
}

void ann_mlp_free(ann_mlp *m) {
    if (!m) return;
    if (m->W_dev) (void)hipFree(m->W_dev);
    if (m->b_dev) (void)hipFree(m->b_dev);
    if (m->head_w_dev) (void)hipFree(m->head_w_dev);
    if (m->frag_dev) (void)hipFree(m->frag_dev);
    delete m;
}

int ann_mlp_uses_mfma(const ann_mlp *m) { return m && m->kernel != MLP_ALU; }

size_t ann_search_workspace_bytes(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t E, int32_t W_max,
                                  int32_t L_max, int32_t k, int32_t max_iters_max) {
    Plan p;
    if (!make_plan(g, m, Q, E, W_max, L_max, k, max_iters_max, &p)) return 0;
    return p.total;
}

static int search_common(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q,
                         const int32_t *entry_dev, int32_t E, const int32_t *W_q, const int32_t *L_q,
                         const int32_t *cap_q, int32_t W, int32_t L, int32_t k, int32_t max_iters, void *workspace_dev,
                         size_t workspace_bytes, int32_t *out_ids_dev, float *out_scores_dev, void *stream) {
    SearchArgs a;
    if (!make_plan(g, m, Q, E, W, L, k, max_iters, &a.plan)) return ANN_EINVAL;
    if (Q > 0 && (!queries_dev || !entry_dev || !out_ids_dev || !out_scores_dev)) {
        set_error("queries_dev, entry_dev, out_ids_dev and out_scores_dev must not be null");
        return ANN_EINVAL;
    }
    if (Q > 0 && (!workspace_dev || ((uintptr_t)workspace_dev & 255))) {
        set_error("workspace_dev must be a 256-byte aligned device pointer");
        return ANN_EINVAL;
    }
    if (workspace_bytes < a.plan.total) {
        set_error("workspace holds %zu bytes, %zu needed", workspace_bytes, a.plan.total);
        return ANN_EWORKSPACE;
    }
    a.g = g;
    a.m = m;
    a.queries = queries_dev;
    a.entries = entry_dev;
    a.W_q = W_q;
    a.L_q = L_q;
    a.cap_q = cap_q;
    a.W = W;
    a.L = L;
    a.cap = max_iters;
    a.ws = (char *)workspace_dev;
    a.out_ids = out_ids_dev;
    a.out_scores = out_scores_dev;
    a.stream = (hipStream_t)stream;
    return run_search(a);
}

int ann_search(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q, const int32_t *entry_dev,
               int32_t E, int32_t W, int32_t L, int32_t k, int32_t max_iters, void *workspace_dev,
               size_t workspace_bytes, int32_t *out_ids_dev, float *out_scores_dev, void *stream) {
    return search_common(g, m, queries_dev, Q, entry_dev, E, nullptr, nullptr, nullptr, W, L, k, max_iters,
                         workspace_dev, workspace_bytes, out_ids_dev, out_scores_dev, stream);
}

int ann_search_ragged(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q,
                      const int32_t *entry_dev, int32_t E, const int32_t *W_q_dev, const int32_t *L_q_dev,
                      const int32_t *iters_q_dev, int32_t W_max, int32_t L_max, int32_t k, int32_t max_iters_max,
                      void *workspace_dev, size_t workspace_bytes, int32_t *out_ids_dev, float *out_scores_dev,
                      void *stream) {
    if (Q > 0 && (!W_q_dev || !L_q_dev || !iters_q_dev)) {
        set_error("W_q_dev, L_q_dev and iters_q_dev must not be null");
        return ANN_EINVAL;
    }
    return search_common(g, m, queries_dev, Q, entry_dev, E, W_q_dev, L_q_dev, iters_q_dev, W_max, L_max, k,
                         max_iters_max, workspace_dev, workspace_bytes, out_ids_dev, out_scores_dev, stream);
}

// Workspace of a layered search: the largest per-layer workspace first (so that the counters sit
// where ann_search_stats looks for them), then two id buffers and one score buffer that carry
// a layer's results to the next.
struct LayerPlan {
    size_t search_bytes, carry_off, carry_ids_bytes, total;
    int32_t k_carry_max;
};

static bool make_layer_plan(const ann_graph *const *graphs, int32_t n_layers, const ann_mlp *m, int32_t Q, int32_t E,
                            const int32_t *W_l, const int32_t *L_l, const int32_t *K_l, int32_t max_iters,
                            LayerPlan *lp) {
    if (!graphs || n_layers < 1 || n_layers > 16 || !W_l || !L_l || !K_l) {
        set_error("graphs, W_l, L_l, K_l must not be null and 1 <= n_layers <= 16");
        return false;
    }
    lp->search_bytes = 0;
    lp->k_carry_max = 1;
    for (int l = 0; l < n_layers; ++l) {
        const ann_graph *g = graphs[l];
        if (!g) {
            set_error("graphs[%d] is null", l);
            return false;
        }
        const ann_graph *base = graphs[n_layers - 1];
        if (g->emb != base->emb || g->d != base->d || g->dtype != base->dtype) {
            set_error("layer %d does not share the embedding table of the base layer", l);
            return false;
        }
        if (l > 0 && g->N < graphs[l - 1]->N) {
            set_error("layer %d holds fewer items than layer %d: layers must be nested, coarsest first", l, l - 1);
            return false;
        }
        Plan p;
        const int32_t seeds = l == 0 ? E : K_l[l - 1];
        if (!make_plan(g, m, Q, seeds, W_l[l], L_l[l], K_l[l], max_iters, &p)) return false;
        if (p.total > lp->search_bytes) lp->search_bytes = p.total;
        if (l + 1 < n_layers && K_l[l] > lp->k_carry_max) lp->k_carry_max = K_l[l];
    }
    lp->carry_off = align256(lp->search_bytes);
    lp->carry_ids_bytes = align256((size_t)(Q > 0 ? Q : 1) * lp->k_carry_max * 4);
    lp->total = lp->carry_off + 3 * lp->carry_ids_bytes;
    return true;
}

size_t ann_search_layers_workspace_bytes(const ann_graph *const *graphs, int32_t n_layers, const ann_mlp *m,
                                         int32_t Q, int32_t E, const int32_t *W_l, const int32_t *L_l,
                                         const int32_t *K_l, int32_t max_iters) {
    LayerPlan lp;
    if (!make_layer_plan(graphs, n_layers, m, Q, E, W_l, L_l, K_l, max_iters, &lp)) return 0;
    return lp.total;
}

int ann_search_layers(const ann_graph *const *graphs, int32_t n_layers, const ann_mlp *m, const void *queries_dev,
                      int32_t Q, const int32_t *entry_dev, int32_t E, const int32_t *W_l, const int32_t *L_l,
                      const int32_t *K_l, int32_t max_iters, void *workspace_dev, size_t workspace_bytes,
                      int32_t *out_ids_dev, float *out_scores_dev, void *stream) {
    LayerPlan lp;
    if (!make_layer_plan(graphs, n_layers, m, Q, E, W_l, L_l, K_l, max_iters, &lp)) return ANN_EINVAL;
    if (Q > 0 && (!queries_dev || !entry_dev || !out_ids_dev || !out_scores_dev)) {
        set_error("queries_dev, entry_dev, out_ids_dev and out_scores_dev must not be null");
        return ANN_EINVAL;
    }
    if (Q > 0 && (!workspace_dev || ((uintptr_t)workspace_dev & 255))) {
        set_error("workspace_dev must be a 256-byte aligned device pointer");
        return ANN_EINVAL;
    }
    if (workspace_bytes < lp.total) {
        set_error("workspace holds %zu bytes, %zu needed", workspace_bytes, lp.total);
        return ANN_EWORKSPACE;
    }
    char *ws = (char *)workspace_dev;
    int32_t *carry[2] = {(int32_t *)(ws + lp.carry_off), (int32_t *)(ws + lp.carry_off + lp.carry_ids_bytes)};
    float *carry_scores = (float *)(ws + lp.carry_off + 2 * lp.carry_ids_bytes);
    int worst = ANN_OK;
    for (int l = 0; l < n_layers; ++l) {
        const bool last = l + 1 == n_layers;
        SearchArgs a;
        const int32_t seeds = l == 0 ? E : K_l[l - 1];
        if (!make_plan(graphs[l], m, Q, seeds, W_l[l], L_l[l], K_l[l], max_iters, &a.plan)) return ANN_EINVAL;
        a.g = graphs[l];
        a.m = m;
        a.queries = queries_dev;
        a.entries = l == 0 ? entry_dev : carry[(l - 1) & 1];
        a.W_q = a.L_q = a.cap_q = nullptr;
        a.W = W_l[l];
        a.L = L_l[l];
        a.cap = max_iters;
        a.ws = ws;
        a.out_ids = last ? out_ids_dev : carry[l & 1];
        a.out_scores = last ? out_scores_dev : carry_scores;
        a.stream = (hipStream_t)stream;
        a.keep_stats = l > 0;
        int rc = run_search(a);
        if (rc == ANN_EWORKSPACE)
            worst = rc;  // a visited table filled up in this layer: the search goes on with what it found
        else if (rc != ANN_OK)
            return rc;
    }
    return worst;
}

size_t ann_search_walkers_workspace_bytes(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t E, int32_t T,
                                          int32_t k) {
    Plan p;
    if (T < 1) {
        set_error("need T >= 1 hops (got %d)", T);
        return 0;
    }
    if (!make_plan(g, m, Q, E, E, 1, k, T, &p)) return 0;
    return p.total;
}

int ann_search_walkers(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q,
                       const int32_t *entry_dev, int32_t E, int32_t T, int32_t k, void *workspace_dev,
                       size_t workspace_bytes, int32_t *out_ids_dev, float *out_scores_dev, void *stream) {
    SearchArgs a;
    if (T < 1) {
        set_error("need T >= 1 hops (got %d)", T);
        return ANN_EINVAL;
    }
    // one walker per seed: expansion width E, list capacity k, T rounds
    if (!make_plan(g, m, Q, E, E, 1, k, T, &a.plan)) return ANN_EINVAL;
    if (Q > 0 && (!queries_dev || !entry_dev || !out_ids_dev || !out_scores_dev)) {
        set_error("queries_dev, entry_dev, out_ids_dev and out_scores_dev must not be null");
        return ANN_EINVAL;
    }
    if (Q > 0 && (!workspace_dev || ((uintptr_t)workspace_dev & 255))) {
        set_error("workspace_dev must be a 256-byte aligned device pointer");
        return ANN_EINVAL;
    }
    if (workspace_bytes < a.plan.total) {
        set_error("workspace holds %zu bytes, %zu needed", workspace_bytes, a.plan.total);
        return ANN_EWORKSPACE;
    }
    a.g = g;
    a.m = m;
    a.queries = queries_dev;
    a.entries = entry_dev;
    a.W_q = a.L_q = a.cap_q = nullptr;
    a.W = E;
    a.L = 1;
    a.cap = T;
    a.ws = (char *)workspace_dev;
    a.out_ids = out_ids_dev;
    a.out_scores = out_scores_dev;
    a.stream = (hipStream_t)stream;
    a.walkers = true;
    return run_search(a);
}

// Workspace of a streamed search: the workspace of a search over `slots` queries, then the slot -> query
// map and the user terms of all queries.
struct StreamPlan {
    Plan plan;
    size_t off_slot_query, off_upre_all, total;
};

static bool make_stream_plan(const ann_graph *g, const ann_mlp *m, int32_t Q_total, int32_t slots, int32_t E, int32_t W,
                             int32_t L, int32_t k, int32_t max_iters, StreamPlan *sp) {
    if (Q_total < 0 || slots < 1) {
        set_error("need Q_total >= 0 and slots >= 1 (got %d, %d)", Q_total, slots);
        return false;
    }
    if (!make_plan(g, m, slots, E, W, L, k, max_iters, &sp->plan)) return false;
    size_t o = align256(sp->plan.total);
    sp->off_slot_query = o;
    o = align256(o + (size_t)slots * 4);
    sp->off_upre_all = o;
    o = align256(o + ((size_t)Q_total * sp->plan.H1 + 32) * 4);
    sp->total = o;
    return true;
}

size_t ann_search_stream_workspace_bytes(const ann_graph *g, const ann_mlp *m, int32_t Q_total, int32_t slots,
                                         int32_t E, int32_t W, int32_t L, int32_t k, int32_t max_iters) {
    StreamPlan sp;
    if (!make_stream_plan(g, m, Q_total, slots, E, W, L, k, max_iters, &sp)) return 0;
    return sp.total;
}

int ann_search_stream(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q_total,
                      const int32_t *entry_dev, int32_t E, int32_t slots, int32_t W, int32_t L, int32_t k,
                      int32_t max_iters, void *workspace_dev, size_t workspace_bytes, int32_t *out_ids_dev,
                      float *out_scores_dev, void *stream) {
    StreamPlan sp;
    if (!make_stream_plan(g, m, Q_total, slots, E, W, L, k, max_iters, &sp)) return ANN_EINVAL;
    if (Q_total > 0 && (!queries_dev || !entry_dev || !out_ids_dev || !out_scores_dev)) {
        set_error("queries_dev, entry_dev, out_ids_dev and out_scores_dev must not be null");
        return ANN_EINVAL;
    }
    if (Q_total > 0 && (!workspace_dev || ((uintptr_t)workspace_dev & 255))) {
        set_error("workspace_dev must be a 256-byte aligned device pointer");
        return ANN_EINVAL;
    }
    if (workspace_bytes < sp.total) {
        set_error("workspace holds %zu bytes, %zu needed", workspace_bytes, sp.total);
        return ANN_EWORKSPACE;
    }
    SearchArgs a;
    a.plan = sp.plan;
    a.g = g;
    a.m = m;
    a.queries = queries_dev;
    a.entries = entry_dev;
    a.W_q = a.L_q = a.cap_q = nullptr;
    a.W = W;
    a.L = L;
    a.cap = max_iters;
    a.ws = (char *)workspace_dev;
    a.out_ids = out_ids_dev;
    a.out_scores = out_scores_dev;
    a.stream = (hipStream_t)stream;
    a.Q_total = Q_total;
    a.slot_query = (int32_t *)(a.ws + sp.off_slot_query);
    a.upre_all = (float *)(a.ws + sp.off_upre_all);
    return run_stream(a);
}

}  // extern "C"

// An open stream (Sec. 3.2, Q-HiPANNS: the scorer keeps listening for requests that arrive at any time): the
// state of ann_search_stream kept between calls, with the number of arrived queries a device word that the
// admission kernel reads, so that queries submitted while others are being searched join the running batches.
struct ann_stream {
    gmpgr::SearchArgs a;
    gmpgr::Mailbox box;
    std::mutex mu;               // submit and the enqueuing of rounds may come from different host threads
    int32_t capacity = 0;        // rows of the caller's arrays
    int32_t submitted = 0;       // queries that have arrived
    int64_t rounds = 0;          // rounds enqueued so far
    int64_t submit_round = 0;    // rounds enqueued when the last submit was published
    size_t elem = 2;             // bytes of one user-vector element
};

namespace gmpgr {

// One round of an open stream: admission, packing, scoring, list update.  Caller holds s->mu.
static int stream_round(ann_stream *s) {
    SearchArgs &a = s->a;
    int rc;
    a.round_index = (int32_t)(s->rounds & 0x3fffffff);
    {
        StageTimer timer(ANN_STAGE_ROUND, a.stream);
        if ((rc = launch_admit(a)) != ANN_OK) return rc;
    }
    {
        StageTimer timer(ANN_STAGE_PACK, a.stream);
        if ((rc = launch_scan_compact(a)) != ANN_OK) return rc;  // its progress word counts the stream's rounds
    }
    if ((rc = score_batch(a)) != ANN_OK) return rc;
    {
        StageTimer timer(ANN_STAGE_ROUND, a.stream);
        if ((rc = launch_round(a)) != ANN_OK) return rc;
    }
    s->rounds += 1;
    return ANN_OK;
}

}  // namespace gmpgr

extern "C" {

int ann_stream_open(const ann_graph *g, const ann_mlp *m, int32_t capacity, int32_t slots, int32_t E, int32_t W,
                    int32_t L, int32_t k, int32_t max_iters, const void *queries_dev, const int32_t *entry_dev,
                    int32_t *out_ids_dev, float *out_scores_dev, void *workspace_dev, size_t workspace_bytes,
                    void *stream, ann_stream **out) {
    if (!out) {
        set_error("out is null");
        return ANN_EINVAL;
    }
    *out = nullptr;
    StreamPlan sp;
    if (capacity < 1) {
        set_error("need capacity >= 1 (got %d)", capacity);
        return ANN_EINVAL;
    }
    if (!make_stream_plan(g, m, capacity, slots, E, W, L, k, max_iters, &sp)) return ANN_EINVAL;
    if (!queries_dev || !entry_dev || !out_ids_dev || !out_scores_dev) {
        set_error("queries_dev, entry_dev, out_ids_dev and out_scores_dev must not be null");
        return ANN_EINVAL;
    }
    if (!workspace_dev || ((uintptr_t)workspace_dev & 255)) {
        set_error("workspace_dev must be a 256-byte aligned device pointer");
        return ANN_EINVAL;
    }
    if (workspace_bytes < sp.total) {
        set_error("workspace holds %zu bytes, %zu needed", workspace_bytes, sp.total);
        return ANN_EWORKSPACE;
    }
    ann_stream *s = new (std::nothrow) ann_stream;
    if (!s) {
        set_error("out of host memory");
        return ANN_ENOMEM;
    }
    if (!s->box.init()) {
        delete s;
        set_error("pinned host allocation failed");
        return ANN_ENOMEM;
    }
    SearchArgs &a = s->a;
    a.plan = sp.plan;
    a.g = g;
    a.m = m;
    a.queries = queries_dev;
    a.entries = entry_dev;
    a.W_q = a.L_q = a.cap_q = nullptr;
    a.W = W;
    a.L = L;
    a.cap = max_iters;
    a.ws = (char *)workspace_dev;
    a.out_ids = out_ids_dev;
    a.out_scores = out_scores_dev;
    a.stream = (hipStream_t)stream;
    a.Q_total = -1;
    a.Q_rows = capacity;
    a.slot_query = (int32_t *)(a.ws + sp.off_slot_query);
    a.upre_all = (float *)(a.ws + sp.off_upre_all);
    a.mailbox = s->box.dev;
    a.mail_tag = s->box.new_tag();
    s->capacity = capacity;
    s->elem = m->dtype == ANN_F32 ? 4 : 2;
    int rc = launch_stream_reset(a);
    if (rc != ANN_OK) {
        s->box.release();
        delete s;
        return rc;
    }
    *out = s;
    return ANN_OK;
}

int ann_stream_submit(ann_stream *s, int32_t n) {
    if (!s || n < 0) {
        set_error("null stream handle or n < 0");
        return ANN_EINVAL;
    }
    std::lock_guard<std::mutex> guard(s->mu);
    if ((int64_t)s->submitted + n > s->capacity) {
        set_error("%d queries have arrived and %d more would exceed the capacity of %d", s->submitted, n, s->capacity);
        return ANN_EINVAL;
    }
    if (n == 0) return ANN_OK;
    SearchArgs &a = s->a;
    const int32_t first = s->submitted;
    int rc;
    if (a.m->kernel == MLP_MFMA2) {  // the user terms of the new rows
        const char *rows = (const char *)a.queries + (size_t)first * a.m->d_user * s->elem;
        if ((rc = launch_user_pre(a.m, rows, n, a.upre_all + (size_t)first * a.plan.H1, a.stream)) != ANN_OK) return rc;
    }
    if ((rc = launch_stream_publish(a, first + n)) != ANN_OK) return rc;
    s->submitted = first + n;
    s->submit_round = s->rounds;
    return ANN_OK;
}

int ann_stream_step(ann_stream *s, int32_t rounds) {
    if (!s || rounds < 0) {
        set_error("null stream handle or rounds < 0");
        return ANN_EINVAL;
    }
    std::lock_guard<std::mutex> guard(s->mu);
    for (int32_t i = 0; i < rounds; ++i)
        if (int rc = stream_round(s); rc != ANN_OK) return rc;
    return ANN_OK;
}

int ann_stream_drain(ann_stream *s) {
    if (!s) {
        set_error("null stream handle");
        return ANN_EINVAL;
    }
    SearchArgs &a = s->a;
    const Plan &p = a.plan;
    // a query ends within this many rounds of its admission (it cannot score more ids than its visited set
    // holds); the loop is bounded even if no report ever said "finished"
    const int64_t per_query = p.max_iters_max > 0 ? (int64_t)p.max_iters_max + 2
                                                  : (p.bitmap_words > 0 ? a.g->N : (int64_t)p.hash_cap / 2) + 3;
    int64_t limit;
    {
        std::lock_guard<std::mutex> guard(s->mu);
        limit = s->rounds + per_query * (((int64_t)s->submitted + p.Q - 1) / p.Q + 1);
    }
    for (;;) {
        int64_t enq, need;
        {
            std::lock_guard<std::mutex> guard(s->mu);
            enq = s->rounds;
            need = s->submit_round;  // a "finished" report counts only from a round enqueued after the last submit
            if (s->submitted == 0) return ANN_OK;
        }
        int64_t seen = 0;
        const int g = s->box.gate(a.mail_tag, enq, a.stream, &seen);
        if (g < 0) {
            set_error(g == -3 ? "no progress report from the search's kernels within the time limit (ann_set_progress_timeout)"
                              : "the stream failed or ran dry without the search's progress report");
            return ANN_EDEVICE;
        }
        if (g > 0 && seen > need) break;
        // "finished" from before the last submit: the rounds enqueued since will report; stay a few ahead of them
        if (g > 0 && seen + Mailbox::AHEAD < enq) continue;
        if (enq >= limit) {
            set_error("the stream did not finish within %lld rounds", (long long)limit);
            return ANN_EDEVICE;
        }
        std::lock_guard<std::mutex> guard(s->mu);
        if (int rc = stream_round(s); rc != ANN_OK) return rc;
    }
    int64_t stats[8];
    ANN_HIP_TRY(hipMemcpyAsync(stats, a.ws + p.off_stats, sizeof(stats), hipMemcpyDeviceToHost, a.stream));
    ANN_HIP_TRY(hipStreamSynchronize(a.stream));
    if (stats[3] > 0) {
        set_error("%lld queries filled their visited table (sized for %d rounds) and stopped early", (long long)stats[3],
                  p.rounds_assumed);
        return ANN_EWORKSPACE;
    }
    return ANN_OK;
}

int ann_stream_close(ann_stream *s) {
    if (!s) return ANN_OK;
    (void)hipStreamSynchronize(s->a.stream);  // no kernel may store to the progress word after it is freed
    s->box.release();
    delete s;
    return ANN_OK;
}

int ann_users_add_noise(const void *users_dev, void *out_dev, int32_t Q, int32_t d, int32_t dtype, double sigma,
                        uint64_t seed, uint64_t draw, void *stream) {
    if (Q < 0 || d < 1 || (dtype != ANN_F32 && dtype != ANN_BF16 && dtype != ANN_F16) || !(sigma >= 0.0) ||
        !(sigma < INFINITY)) {
        set_error("need Q >= 0, d >= 1, dtype ANN_F32, ANN_BF16 or ANN_F16, finite sigma >= 0");
        return ANN_EINVAL;
    }
    if (Q == 0) return ANN_OK;
    if (!users_dev || !out_dev) {
        set_error("users_dev and out_dev must not be null");
        return ANN_EINVAL;
    }
    return launch_users_add_noise(users_dev, out_dev, (int64_t)Q * d, dtype, sigma, seed, draw, (hipStream_t)stream);
}

int ann_quantize_e4m3(const void *src_dev, int32_t src_dtype, int64_t n, float scale, uint8_t *dst_dev,
                      void *stream) {
    if (n < 0 || (src_dtype != ANN_F32 && src_dtype != ANN_BF16) || !(scale > 0.f) || !(scale < INFINITY)) {
        set_error("need n >= 0, a source of ANN_F32 or ANN_BF16, a finite scale > 0");
        return ANN_EINVAL;
    }
    if (n == 0) return ANN_OK;
    if (!src_dev || !dst_dev) {
        set_error("src_dev and dst_dev must not be null");
        return ANN_EINVAL;
    }
    return launch_quantize_e4m3(src_dev, src_dtype, n, scale, dst_dev, (hipStream_t)stream);
}

int ann_score_pairs(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q, int64_t M,
                    const int32_t *q_idx_dev, const int32_t *item_dev, float *out_dev, int32_t tile_rows,
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
    if (M < 0 || M > 0x7fffffffll || Q < 1 || tile_rows < 0) {
        set_error("need 0 <= M < 2^31, Q >= 1, tile_rows >= 0");
        return ANN_EINVAL;
    }
    if (M == 0) return ANN_OK;
    if (!queries_dev || !q_idx_dev || !item_dev || !out_dev) {
        set_error("queries_dev, q_idx_dev, item_dev and out_dev must not be null");
        return ANN_EINVAL;
    }
    hipStream_t s = (hipStream_t)stream;
    if (m->kernel != MLP_MFMA2)
        return launch_mlp_alu(g, m, queries_dev, q_idx_dev, item_dev, nullptr, M, Q, out_dev, tile_rows, s);
    char *tmp = nullptr;
    size_t upre_bytes = ((size_t)Q * m->dims[1] + 32) * sizeof(float);
    if (hipMalloc((void **)&tmp, 256 + upre_bytes) != hipSuccess) {
        set_error("device allocation of %zu bytes failed", 256 + upre_bytes);
        return ANN_ENOMEM;
    }
    int32_t M32 = (int32_t)M;
    int rc = ANN_OK;
    hipError_t e = hipMemcpyAsync(tmp, &M32, 4, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) {
        set_error("hipMemcpyAsync failed: %s", hipGetErrorString(e));
        rc = ANN_EDEVICE;
    }
    if (rc == ANN_OK) rc = launch_user_pre(m, queries_dev, Q, (float *)(tmp + 256), s);
    if (rc == ANN_OK)
        rc = launch_mlp_mfma(g, m, (const float *)(tmp + 256), q_idx_dev, item_dev, (const int32_t *)tmp, M, Q,
                             out_dev, tile_rows, s);
    e = hipStreamSynchronize(s);
    if (rc == ANN_OK && e != hipSuccess) {
        set_error("hipStreamSynchronize failed: %s", hipGetErrorString(e));
        rc = ANN_EDEVICE;
    }
    (void)hipFree(tmp);
    return rc;
}

int ann_set_progress_timeout(double seconds) {
    if (!(seconds >= 0.0)) {
        set_error("the time limit must be >= 0 seconds (0 = none)");
        return ANN_EINVAL;
    }
    g_wait_limit_s.store(seconds, std::memory_order_relaxed);
    return ANN_OK;
}

int ann_profile_enable(int on) {
    g_prof.on = on != 0;
    g_prof.used = 0;
    return ANN_OK;
}

int ann_profile_read(double *ms_out, int64_t *launches_out) {
    if (!ms_out || !launches_out) {
        set_error("ms_out and launches_out must not be null");
        return ANN_EINVAL;
    }
    for (int i = 0; i < ANN_STAGE_COUNT; ++i) {
        ms_out[i] = 0.0;
        launches_out[i] = 0;
    }
    for (size_t i = 0; i < g_prof.used; ++i) {
        ANN_HIP_TRY(hipEventSynchronize(g_prof.events[2 * i + 1]));
        float ms = 0.f;
        ANN_HIP_TRY(hipEventElapsedTime(&ms, g_prof.events[2 * i], g_prof.events[2 * i + 1]));
        ms_out[g_prof.stage[i]] += ms;
        launches_out[g_prof.stage[i]] += 1;
    }
    g_prof.used = 0;
    return ANN_OK;
}

__global__ void profile_copy_kernel(uint4 *dst, const uint4 *src, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += step) dst[i] = src[i];
}

int ann_profile_copy(void *dst_dev, const void *src_dev, size_t bytes, void *stream) {
    if (!dst_dev || !src_dev || (bytes & 15) || ((uintptr_t)dst_dev & 15) || ((uintptr_t)src_dev & 15)) {
        set_error("dst_dev, src_dev must be non-null and 16-byte aligned, bytes a multiple of 16");
        return ANN_EINVAL;
    }
    if (bytes == 0) return ANN_OK;
    hipLaunchKernelGGL(profile_copy_kernel, dim3(4096), dim3(256), 0, (hipStream_t)stream, (uint4 *)dst_dev,
                       (const uint4 *)src_dev, bytes / 16);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

int ann_search_stats(const void *workspace_dev, ann_stats *out_host, void *stream) {
    if (!workspace_dev || !out_host) {
        set_error("workspace_dev and out_host must not be null");
        return ANN_EINVAL;
    }
    int64_t st[8];
    hipStream_t s = (hipStream_t)stream;
    ANN_HIP_TRY(hipMemcpyAsync(st, (const char *)workspace_dev + STATS_OFFSET, sizeof(st), hipMemcpyDeviceToHost, s));
    ANN_HIP_TRY(hipStreamSynchronize(s));
    out_host->pairs_scored = st[0];
    out_host->nodes_expanded = st[1];
    out_host->max_query_iters = st[2];
    out_host->visited_overflow = st[3];
    out_host->queries = st[4];
    out_host->adjacency_bytes = st[1] * st[5];
    out_host->embedding_bytes = st[0] * st[6];
    out_host->pair_list_bytes = st[0] * 12;
    return ANN_OK;
}

}  // extern "C"
