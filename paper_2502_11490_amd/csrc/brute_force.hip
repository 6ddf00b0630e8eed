// ann_brute_force: the exhaustive search, i.e. the best k items of the whole table under the metric the graph
// search approximates (the ground truth of the recall measure, Sec. 5.1.3; relevance of Eq. 5-8).
//
// The table is walked in chunks of items, a block of queries at a time: a fill kernel writes the dense
// (query, item) pair list of "every query of the block x every item of the chunk", the metric's own scoring
// kernel scores it (the same launchers the search uses, so an item's relevance here is bit for bit the one a
// search sees), and one workgroup per query folds the chunk's scores into that query's running best-k list.
// Order: relevance descending, ties by ascending id, i.e. ascending order-preserving keys, as in the search.
//
// ann_rerank is the same fold over a caller's candidate lists instead of the whole table: the lists of a search
// under a cheaper metric (the 8-bit one) are scored again under this metric and its best k returned.
#include "common.h"
#include "keys.h"

namespace gmpgr {

constexpr int BF_BLOCK = 256;
constexpr int BF_PIECE = BF_BLOCK * 4;  // scores looked at between two looks at the buffer's fill
constexpr int BF_CAND = 2048;           // keys better than the current k-th, waiting to be merged
constexpr int BF_KMAX = 2048;           // largest k
constexpr int64_t BF_PAIRS = (int64_t)1 << 24;  // pairs scored per pass
constexpr int BF_CHUNK = 1 << 16;       // items per pass and query

__global__ void __launch_bounds__(256)
bf_fill_pairs_kernel(int32_t *pair_q, int32_t *pair_id, int q0, int32_t i0, int nc, int total, int32_t *count) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *count = total;
    for (int p = blockIdx.x * blockDim.x + threadIdx.x; p < total; p += gridDim.x * blockDim.x) {
        const int q = p / nc;
        pair_q[p] = q0 + q;
        if (pair_id) pair_id[p] = i0 + (p - q * nc);
    }
}

__global__ void __launch_bounds__(256) bf_clear_kernel(uint64_t *best, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        best[i] = KEY_SENTINEL;
}

// Folds scores[b * nc .. (b + 1) * nc) of query q0 + b into best[(q0 + b) * k .. + k): ascending keys,
// KEY_SENTINEL = no entry yet.  The scores belong to items i0 .. i0 + nc (ids == nullptr) or to the ids
// ids[b * nc ..] (entries outside [0, N) are no candidates).  Keys that cannot enter (not below the current
// k-th) are dropped as they are read; the others wait in an LDS buffer that is sorted and merged by rank whenever
// the next piece might not fit.  A waiting key goes behind the list's keys that equal it (a candidate id given
// twice), so the merge's destinations are a permutation whether or not the keys are distinct.
__global__ void __launch_bounds__(BF_BLOCK)
bf_topk_kernel(const float *__restrict__ scores, int nc, int32_t i0, const int32_t *__restrict__ ids, int64_t N,
               uint64_t *best_g, int k, int q0) {
    __shared__ uint64_t best[2][BF_KMAX];
    __shared__ uint64_t cand[BF_CAND];
    __shared__ int n_cand;
    __shared__ uint64_t worst;  // the k-th key, KEY_SENTINEL while fewer than k entries are held
    const float *row = scores + (size_t)blockIdx.x * nc;
    const int32_t *row_ids = ids ? ids + (size_t)blockIdx.x * nc : nullptr;
    uint64_t *mine = best_g + (size_t)(q0 + blockIdx.x) * k;
    for (int i = threadIdx.x; i < k; i += BF_BLOCK) best[0][i] = mine[i];
    if (threadIdx.x == 0) n_cand = 0;
    __syncthreads();
    if (threadIdx.x == 0) worst = best[0][k - 1];
    int cur = 0;
    int n_best = lower_bound_keys(best[0], k, KEY_SENTINEL);

    // n: the buffer's fill, read by every thread between two barriers.  Every thread calls.
    auto fold = [&](const int n) {
        if (n == 0) return;
        int n_pad = 1;
        while (n_pad < n) n_pad <<= 1;
        for (int i = n + threadIdx.x; i < n_pad; i += BF_BLOCK) cand[i] = KEY_SENTINEL;
        __syncthreads();
        bitonic_sort<BF_BLOCK>(cand, n_pad);
        const uint64_t *from = best[cur];
        uint64_t *to = best[cur ^ 1];
        for (int i = threadIdx.x; i < n_best; i += BF_BLOCK) {
            const uint64_t key = from[i];
            const int pos = i + lower_bound_keys(cand, n, key);
            if (pos < k) to[pos] = key;
        }
        for (int j = threadIdx.x; j < n; j += BF_BLOCK) {  // behind equal keys of the list (a repeated candidate)
            const uint64_t key = cand[j];
            const int pos = j + lower_bound_keys(from, n_best, key + 1);
            if (pos < k) to[pos] = key;
        }
        n_best = min(k, n_best + n);
        for (int i = n_best + threadIdx.x; i < k; i += BF_BLOCK) to[i] = KEY_SENTINEL;
        cur ^= 1;
        __syncthreads();
        if (threadIdx.x == 0) {
            n_cand = 0;
            worst = to[k - 1];
        }
        __syncthreads();
    };

    for (int base = 0; base < nc; base += BF_PIECE) {
        __syncthreads();
        const int held = n_cand;
        __syncthreads();  // nobody appends before everybody has read the fill
        if (held + BF_PIECE > BF_CAND) fold(held);
        const uint64_t bar = worst;
        float s[4];
        int32_t id[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int idx = base + r * BF_BLOCK + threadIdx.x;
            s[r] = idx < nc ? row[idx] : 0.0f;
            id[r] = idx >= nc ? -1 : row_ids ? row_ids[idx] : i0 + idx;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (id[r] >= 0 && (int64_t)id[r] < N) {
                const uint64_t key = make_key(s[r], id[r], 0);
                if (key < bar) cand[atomicAdd(&n_cand, 1)] = key;
            }
        }
    }
    __syncthreads();
    fold(n_cand);
    for (int i = threadIdx.x; i < k; i += BF_BLOCK) mine[i] = best[cur][i];
}

__global__ void __launch_bounds__(256)
bf_emit_kernel(const uint64_t *best, int64_t n, int32_t *out_ids, float *out_scores) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const uint64_t key = best[i];
        const bool none = key == KEY_SENTINEL;
        out_ids[i] = none ? -1 : key_id(key);
        out_scores[i] = none ? -INFINITY : key_score(key);
    }
}

static int grid_for(int64_t n) {
    int64_t blocks = (n + 255) / 256;
    return (int)(blocks < 1 ? 1 : blocks > 8192 ? 8192 : blocks);
}

}  // namespace gmpgr

using namespace gmpgr;

// Temporary of one call: count word, per-query user terms, one pass's pair list and scores, the running lists.
struct BestKPlan {
    int nc_max, Qb;
    size_t off_upre, off_pq, off_pi, off_sc, off_best, total;
};

static bool best_k_plan(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t k, bool cand, int32_t n,
                        BestKPlan *p) {
    if (!g || !m) {
        set_error("null graph or metric handle");
        return false;
    }
    if (m->d_item != g->d || m->dtype != g->dtype) {
        set_error("metric (item width %d, dtype %d) does not match graph (%d, %d)", m->d_item, m->dtype, g->d,
                  g->dtype);
        return false;
    }
    if (Q < 1 || k < 1 || k > BF_KMAX) {
        set_error("need Q >= 1 and 1 <= k <= %d", BF_KMAX);
        return false;
    }
    if (cand && (n < 1 || n > BF_CHUNK)) {
        set_error("need 1 <= n <= %d candidates per query", BF_CHUNK);
        return false;
    }
    if (g->N < 1 || g->N > 0x7fffffffll) {
        set_error("the item table has %lld rows", (long long)g->N);
        return false;
    }
    // items (or candidates) per pass and query, queries per pass
    p->nc_max = cand ? n : (int)(g->N < BF_CHUNK ? g->N : BF_CHUNK);
    const int64_t qb64 = BF_PAIRS / p->nc_max;
    p->Qb = (int)(qb64 > Q ? Q : qb64 < 1 ? 1 : qb64);
    const size_t pairs = (size_t)p->Qb * p->nc_max;
    const size_t upre_bytes = m->kernel == MLP_MFMA2 ? ((size_t)Q * m->dims[1] + 32) * sizeof(float) : 0;
    auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
    p->off_upre = 256;
    p->off_pq = up(p->off_upre + upre_bytes);
    p->off_pi = up(p->off_pq + pairs * 4);
    p->off_sc = up(p->off_pi + (cand ? 0 : pairs * 4));
    p->off_best = up(p->off_sc + pairs * 4);
    p->total = up(p->off_best + (size_t)Q * k * 8);
    return true;
}

// Best k per query over the whole table (cand == nullptr) or over cand[q][0..n) (device, [Q][n]).
// ws == nullptr: the temporary is allocated and freed here and the stream is synchronised; otherwise the call
// only enqueues.
static int best_k(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q, int32_t k,
                  const int32_t *cand, int32_t n, int32_t *out_ids_dev, float *out_scores_dev, void *ws,
                  size_t ws_bytes, void *stream) {
    BestKPlan p;
    if (!best_k_plan(g, m, Q, k, cand != nullptr, n, &p)) return ANN_EINVAL;
    if (!queries_dev || !out_ids_dev || !out_scores_dev) {
        set_error("queries_dev, out_ids_dev and out_scores_dev must not be null");
        return ANN_EINVAL;
    }
    if (ws && ws_bytes < p.total) {
        set_error("workspace of %zu bytes given, %zu needed", ws_bytes, p.total);
        return ANN_EWORKSPACE;
    }
    if (ws && ((uintptr_t)ws & 255)) {
        set_error("the workspace must be 256-byte aligned");
        return ANN_EINVAL;
    }
    hipStream_t s = (hipStream_t)stream;
    const bool mfma = m->kernel == MLP_MFMA2;
    const int nc_max = p.nc_max, Qb = p.Qb;
    const int64_t total_per_query = cand ? n : g->N;
    char *tmp = (char *)ws;
    if (!tmp && hipMalloc((void **)&tmp, p.total) != hipSuccess) {
        set_error("device allocation of %zu bytes failed", p.total);
        return ANN_ENOMEM;
    }
    int32_t *count = (int32_t *)tmp;
    float *upre = (float *)(tmp + p.off_upre);
    int32_t *pq = (int32_t *)(tmp + p.off_pq), *pi = cand ? nullptr : (int32_t *)(tmp + p.off_pi);
    float *sc = (float *)(tmp + p.off_sc);
    uint64_t *best = (uint64_t *)(tmp + p.off_best);

    int rc = ANN_OK;
    auto launched = [&]() {
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess && rc == ANN_OK) {
            set_error("kernel launch failed: %s", hipGetErrorString(e));
            rc = ANN_EDEVICE;
        }
    };
    hipLaunchKernelGGL(bf_clear_kernel, dim3(grid_for((int64_t)Q * k)), dim3(256), 0, s, best, (int64_t)Q * k);
    launched();
    if (rc == ANN_OK && mfma) rc = launch_user_pre(m, queries_dev, Q, upre, s);
    for (int q0 = 0; q0 < Q && rc == ANN_OK; q0 += Qb) {
        const int qb = Q - q0 < Qb ? Q - q0 : Qb;
        for (int64_t i0 = 0; i0 < total_per_query && rc == ANN_OK; i0 += nc_max) {
            const int nc = (int)(total_per_query - i0 < nc_max ? total_per_query - i0 : nc_max);
            const int M = qb * nc;
            const int32_t *ids = cand ? cand + (size_t)q0 * n : nullptr;  // one pass per block of queries
            hipLaunchKernelGGL(bf_fill_pairs_kernel, dim3(grid_for(M)), dim3(256), 0, s, pq, pi, q0, (int32_t)i0, nc, M,
                               count);
            launched();
            if (rc != ANN_OK) break;
            rc = mfma ? launch_mlp_mfma(g, m, upre, pq, cand ? ids : pi, count, M, Q, sc, 0, s)
                      : launch_mlp_alu(g, m, queries_dev, pq, cand ? ids : pi, nullptr, M, Q, sc, 0, s);
            if (rc != ANN_OK) break;
            hipLaunchKernelGGL(bf_topk_kernel, dim3(qb), dim3(BF_BLOCK), 0, s, sc, nc, (int32_t)i0, ids, g->N, best, k,
                               q0);
            launched();
        }
    }
    if (rc == ANN_OK) {
        hipLaunchKernelGGL(bf_emit_kernel, dim3(grid_for((int64_t)Q * k)), dim3(256), 0, s, best, (int64_t)Q * k,
                           out_ids_dev, out_scores_dev);
        launched();
    }
    if (ws) return rc;
    const hipError_t e = hipStreamSynchronize(s);
    if (rc == ANN_OK && e != hipSuccess) {
        set_error("hipStreamSynchronize failed: %s", hipGetErrorString(e));
        rc = ANN_EDEVICE;
    }
    (void)hipFree(tmp);
    return rc;
}

extern "C" size_t ann_brute_force_workspace_bytes(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t k) {
    BestKPlan p;
    return best_k_plan(g, m, Q, k, false, 0, &p) ? p.total : 0;
}

extern "C" size_t ann_rerank_workspace_bytes(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t n, int32_t k) {
    BestKPlan p;
    return best_k_plan(g, m, Q, k, true, n, &p) ? p.total : 0;
}

extern "C" int ann_brute_force(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q, int32_t k,
                               int32_t *out_ids_dev, float *out_scores_dev, void *workspace_dev,
                               size_t workspace_bytes, void *stream) {
    return best_k(g, m, queries_dev, Q, k, nullptr, 0, out_ids_dev, out_scores_dev, workspace_dev, workspace_bytes,
                  stream);
}

extern "C" int ann_rerank(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q,
                          const int32_t *cand_dev, int32_t n, int32_t k, int32_t *out_ids_dev, float *out_scores_dev,
                          void *workspace_dev, size_t workspace_bytes, void *stream) {
    if (!cand_dev) {
        set_error("cand_dev must not be null");
        return ANN_EINVAL;
    }
    return best_k(g, m, queries_dev, Q, k, cand_dev, n, out_ids_dev, out_scores_dev, workspace_dev, workspace_bytes,
                  stream);
}
