/*
 * CPU oracle for the batched graph search with a learned MLP relevance score.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct
 * statement of what the GPU library must compute.  It shares no code with the
 * HIP path and must never be called from it; only the tests, the smoke check
 * and the CPU-baseline leg of the benchmark may use it.
 *
 * What it follows (arXiv 2502.11490):
 *   - relevance of one (user, item) pair: Sec. 3.1 (1), Eq. 5-8.  The MLP input
 *     is the user vector followed by the item vector (Eq. 5); every layer is
 *     W h + b with W stored [out][in] (Eq. 7); the J outputs of the last layer
 *     are the per-behaviour predictions (Eq. 6) and the relevance is their fixed
 *     weighted combination (Eq. 8).
 *   - the search: Sec. 3.2 / Algorithm 1.  Several seeds per query are searched
 *     jointly, every scored neighbour is pushed into ONE bounded best-first
 *     container per query, larger relevance is better (Eq. 4).
 *   - ground truth for recall: brute-force sorted items (Sec. 5.1.3).
 *
 * Readings adopted where the paper is silent (kept identical in the GPU path):
 *   - ReLU after every hidden layer, none on the last layer; each head goes
 *     through a logistic sigmoid before the weighted sum;
 *   - the serendipity vector of Eq. 5 is not drawn inside the search: a caller who
 *     wants it adds it to the user vectors beforehand, with oracle_users_add_noise
 *     (a counter-based generator, so that the same draw can be repeated anywhere);
 *   - one sorted list per query of capacity C = max(L, k); per iteration the
 *     first <= W not-yet-expanded entries among the first L ranks are expanded
 *     together; order everywhere is (score descending, id ascending);
 *   - an id is scored at most once per query (exact visited set, seeds included);
 *     duplicates inside one iteration keep their first occurrence;
 *   - a query stops when none of its first L ranks is unexpanded or when its
 *     iteration cap (if > 0) is reached; seeding is not an iteration.
 *
 * Arithmetic: inputs are used exactly as stored (fp32, or bf16 widened exactly);
 * all sums and the sigmoid are in double; the relevance is rounded once to fp32.
 * With act_round = 1 each hidden activation is additionally rounded
 * double -> fp32 -> bf16 (round to nearest even) after the ReLU: that is the
 * precision the bf16 GPU kernels keep between layers, and is offered so that
 * rank decisions can be compared at the kernel's precision.
 * With act_round = 2 (the 8-bit metric) the activation of hidden layer l (l = 1, 2, ..) is
 * instead clamped to [0, 448 / s_l], s_l = 4^l, and rounded double -> fp32 -> e4m3 at that
 * scale (OCP 8-bit float, 4 exponent and 3 mantissa bits, bias 7, largest value 448,
 * nearest even), i.e. to e4m3(s_l * a) / s_l.  Weights and item vectors of that metric are
 * quantised by the caller beforehand (oracle_e4m3_encode / _quantize) and arrive here as
 * ordinary numbers.
 * With act_round = 3 (the fp16 metric, the 16-bit format of Sec. 4.3) each hidden activation is
 * rounded double -> fp32 -> binary16 (nearest even, overflow to infinity) after the ReLU; fp16
 * inputs and weights arrive widened to fp32, which is exact.
 *
 * Parity pins (tests/test_oracle_*.py): closed forms and hand-worked values for
 * the relevance, a library MLP forward pass, brute-force equality on complete
 * graphs / L >= N, a hand-derived ring-graph trajectory, an independently
 * written priority-queue best-first search for W = E = 1, monotonicity and
 * uniqueness invariants, and entry/batch permutation symmetries; for the binary16
 * rounding an independent library's conversion; for the noise
 * draw the generator's published known-answer vectors, goodness-of-fit of the
 * variates and of the Box-Muller pairs, and an independent bf16 rounding.  The recall
 * level reached on the synthetic graphs has no external pin: "parity unpinned"
 * for that single quantity.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { MAX_W = 1024 }; /* largest per-iteration expansion width accepted */

typedef struct {
    int n_layers;
    const int32_t *dims;   /* [n_layers + 1] */
    const float *W;        /* layers back to back, each [out][in] row-major */
    const float *b;        /* layers back to back, each [out] */
    const float *head_w;   /* [dims[n_layers]] */
    int act_round;
    int max_width;
} mlp_t;

static float widen_bf16(uint16_t bits) {
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static double load_elem(const void *base, int dtype, int64_t idx) {
    if (dtype == ORACLE_BF16) return (double)widen_bf16(((const uint16_t *)base)[idx]);
    return (double)((const float *)base)[idx];
}

/* double -> fp32 -> bf16, both round-to-nearest-even, returned widened */
static double round_to_bf16(double v) {
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return (double)f; /* inf / nan unchanged */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* Nearest e4m3 value (ties to even) of v after rounding v to fp32; |v| above 448 gives +-448.
 * e4m3: sign, 4 exponent bits (bias 7), 3 mantissa bits; normal values 2^(e-7) * (1 + m/8) for
 * e = 1..15 (without e = 15, m = 7, which is NaN), subnormals m/8 * 2^-6. */
static double round_to_e4m3(double v) {
    double a = fabs((double)(float)v);
    if (!(a == a)) return v;
    if (a > 448.0) a = 448.0;
    double quantum;
    if (a < 0.015625) { /* below 2^-6: subnormal spacing */
        quantum = 0.001953125; /* 2^-9 */
    } else {
        int e;
        (void)frexp(a, &e);            /* a = f * 2^e, f in [0.5, 1) */
        quantum = ldexp(1.0, e - 1 - 3); /* 2^(floor(log2 a) - 3) */
    }
    double q = nearbyint(a / quantum) * quantum; /* default rounding mode: nearest even */
    if (q > 448.0) q = 448.0;
    return signbit(v) ? -q : q;
}

/* the 8-bit code of an e4m3 value produced by round_to_e4m3 */
static uint8_t e4m3_code(double q) {
    uint8_t sign = (q < 0 || (q == 0 && signbit(q))) ? 0x80 : 0;
    double a = fabs(q);
    if (a == 0) return sign;
    if (a < 0.015625) return (uint8_t)(sign | (uint8_t)(a / 0.001953125));
    int e;
    double f = frexp(a, &e); /* a = f * 2^e, f in [0.5, 1) -> 1.m = 2f, exponent e - 1 */
    int m = (int)((2.0 * f - 1.0) * 8.0);
    return (uint8_t)(sign | ((e - 1 + 7) << 3) | m);
}

/* codes[i] = e4m3(scale * in[i]); returns the number of elements whose magnitude had to be clamped */
int64_t oracle_e4m3_encode(const float *in, int64_t n, double scale, uint8_t *codes) {
    int64_t clamped = 0;
    for (int64_t i = 0; i < n; ++i) {
        double v = (double)in[i] * scale;
        if (fabs((double)(float)v) > 448.0) ++clamped;
        codes[i] = e4m3_code(round_to_e4m3(v));
    }
    return clamped;
}

/* out[i] = e4m3(scale * in[i]) / scale */
/* double -> fp32 -> binary16 (5 exponent bits, 10 fraction bits, subnormals below 2^-14), both
 * round-to-nearest-even; beyond the largest value 65504 the result is infinity; returned widened */
static double round_to_f16(double v) {
    float f = (float)v;
    if (f != f || f == 0.0f || isinf(f)) return (double)f;
    float a = fabsf(f);
    if (a >= 65520.0f) return f < 0 ? -INFINITY : INFINITY; /* 65520: half-way to 2^16, ties go to even */
    int e;
    (void)frexpf(a, &e);            /* a = m 2^e with m in [0.5, 1): 11 significant bits -> spacing 2^(e-11) */
    int q = e - 11;
    if (q < -24) q = -24;           /* subnormal spacing */
    float r = ldexpf(nearbyintf(ldexpf(a, -q)), q); /* scaling by powers of two is exact */
    return (double)(f < 0 ? -r : r);
}

void oracle_f16_round(const float *in, int64_t n, float *out) {
    for (int64_t i = 0; i < n; ++i) out[i] = (float)round_to_f16((double)in[i]);
}

int64_t oracle_e4m3_quantize(const float *in, int64_t n, double scale, float *out) {
    int64_t clamped = 0;
    for (int64_t i = 0; i < n; ++i) {
        double v = (double)in[i] * scale;
        if (fabs((double)(float)v) > 448.0) ++clamped;
        out[i] = (float)(round_to_e4m3(v) / scale);
    }
    return clamped;
}

static int mlp_max_width(const mlp_t *m) {
    int w = 0;
    for (int l = 0; l <= m->n_layers; ++l)
        if (m->dims[l] > w) w = m->dims[l];
    return w;
}

/* Eq. 5-8 for one pair.  x holds concat(user, item) in double; h0/h1 are scratch of max width. */
static float relevance(const mlp_t *m, const double *x, double *h0, double *h1) {
    const double *in = x;
    double *out = h0;
    const float *W = m->W;
    const float *b = m->b;
    for (int l = 0; l < m->n_layers; ++l) {
        int n_in = m->dims[l], n_out = m->dims[l + 1];
        int last = (l == m->n_layers - 1);
        for (int o = 0; o < n_out; ++o) {
            double acc = 0.0;
            const float *row = W + (int64_t)o * n_in;
            for (int i = 0; i < n_in; ++i) acc += (double)row[i] * in[i];
            acc += (double)b[o];
            if (!last) {
                if (acc < 0.0) acc = 0.0;
                if (m->act_round == 1) acc = round_to_bf16(acc);
                if (m->act_round == 3) acc = round_to_f16(acc);
                if (m->act_round == 2) {
                    double scale = ldexp(1.0, 2 * (l + 1)); /* 4^(l+1) */
                    acc = round_to_e4m3(acc * scale) / scale;
                }
            }
            out[o] = acc;
        }
        W += (int64_t)n_in * n_out;
        b += n_out;
        in = out;
        out = (out == h0) ? h1 : h0;
    }
    int J = m->dims[m->n_layers];
    double s = 0.0;
    for (int j = 0; j < J; ++j) s += (double)m->head_w[j] * (1.0 / (1.0 + exp(-in[j])));
    return (float)s;
}

static void build_input(double *x, const void *users, int dtype, int d_u, int64_t q,
                        const void *emb, int d, int64_t v) {
    for (int i = 0; i < d_u; ++i) x[i] = load_elem(users, dtype, q * d_u + i);
    for (int i = 0; i < d; ++i) x[d_u + i] = load_elem(emb, dtype, v * d + i);
}

static mlp_t make_mlp(int n_layers, const int32_t *dims, const float *W, const float *b,
                      const float *head_w, int act_round) {
    mlp_t m;
    m.n_layers = n_layers;
    m.dims = dims;
    m.W = W;
    m.b = b;
    m.head_w = head_w;
    m.act_round = act_round;
    m.max_width = 0;
    m.max_width = mlp_max_width(&m);
    return m;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* relevance of an explicit list of pairs */
int oracle_score_pairs(const void *emb, int dtype, int64_t N, int d, const void *users, int d_u,
                       int64_t Q, int n_layers, const int32_t *dims, const float *W,
                       const float *b, const float *head_w, int act_round, int64_t M,
                       const int32_t *q_idx, const int32_t *item, float *out, int n_threads) {
    if (n_layers < 1 || dims[0] != d_u + d) return -1;
    mlp_t m = make_mlp(n_layers, dims, W, b, head_w, act_round);
    for (int64_t r = 0; r < M; ++r)
        if (q_idx[r] < 0 || q_idx[r] >= Q || item[r] < 0 || item[r] >= N) return -1;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel num_threads(n_threads)
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)(dims[0] + 2 * m.max_width));
        double *h0 = x + dims[0], *h1 = h0 + m.max_width;
#pragma omp for schedule(dynamic, 16)
        for (int64_t r = 0; r < M; ++r) {
            build_input(x, users, dtype, d_u, q_idx[r], emb, d, item[r]);
            out[r] = relevance(&m, x, h0, h1);
        }
        free(x);
    }
    return 0;
}

typedef struct {
    float score;
    int32_t id;
    int32_t expanded;
} entry_t;

/* (score descending, id ascending) */
static int entry_cmp(const void *pa, const void *pb) {
    const entry_t *a = (const entry_t *)pa, *b = (const entry_t *)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    if (a->id < b->id) return -1;
    if (a->id > b->id) return 1;
    return 0;
}

static int bit_get(const uint8_t *bm, int64_t i) { return (bm[i >> 3] >> (i & 7)) & 1; }
static void bit_set(uint8_t *bm, int64_t i) { bm[i >> 3] |= (uint8_t)(1u << (i & 7)); }

/*
 * Synchronous search, one query after another (Algorithm 1, shared container).
 * W_q, L_q, cap_q: per-query expansion width, eligible ranks, iteration cap (0 = none).
 * Optional traces (NULL to skip):
 *   n_scored[Q], n_expanded[Q], n_iters[Q];
 *   visited_out[Q][visited_cap]: ids in the order they were scored (-1 padded);
 *   worst_trace[Q][trace_cap]: entry t = score at rank L after iteration t (t = 0 is the
 *   seeding), -inf while the list is shorter than L; unused slots = NaN.
 */
int oracle_search(const void *emb, int dtype, int64_t N, int d, const int32_t *adj, int R,
                  const void *users, int d_u, int64_t Q, int n_layers, const int32_t *dims,
                  const float *W, const float *b, const float *head_w, int act_round,
                  const int32_t *entries, int E, const int32_t *W_q, const int32_t *L_q,
                  const int32_t *cap_q, int k, int32_t *out_ids, float *out_scores,
                  int64_t *n_scored, int64_t *n_expanded, int32_t *n_iters, int32_t *visited_out,
                  int64_t visited_cap, float *worst_trace, int trace_cap, int n_threads) {
    if (n_layers < 1 || dims[0] != d_u + d || k < 1 || E < 1 || R < 1) return -1;
    for (int64_t q = 0; q < Q; ++q)
        if (W_q[q] < 1 || W_q[q] > MAX_W || L_q[q] < 1 || cap_q[q] < 0) return -1;
    mlp_t m = make_mlp(n_layers, dims, W, b, head_w, act_round);
    if (n_threads < 1) n_threads = 1;
    int fail = 0;
#pragma omp parallel num_threads(n_threads)
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)(dims[0] + 2 * m.max_width));
        double *h0 = x + dims[0], *h1 = h0 + m.max_width;
        uint8_t *visited = (uint8_t *)malloc((size_t)((N + 7) / 8));
        entry_t *list = NULL;
        int32_t *fresh = NULL;
        size_t list_cap = 0, fresh_cap = 0;
#pragma omp for schedule(dynamic, 1)
        for (int64_t q = 0; q < Q; ++q) {
            const int Wq = W_q[q], Lq = L_q[q], cap = cap_q[q];
            const int C = Lq > k ? Lq : k;
            size_t need_list = (size_t)C + (size_t)Wq * R + (size_t)E;
            size_t need_fresh = (size_t)Wq * R + (size_t)E;
            if (need_list > list_cap) {
                list = (entry_t *)realloc(list, need_list * sizeof(entry_t));
                list_cap = need_list;
            }
            if (need_fresh > fresh_cap) {
                fresh = (int32_t *)realloc(fresh, need_fresh * sizeof(int32_t));
                fresh_cap = need_fresh;
            }
            if (!x || !visited || !list || !fresh) {
                fail = 1;
                continue;
            }
            memset(visited, 0, (size_t)((N + 7) / 8));
            int64_t scored = 0, expanded = 0;
            int len = 0;
            if (worst_trace)
                for (int t = 0; t < trace_cap; ++t) worst_trace[q * trace_cap + t] = NAN;
            if (visited_out)
                for (int64_t i = 0; i < visited_cap; ++i) visited_out[q * visited_cap + i] = -1;

            /* seeds, in the order given */
            for (int e = 0; e < E; ++e) {
                int32_t v = entries[q * E + e];
                if (v < 0 || v >= N || bit_get(visited, v)) continue;
                bit_set(visited, v);
                build_input(x, users, dtype, d_u, q, emb, d, v);
                list[len].score = relevance(&m, x, h0, h1);
                list[len].id = v;
                list[len].expanded = 0;
                ++len;
                if (visited_out && scored < visited_cap) visited_out[q * visited_cap + scored] = v;
                ++scored;
            }
            qsort(list, (size_t)len, sizeof(entry_t), entry_cmp);
            if (len > C) len = C;
            if (worst_trace && trace_cap > 0)
                worst_trace[q * trace_cap] = (len >= Lq) ? list[Lq - 1].score : -INFINITY;

            int t = 0;
            for (;;) {
                if (cap > 0 && t == cap) break;
                /* the first <= W unexpanded entries among the first L ranks; all are chosen
                   before any of their neighbours is merged */
                int n_par = 0;
                int32_t parents[MAX_W];
                int lim = len < Lq ? len : Lq;
                for (int r = 0; r < lim && n_par < Wq; ++r)
                    if (!list[r].expanded) {
                        list[r].expanded = 1;
                        parents[n_par++] = list[r].id;
                    }
                if (n_par == 0) break;
                expanded += n_par;
                int n_new = 0;
                for (int p = 0; p < n_par; ++p)
                    for (int s = 0; s < R; ++s) {
                        int32_t v = adj[(int64_t)parents[p] * R + s];
                        if (v < 0 || v >= N || bit_get(visited, v)) continue;
                        bit_set(visited, v);
                        fresh[n_new++] = v;
                    }
                for (int i = 0; i < n_new; ++i) {
                    int32_t v = fresh[i];
                    build_input(x, users, dtype, d_u, q, emb, d, v);
                    list[len].score = relevance(&m, x, h0, h1);
                    list[len].id = v;
                    list[len].expanded = 0;
                    ++len;
                    if (visited_out && scored < visited_cap)
                        visited_out[q * visited_cap + scored] = v;
                    ++scored;
                }
                qsort(list, (size_t)len, sizeof(entry_t), entry_cmp);
                if (len > C) len = C;
                ++t;
                if (worst_trace && t < trace_cap)
                    worst_trace[q * trace_cap + t] = (len >= Lq) ? list[Lq - 1].score : -INFINITY;
            }
            for (int i = 0; i < k; ++i) {
                out_ids[q * k + i] = i < len ? list[i].id : -1;
                out_scores[q * k + i] = i < len ? list[i].score : -INFINITY;
            }
            if (n_scored) n_scored[q] = scored;
            if (n_expanded) n_expanded[q] = expanded;
            if (n_iters) n_iters[q] = t;
        }
        free(x);
        free(visited);
        free(list);
        free(fresh);
    }
    return fail ? -2 : 0;
}

/* Paper-literal inter-candidate search (Sec. 3.2, Algorithm 1 read as K independent walkers
 * sharing one result container: one search process per seed runs at the same time as the
 * others, each moving through the graph towards its most relevant neighbours, and the only
 * thing the processes have in common is the bounded container that keeps the best items any
 * of them has found).
 *
 * Per query: every distinct in-range seed, in the order given, is scored, pushed into the
 * shared list and becomes the position of one walker (walker index = position of the seed in
 * the entries row).  Then T hops: in walker order, every live walker looks at the R neighbours
 * of its position; the ones no walker of this query has scored before (shared visited set,
 * first occurrence wins) are scored and pushed; the walker moves to the best of ITS newly
 * scored neighbours (score desc, id asc) and dies if it has none.  All walkers of a hop read
 * their neighbours before any of them moves.  Result: the k best of everything scored. */
int oracle_search_walkers(const void *emb, int dtype, int64_t N, int d, const int32_t *adj, int R,
                          const void *users, int d_u, int64_t Q, int n_layers, const int32_t *dims,
                          const float *W, const float *b, const float *head_w, int act_round,
                          const int32_t *entries, int E, int T, int k, int32_t *out_ids,
                          float *out_scores, int64_t *n_scored, int64_t *n_expanded,
                          int32_t *n_iters, int32_t *visited_out, int64_t visited_cap,
                          int n_threads) {
    if (n_layers < 1 || dims[0] != d_u + d || k < 1 || E < 1 || R < 1 || T < 0) return -1;
    mlp_t m = make_mlp(n_layers, dims, W, b, head_w, act_round);
    if (n_threads < 1) n_threads = 1;
    int fail = 0;
#pragma omp parallel num_threads(n_threads)
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)(dims[0] + 2 * m.max_width));
        double *h0 = x + dims[0], *h1 = h0 + m.max_width;
        uint8_t *visited = (uint8_t *)malloc((size_t)((N + 7) / 8));
        entry_t *list = (entry_t *)malloc(sizeof(entry_t) * ((size_t)k + (size_t)E * R + (size_t)E));
        int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);   /* walker -> item, -1 dead */
        entry_t *best = (entry_t *)malloc(sizeof(entry_t) * (size_t)E);
#pragma omp for schedule(dynamic, 1)
        for (int64_t q = 0; q < Q; ++q) {
            if (!x || !visited || !list || !pos || !best) {
                fail = 1;
                continue;
            }
            memset(visited, 0, (size_t)((N + 7) / 8));
            int64_t scored = 0, expanded = 0;
            int len = 0;
            if (visited_out)
                for (int64_t i = 0; i < visited_cap; ++i) visited_out[q * visited_cap + i] = -1;
            for (int e = 0; e < E; ++e) {
                int32_t v = entries[q * E + e];
                pos[e] = -1;
                if (v < 0 || v >= N || bit_get(visited, v)) continue;
                bit_set(visited, v);
                pos[e] = v;
                build_input(x, users, dtype, d_u, q, emb, d, v);
                list[len].score = relevance(&m, x, h0, h1);
                list[len].id = v;
                list[len].expanded = 0;
                ++len;
                if (visited_out && scored < visited_cap) visited_out[q * visited_cap + scored] = v;
                ++scored;
            }
            qsort(list, (size_t)len, sizeof(entry_t), entry_cmp);
            if (len > k) len = k;
            int t = 0;
            for (; t < T; ++t) {
                int live = 0;
                for (int e = 0; e < E; ++e) live += (pos[e] >= 0);
                if (!live) break;
                expanded += live;
                for (int e = 0; e < E; ++e) {
                    int have = 0;
                    if (pos[e] >= 0)
                        for (int s = 0; s < R; ++s) {
                            int32_t v = adj[(int64_t)pos[e] * R + s];
                            if (v < 0 || v >= N || bit_get(visited, v)) continue;
                            bit_set(visited, v);
                            build_input(x, users, dtype, d_u, q, emb, d, v);
                            entry_t c;
                            c.score = relevance(&m, x, h0, h1);
                            c.id = v;
                            c.expanded = 0;
                            list[len++] = c;
                            if (!have || entry_cmp(&c, &best[e]) < 0) best[e] = c;
                            have = 1;
                            if (visited_out && scored < visited_cap)
                                visited_out[q * visited_cap + scored] = v;
                            ++scored;
                        }
                    /* positions change only after every walker has read its neighbours: they
                       are taken from pos[], which is rewritten below */
                    best[e].expanded = have;
                }
                for (int e = 0; e < E; ++e)
                    if (pos[e] >= 0) pos[e] = best[e].expanded ? best[e].id : -1;
                qsort(list, (size_t)len, sizeof(entry_t), entry_cmp);
                if (len > k) len = k;
            }
            for (int i = 0; i < k; ++i) {
                out_ids[q * k + i] = i < len ? list[i].id : -1;
                out_scores[q * k + i] = i < len ? list[i].score : -INFINITY;
            }
            if (n_scored) n_scored[q] = scored;
            if (n_expanded) n_expanded[q] = expanded;
            if (n_iters) n_iters[q] = t;
        }
        free(x);
        free(visited);
        free(list);
        free(pos);
        free(best);
    }
    return fail ? -2 : 0;
}


/* exhaustive top-k of the same relevance (ground truth for recall) */
int oracle_brute_force(const void *emb, int dtype, int64_t N, int d, const void *users, int d_u,
                       int64_t Q, int n_layers, const int32_t *dims, const float *W,
                       const float *b, const float *head_w, int act_round, int k,
                       int32_t *out_ids, float *out_scores, int n_threads) {
    if (n_layers < 1 || dims[0] != d_u + d || k < 1) return -1;
    mlp_t m = make_mlp(n_layers, dims, W, b, head_w, act_round);
    if (n_threads < 1) n_threads = 1;
    int fail = 0;
#pragma omp parallel num_threads(n_threads)
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)(dims[0] + 2 * m.max_width));
        double *h0 = x + dims[0], *h1 = h0 + m.max_width;
        entry_t *all = (entry_t *)malloc(sizeof(entry_t) * (size_t)(N > 0 ? N : 1));
#pragma omp for schedule(dynamic, 1)
        for (int64_t q = 0; q < Q; ++q) {
            if (!x || !all) {
                fail = 1;
                continue;
            }
            for (int64_t v = 0; v < N; ++v) {
                build_input(x, users, dtype, d_u, q, emb, d, v);
                all[v].score = relevance(&m, x, h0, h1);
                all[v].id = (int32_t)v;
                all[v].expanded = 0;
            }
            qsort(all, (size_t)N, sizeof(entry_t), entry_cmp);
            for (int i = 0; i < k; ++i) {
                out_ids[q * k + i] = i < N ? all[i].id : -1;
                out_scores[q * k + i] = i < N ? all[i].score : -INFINITY;
            }
        }
        free(x);
        free(all);
    }
    return fail ? -2 : 0;
}

/* ------------------------------------------------------------------------------------------
 * Serendipity vector (Eq. 5): the user half of the metric input is h_u + h~ with h~ drawn from a
 * normal distribution, which the paper gives as N(0, 1); sigma scales it (sigma = 1 is the paper's).
 *
 * The draw is a pure function of (seed, stream, element index), so any implementation repeats it:
 *   - Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
 *     SC'11): counter = (block lo, block hi, stream lo, stream hi), key = (seed lo, seed hi), where
 *     element e = q * d + c of the [Q][d] array lies in block e / 4 and takes output word e % 4;
 *   - uniforms u_i = (x_i + 1/2) / 2^32, strictly inside (0, 1);
 *   - Box-Muller on the pairs (u_0, u_1) and (u_2, u_3): r = sqrt(-2 ln u_a), t = 2 pi u_b,
 *     the even word of a pair takes r cos t, the odd word r sin t;
 *   - out = user + sigma * z in double, rounded double -> fp32 (-> bf16 for a bf16 array).
 */
static void mulhilo32(uint32_t a, uint32_t b, uint32_t *hi, uint32_t *lo) {
    uint64_t p = (uint64_t)a * (uint64_t)b;
    *hi = (uint32_t)(p >> 32);
    *lo = (uint32_t)p;
}

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint32_t hi0, lo0, hi1, lo1;
        mulhilo32(0xD2511F53u, c0, &hi0, &lo0);
        mulhilo32(0xCD9E8D57u, c2, &hi1, &lo1);
        uint32_t n0 = hi1 ^ c1 ^ k0, n1 = lo1, n2 = hi0 ^ c3 ^ k1, n3 = lo0;
        c0 = n0, c1 = n1, c2 = n2, c3 = n3;
        k0 += 0x9E3779B9u; /* golden ratio */
        k1 += 0xBB67AE85u; /* sqrt(3) - 1 */
    }
    out[0] = c0, out[1] = c1, out[2] = c2, out[3] = c3;
}

/* the standard normal variate of element e (see above) */
double oracle_noise_element(uint64_t seed, uint64_t stream, uint64_t e) {
    const uint64_t block = e >> 2;
    const int word = (int)(e & 3);
    const uint32_t ctr[4] = {(uint32_t)block, (uint32_t)(block >> 32), (uint32_t)stream, (uint32_t)(stream >> 32)};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t x[4];
    oracle_philox4x32_10(ctr, key, x);
    const int a = word & 2; /* first word of the pair */
    const double ua = ((double)x[a] + 0.5) / 4294967296.0;
    const double ub = ((double)x[a + 1] + 0.5) / 4294967296.0;
    const double r = sqrt(-2.0 * log(ua));
    const double t = 6.283185307179586476925286766559 * ub;
    return (word & 1) ? r * sin(t) : r * cos(t);
}

int oracle_users_add_noise(const void *users, int dtype, int64_t Q, int d, double sigma, uint64_t seed,
                           uint64_t stream, void *out) {
    if (Q < 0 || d < 1 || (dtype != ORACLE_F32 && dtype != ORACLE_BF16)) return -1;
    for (int64_t e = 0; e < Q * (int64_t)d; ++e) {
        const double v = load_elem(users, dtype, e) + sigma * oracle_noise_element(seed, stream, (uint64_t)e);
        if (dtype == ORACLE_BF16) {
            float f = (float)round_to_bf16(v);
            uint32_t u;
            memcpy(&u, &f, 4);
            ((uint16_t *)out)[e] = (uint16_t)(u >> 16);
        } else {
            ((float *)out)[e] = (float)v;
        }
    }
    return 0;
}
