/*
 * sanitize_driver.c - runs the CPU oracle's entry points under the host sanitizers (test infrastructure).
 *
 * Built by tests/test_oracle_sanitize.py together with gmp_oracle.c with
 *     gcc -fsanitize=address,undefined -fno-sanitize-recover=all
 * so that an out-of-bounds access, a use after free, a signed overflow or a misaligned access anywhere in the
 * oracle ends the program with a report instead of going unseen behind a plausible result.
 *
 * Input (stdin): hand-derived trajectories on the directed ring graph adj[i] = (i+1 .. i+R) mod N with a
 * relevance strictly monotone in the item id, one case per line, numbers only:
 *     F N R dir W L k max_iters  n_seeds s..  n_ids id..  n_visited v..  n_expanded n_scored n_iters     (joint search)
 *     K N R dir T k              n_seeds s..  n_ids id..  n_visited v..  n_expanded n_scored n_iters     (walkers)
 * dir = 1 increasing, -1 decreasing.  The expected values come from the committed golden files; this program
 * holds none.  After the cases it drives brute force, pair scoring, the quantisers and the noise draw over
 * small inputs with awkward sizes (k larger than the item count, invalid pair indices, all-invalid seeds).
 * Exit status 0 and "sanitize_driver: ok" on stdout mean every call returned what it should.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_score_pairs(const void *emb, int dtype, int64_t N, int d, const void *users, int d_u, int64_t Q,
                       int n_layers, const int32_t *dims, const float *W, const float *b, const float *head_w,
                       int act_round, int64_t M, const int32_t *q_idx, const int32_t *item, float *out,
                       int n_threads);
int oracle_search(const void *emb, int dtype, int64_t N, int d, const int32_t *adj, int R, const void *users,
                  int d_u, int64_t Q, int n_layers, const int32_t *dims, const float *W, const float *b,
                  const float *head_w, int act_round, const int32_t *entries, int E, const int32_t *W_q,
                  const int32_t *L_q, const int32_t *cap_q, int k, int32_t *out_ids, float *out_scores,
                  int64_t *n_scored, int64_t *n_expanded, int32_t *n_iters, int32_t *visited_out,
                  int64_t visited_cap, float *worst_trace, int trace_cap, int n_threads);
int oracle_search_walkers(const void *emb, int dtype, int64_t N, int d, const int32_t *adj, int R,
                          const void *users, int d_u, int64_t Q, int n_layers, const int32_t *dims,
                          const float *W, const float *b, const float *head_w, int act_round,
                          const int32_t *entries, int E, int T, int k, int32_t *out_ids, float *out_scores,
                          int64_t *n_scored, int64_t *n_expanded, int32_t *n_iters, int32_t *visited_out,
                          int64_t visited_cap, int n_threads);
int oracle_brute_force(const void *emb, int dtype, int64_t N, int d, const void *users, int d_u, int64_t Q,
                       int n_layers, const int32_t *dims, const float *W, const float *b, const float *head_w,
                       int act_round, int k, int32_t *out_ids, float *out_scores, int n_threads);
int64_t oracle_e4m3_encode(const float *in, int64_t n, double scale, uint8_t *codes);
int64_t oracle_e4m3_quantize(const float *in, int64_t n, double scale, float *out);
void oracle_f16_round(const float *in, int64_t n, float *out);
int oracle_users_add_noise(const void *users, int dtype, int64_t Q, int d, double sigma, uint64_t seed,
                           uint64_t stream, void *out);

#define CHECK(cond, ...)                                  \
    do {                                                  \
        if (!(cond)) {                                    \
            fprintf(stderr, "sanitize_driver: " __VA_ARGS__); \
            fprintf(stderr, "\n");                        \
            exit(1);                                      \
        }                                                 \
    } while (0)

static int read_int(void) {
    int v;
    CHECK(scanf("%d", &v) == 1, "malformed input");
    return v;
}

static int *read_list(int *n) {
    *n = read_int();
    CHECK(*n >= 0 && *n < 100000, "bad list length");
    int *a = (int *)malloc(sizeof(int) * (size_t)(*n > 0 ? *n : 1));
    for (int i = 0; i < *n; ++i) a[i] = read_int();
    return a;
}

/* exactly sized arrays everywhere, so that the sanitizer sees any access one element too far */
static void run_case(char kind) {
    const int N = read_int(), R = read_int(), dir = read_int();
    int W = 1, L = 1, k, iters = 0, T = 0;
    if (kind == 'F') {
        W = read_int(), L = read_int(), k = read_int(), iters = read_int();
    } else {
        T = read_int(), k = read_int();
    }
    int n_seeds, n_ids, n_vis;
    int *seeds = read_list(&n_seeds), *want_ids = read_list(&n_ids), *want_vis = read_list(&n_vis);
    const int n_expanded = read_int(), n_scored = read_int(), n_iters = read_int();
    CHECK(n_ids == k, "a case lists %d ids for k = %d", n_ids, k);

    int32_t *adj = (int32_t *)malloc(sizeof(int32_t) * (size_t)N * R);
    float *emb = (float *)calloc((size_t)N * 2, sizeof(float));
    for (int i = 0; i < N; ++i) {
        for (int s = 0; s < R; ++s) adj[(size_t)i * R + s] = (i + 1 + s) % N;
        emb[2 * i] = (float)i / (float)N;
    }
    const int32_t dims[2] = {4, 1};
    const float Wt[4] = {0.f, 0.f, dir > 0 ? 4.f : -4.f, 0.f}, b[1] = {0.f}, hw[1] = {1.f}, users[2] = {0.f, 0.f};
    int32_t *entries = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_seeds);
    for (int i = 0; i < n_seeds; ++i) entries[i] = seeds[i];
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
    float *sc = (float *)malloc(sizeof(float) * (size_t)k);
    int32_t *vis = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_vis + 1));
    int64_t ns = -1, ne = -1;
    int32_t ni = -1;
    int rc;
    if (kind == 'F') {
        const int32_t Wq[1] = {W}, Lq[1] = {L}, cq[1] = {iters};
        float trace[8];
        rc = oracle_search(emb, 0, N, 2, adj, R, users, 2, 1, 1, dims, Wt, b, hw, 0, entries, n_seeds, Wq, Lq, cq, k,
                           ids, sc, &ns, &ne, &ni, vis, n_vis + 1, trace, 8, 1);
    } else {
        rc = oracle_search_walkers(emb, 0, N, 2, adj, R, users, 2, 1, 1, dims, Wt, b, hw, 0, entries, n_seeds, T, k, ids,
                                   sc, &ns, &ne, &ni, vis, n_vis + 1, 1);
    }
    CHECK(rc == 0, "search returned %d", rc);
    for (int i = 0; i < k; ++i) CHECK(ids[i] == want_ids[i], "result %d is %d, expected %d", i, ids[i], want_ids[i]);
    for (int i = 0; i < n_vis; ++i) CHECK(vis[i] == want_vis[i], "visit %d is %d, expected %d", i, vis[i], want_vis[i]);
    CHECK(vis[n_vis] == -1, "more ids visited than expected");
    CHECK(ns == n_scored && ne == n_expanded && ni == n_iters, "counters %lld %lld %d, expected %d %d %d",
          (long long)ns, (long long)ne, ni, n_scored, n_expanded, n_iters);
    free(adj), free(emb), free(entries), free(ids), free(sc), free(vis), free(seeds), free(want_ids), free(want_vis);
}

static uint32_t lcg(uint32_t *s) { return *s = *s * 1664525u + 1013904223u; }
static float unit(uint32_t *s) { return (float)(lcg(s) >> 8) / 16777216.0f * 2.f - 1.f; }

/* Calls with awkward sizes over a small random problem, fp32 and bf16 tables, every activation-rounding mode. */
static void odd_sizes(void) {
    enum { N = 37, R = 5, D = 6, DU = 3, H = 7, J = 3, Q = 4, E = 3 };
    uint32_t s = 12345u;
    float emb[N * D], users[Q * DU], W[(DU + D) * H + H * J], b[H + J], hw[J] = {0.5f, 0.3f, 0.2f};
    uint16_t emb16[N * D], users16[Q * DU];
    for (int i = 0; i < N * D; ++i) emb[i] = unit(&s);
    for (int i = 0; i < Q * DU; ++i) users[i] = unit(&s);
    for (size_t i = 0; i < sizeof(W) / sizeof(W[0]); ++i) W[i] = unit(&s) * 0.5f;
    for (int i = 0; i < H + J; ++i) b[i] = unit(&s) * 0.1f;
    for (int i = 0; i < N * D; ++i) {
        uint32_t u;
        memcpy(&u, &emb[i], 4);
        emb16[i] = (uint16_t)(u >> 16);
    }
    for (int i = 0; i < Q * DU; ++i) {
        uint32_t u;
        memcpy(&u, &users[i], 4);
        users16[i] = (uint16_t)(u >> 16);
    }
    int32_t adj[N * R];
    for (int i = 0; i < N * R; ++i) adj[i] = (int32_t)(lcg(&s) % (N + 3)) - 1; /* some ids invalid: -1, N, N+1 */
    const int32_t dims[3] = {DU + D, H, J};
    const int32_t entries[Q * E] = {0, 0, 5, -1, N, N + 7, 36, 1, 36, 3, 2, 1};
    const int32_t Wq[Q] = {1, 2, 3, 64}, Lq[Q] = {1, 4, 50, 3}, cq[Q] = {0, 2, 0, 1};
    for (int mode = 0; mode < 4; ++mode)
        for (int dt = 0; dt < 2; ++dt) {
            const void *e = dt ? (const void *)emb16 : (const void *)emb, *u = dt ? (const void *)users16 : (const void *)users;
            enum { K = N + 5 }; /* more results asked for than items exist */
            int32_t ids[Q * K];
            float sc[Q * K];
            CHECK(oracle_brute_force(e, dt, N, D, u, DU, Q, 2, dims, W, b, hw, mode, K, ids, sc, 2) == 0, "brute force");
            for (int q = 0; q < Q; ++q) {
                for (int i = 0; i < N; ++i) CHECK(ids[q * K + i] >= 0 && ids[q * K + i] < N, "brute-force id");
                for (int i = N; i < K; ++i) CHECK(ids[q * K + i] == -1 && isinf(sc[q * K + i]), "brute-force padding");
            }
            int64_t ns[Q], ne[Q];
            int32_t ni[Q], vis[Q * N];
            float tr[Q * 3];
            CHECK(oracle_search(e, dt, N, D, adj, R, u, DU, Q, 2, dims, W, b, hw, mode, entries, E, Wq, Lq, cq, K, ids, sc,
                                ns, ne, ni, vis, N, tr, 3, 2) == 0, "search");
            CHECK(ns[1] == 0 && ids[1 * K] == -1, "a query without a valid seed must return padding only");
            CHECK(oracle_search_walkers(e, dt, N, D, adj, R, u, DU, Q, 2, dims, W, b, hw, mode, entries, E, 4, K, ids, sc,
                                        ns, ne, ni, vis, N, 2) == 0, "walkers");
            const int32_t qi[5] = {0, 3, Q, -1, 2}, it[5] = {0, N - 1, 1, 1, N};
            float out[5];
            CHECK(oracle_score_pairs(e, dt, N, D, u, DU, Q, 2, dims, W, b, hw, mode, 5, qi, it, out, 2) == -1,
                  "pair indices out of range must be refused");
            CHECK(oracle_score_pairs(e, dt, N, D, u, DU, Q, 2, dims, W, b, hw, mode, 2, qi, it, out, 2) == 0, "score_pairs");
            CHECK(isfinite(out[0]) && isfinite(out[1]) && out[0] > 0.f && out[0] < 1.f, "a relevance lies in (0, 1)");
        }
    float big[9] = {0.f, -0.f, 1e-9f, 447.9f, 448.f, 449.f, -1e30f, 0.0019531f, 3.14159f}, q[9], h[9];
    uint8_t codes[9];
    CHECK(oracle_e4m3_encode(big, 9, 1.0, codes) == 2, "two magnitudes exceed the 8-bit range");
    CHECK(oracle_e4m3_quantize(big, 9, 4.0, q) >= 2, "scaled quantiser");
    oracle_f16_round(big, 9, h);
    float noisy[Q * DU];
    uint16_t noisy16[Q * DU];
    CHECK(oracle_users_add_noise(users, 0, Q, DU, 1.0, 77u, 3u, noisy) == 0, "noise fp32");
    CHECK(oracle_users_add_noise(users16, 1, Q, DU, 0.5, 77u, 3u, noisy16) == 0, "noise bf16");
}

int main(void) {
    int n_cases = 0;
    char kind;
    while (scanf(" %c", &kind) == 1) {
        CHECK(kind == 'F' || kind == 'K', "unknown case kind %c", kind);
        run_case(kind);
        ++n_cases;
    }
    odd_sizes();
    printf("sanitize_driver: ok, %d hand cases\n", n_cases);
    return 0;
}
