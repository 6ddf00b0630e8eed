/*
 * gmpgr_ann.h - C ABI of the MI355X graph-retrieval hot path.
 *
 * What the library computes (arXiv 2502.11490):
 *   - the relevance of a (user, item) pair is a small multi-head MLP over
 *     concat(user vector, item vector) (Sec. 3.1 (1), Eq. 5-7) whose J outputs are
 *     combined with fixed weights (Eq. 8).  Readings fixed by this library: ReLU
 *     after every hidden layer, a logistic sigmoid on every head, so
 *         relevance = sum_j head_w[j] * sigmoid(z_j);
 *   - retrieval is a joint best-first search on a fixed-degree item graph
 *     (Sec. 3.2, Algorithm 1): all seeds of a query share ONE bounded candidate
 *     container; larger relevance is better (Eq. 4);
 *   - the ragged (user, item) groups produced by all queries in one round are
 *     packed into dense fixed-size batches for the MLP (Sec. 3.2, Algorithm 2).
 *
 * Search rule (identical for every query, queries are independent):
 *   list  = sorted by (relevance descending, id ascending), capacity C = max(L, k)
 *   seed  : every distinct in-range entry id is scored once and inserted
 *   round : the first <= W not-yet-expanded entries among the first L ranks are
 *           marked expanded together; their adjacency rows are read; ids that are
 *           out of range, already scored for this query, or repeated inside the
 *           round are dropped (first occurrence kept); the rest are scored and
 *           merged into the list
 *   stop  : no unexpanded entry among the first L ranks, or max_iters rounds done
 *   out   : first k list entries; unused slots are id -1, score -inf
 *
 * Conventions
 *   - every pointer named *_dev is DEVICE memory, *_host is HOST memory;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream); all
 *     work is enqueued on it in order;
 *   - every function returns ANN_OK (0) or a negative code and never throws,
 *     aborts or prints; ann_last_error() gives the reason (thread local);
 *   - arguments are checked before anything is launched; a failed call launches
 *     nothing unless stated otherwise;
 *   - the library performs every step on the GPU.  There is no CPU fallback.
 */
#ifndef GMPGR_ANN_H
#define GMPGR_ANN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ANN_OK = 0,
    ANN_EINVAL = -1,     /* bad argument or argument combination */
    ANN_ENOMEM = -2,     /* host or device allocation failed */
    ANN_EDEVICE = -3,    /* a HIP call failed */
    ANN_ENOTIMPL = -4,   /* shape / dtype outside what the kernels support */
    ANN_EWORKSPACE = -5  /* workspace too small, or a per-query visited table filled up */
};

enum { ANN_F32 = 0, ANN_BF16 = 1, ANN_F8 = 2, ANN_F16 = 3 };

enum {
    ANN_VALIDATE = 1u,   /* ann_graph_load: check on the device that every adjacency id is < N */
    ANN_MLP_GENERIC = 2u /* ann_mlp_load: never pick the MFMA kernels (plain fp32-ALU path) */
};

typedef struct ann_graph ann_graph; /* opaque */
typedef struct ann_mlp ann_mlp;     /* opaque */

/* Counters of the last search that used a workspace (see ann_search_stats). */
typedef struct ann_stats {
    int64_t pairs_scored;    /* (user,item) pairs evaluated by the MLP, seeds included */
    int64_t nodes_expanded;  /* adjacency rows read */
    int64_t max_query_iters; /* largest number of rounds any query ran */
    int64_t visited_overflow;/* queries stopped because their visited table filled up */
    int64_t queries;         /* Q of that search */
    /* algorithmic bytes of the gather stages: what the method has to move, not what the caches moved */
    int64_t adjacency_bytes; /* nodes_expanded * R * 4: neighbour gather (Algorithm 1) */
    int64_t embedding_bytes; /* pairs_scored * bytes of one item row: embedding gather of the MLP stage (Eq. 5) */
    int64_t pair_list_bytes; /* pairs_scored * 12: user index, item id and score of the dense pair list (Algorithm 2) */
} ann_stats;

/*
 * The item graph of Sec. 3.2 (base layer, fixed out-degree).
 *   adj_dev : [N][R] int32 row-major neighbour ids; ids outside [0, N) are ignored by the search
 *   emb_dev : [N][d] row-major item vectors, fp32 (ANN_F32), bf16 (ANN_BF16) or fp16 (ANN_F16)
 * Both arrays are BORROWED: they must stay valid and unchanged until ann_graph_free.
 * Requirements: 1 <= N < 2^31, 1 <= R <= 64, 1 <= d <= 1024; rows must be 4-byte aligned,
 * 16-byte alignment of emb_dev and d*sizeof(elem) % 16 == 0 are needed for the MFMA path.
 * ANN_VALIDATE makes the call synchronise `stream` and return ANN_EINVAL if an id is >= N
 * (negative ids are allowed and mean "no edge").
 */
int ann_graph_load(const int32_t *adj_dev, const void *emb_dev, int64_t N, int32_t R, int32_t d,
                   int32_t dtype, uint32_t flags, void *stream, ann_graph **out);
void ann_graph_free(ann_graph *g);

/*
 * Locality order of the visited set (optional; changes no result).  Where a search keeps its exact visited set
 * (the ids scored for a query, Sec. 3.2's search: an id is scored once) as one bit per item, the bit of item v
 * is bit rank_dev[v] instead of bit v.  A rank under which items joined by edges lie close together (for
 * instance a numbering of the graph's communities) lets the neighbours of an expanded node fall into the same
 * 64-byte lines of the bitmap; ids, results, their order and every counter stay exactly those of the search
 * without it.  Searches whose visited set is the hash table ignore the rank.
 * rank_dev: [N] int32, a permutation of 0 .. N-1, device memory, BORROWED until the graph is freed or the call is
 * repeated; NULL removes the order.  The call checks on the device that rank_dev is a permutation (ANN_EINVAL if
 * not), builds its own [N][R] table of the adjacency entries' ranks (N * R * 4 bytes of device memory, freed with
 * the graph; ANN_ENOMEM), and synchronises `stream`.  Not to be called while a search on this graph is running.
 */
int ann_graph_set_locality(ann_graph *g, const int32_t *rank_dev, void *stream);

/*
 * Which form the exact visited set of a search with these parameters takes (arguments as for
 * ann_search_workspace_bytes): 1 = one bit per item (long lists on a moderate item count; the form
 * ann_graph_set_locality acts on), 0 = the per-query hash table; ANN_EINVAL for arguments the search would refuse.
 */
int ann_search_visited_set_is_bitmap(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t E, int32_t W_max,
                                     int32_t L_max, int32_t k, int32_t max_iters_max);

/*
 * The relevance metric of Sec. 3.1 (1): n_layers affine layers, Eq. 7 (W h + b).
 *   dims_host   : [n_layers + 1]; dims[0] = d_user + d_item, dims[n_layers] = J (1 <= J <= 8)
 *   W_host[l]   : [dims[l+1]][dims[l]] row-major, fp32, bf16 or fp16 as `dtype`; the first d_user
 *                 columns of W_host[0] multiply the user vector (Eq. 5: user first)
 *   b_host[l]   : [dims[l+1]] fp32
 *   head_w_host : [J] fp32 combination weights (the vector A of Eq. 8)
 * Everything is COPIED to the device (and re-laid-out for the kernels); the host arrays may
 * be freed afterwards.  1 <= n_layers <= 8, every width <= 2048.
 * dtype = ANN_BF16 means: items, users and weights are bf16, products are accumulated in
 * fp32, every hidden activation is rounded to bf16 (nearest even) after its ReLU, head
 * logits, sigmoid and the weighted sum stay in fp32 (the 16-bit deployment of Sec. 4.3).
 * dtype = ANN_F16 is the same with IEEE binary16 in place of bf16 (the format Sec. 4.3 names): items,
 * users and weights are fp16, hidden activations are rounded to fp16 (nearest even) after the ReLU.
 * ann_quantize_e4m3 does not take fp16 arrays.
 */
int ann_mlp_load(int32_t n_layers, const int32_t *dims_host, const void *const *W_host,
                 const float *const *b_host, const float *head_w_host, int32_t d_user,
                 int32_t dtype, uint32_t flags, void *stream, ann_mlp **out);
void ann_mlp_free(ann_mlp *m);

/* 1 if searches with this metric run the MFMA kernels, 0 if the plain ALU kernels. */
int ann_mlp_uses_mfma(const ann_mlp *m);

/*
 * Bytes of device workspace ann_search / ann_search_ragged need for at most Q queries,
 * E entry points, expansion width <= W_max, eligible ranks <= L_max, k results and
 * <= max_iters_max rounds per query.  The per-query visited table is sized for
 *     E + rounds * W_max * R ids,  rounds = max_iters_max > 0 ? max_iters_max
 *                                                            : 2 * ceil(L_max / W_max) + 32
 * (at most N).  A query that would outgrow its table stops early and is counted in
 * ann_stats.visited_overflow.  Where such a table takes a megabyte or more and one bit per item (N / 8 bytes
 * per query) is at most twice its size, the visited set is that bitmap instead, which cannot fill up.  The
 * environment variable GMPGR_VISITED_SET = "hash" or "bitmap", read by this call and by every search,
 * overrides the choice (for measurements and tests; it must not change between sizing and searching).
 * Returns 0 on invalid arguments (see ann_last_error).
 */
size_t ann_search_workspace_bytes(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t E,
                                  int32_t W_max, int32_t L_max, int32_t k,
                                  int32_t max_iters_max);

/*
 * Batched search (Sec. 3.2, Algorithms 1 and 2) for Q independent queries.
 *   queries_dev   : [Q][d_user] user vectors, dtype of the metric
 *   entry_dev     : [Q][E] int32 seed ids (out-of-range or repeated ids are ignored)
 *   W, L, k       : expansion width, eligible ranks, results per query (all >= 1)
 *   max_iters     : rounds per query, 0 = until converged
 *   workspace_dev : >= ann_search_workspace_bytes(g, m, Q, E, W, L, k, max_iters) bytes,
 *                   256-byte aligned; contents need not be preserved between calls
 *   out_ids_dev   : [Q][k] int32, out_scores_dev : [Q][k] fp32 (padding: -1 / -inf)
 * With max_iters > 0 the call only enqueues work.  With max_iters = 0 it also follows the
 * device's progress (a word in pinned host memory that the kernels update every round) to learn
 * when every query has converged, stays a few rounds ahead of the device meanwhile, and waits
 * on `stream` once, at the end (so such a call cannot be recorded into a HIP graph; a capped
 * one can: it launches kernels only).  Work enqueued on `stream` before the call is waited for up to
 * the limit of ann_set_progress_timeout; ANN_EDEVICE if the stream reports an error, runs dry without the
 * progress the kernels report, or reports nothing within that limit.
 * Limits: W*R <= 4096, E <= 1024; L and k are bounded by the workspace only (the list of a query lives in
 * device memory, 8 bytes per entry, and is merged in place through a tile in LDS).
 * Returns ANN_EWORKSPACE (results still written, for the truncated search) if the call
 * waited on the stream and saw a query fill its visited table; with max_iters > 0 use
 * ann_search_stats to learn about that.
 * Calls that share a workspace must not overlap in time.
 */
int ann_search(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q,
               const int32_t *entry_dev, int32_t E, int32_t W, int32_t L, int32_t k,
               int32_t max_iters, void *workspace_dev, size_t workspace_bytes,
               int32_t *out_ids_dev, float *out_scores_dev, void *stream);

/*
 * Same search with per-query parameters (device arrays of Q int32 each):
 *   W_q_dev in [1, W_max], L_q_dev in [1, L_max], iters_q_dev in [0, max_iters_max]
 *   (0 = until converged; allowed only when max_iters_max = 0).
 * W_max, L_max, max_iters_max are the bounds the workspace was sized with; values outside
 * them are clamped on the device.
 */
int ann_search_ragged(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q,
                      const int32_t *entry_dev, int32_t E, const int32_t *W_q_dev,
                      const int32_t *L_q_dev, const int32_t *iters_q_dev, int32_t W_max,
                      int32_t L_max, int32_t k, int32_t max_iters_max, void *workspace_dev,
                      size_t workspace_bytes, int32_t *out_ids_dev, float *out_scores_dev,
                      void *stream);

/*
 * Search down a hierarchy of nested graphs (Sec. 3.2: the search runs layer by layer through
 * the HNSW structure, the items selected in one layer being the seeds of the next; the outer
 * loop of Algorithm 1).
 *   graphs    : host array of n_layers handles, coarsest first, finest (base) last.  Layer l
 *               holds the items 0 .. N_l - 1 of ONE embedding table (the same emb_dev, d and
 *               dtype in every handle, N_0 <= N_1 <= ...), so an id means the same item in
 *               every layer that has it
 *   entry_dev : [Q][E] seeds of the coarsest layer (ids >= N_0 are ignored there)
 *   W_l, L_l  : host arrays [n_layers]: expansion width and eligible ranks per layer
 *   K_l       : host array [n_layers]: results taken from layer l; K_l[l] of them seed layer
 *               l + 1 (all of them, in rank order), K_l[n_layers - 1] = k are the output
 *   max_iters : rounds per query and layer, 0 = until converged
 * Each layer is one ann_search with the previous layer's result list as entry points; nothing
 * else is carried over (a finer layer scores its seeds again: the visited set is per layer).
 * out_ids_dev [Q][k], out_scores_dev [Q][k] as for ann_search.  Counters read by
 * ann_search_stats are summed over the layers (max_query_iters: the maximum).
 * Workspace: ann_search_layers_workspace_bytes with the same arguments; 0 on invalid ones.
 */
size_t ann_search_layers_workspace_bytes(const ann_graph *const *graphs, int32_t n_layers,
                                         const ann_mlp *m, int32_t Q, int32_t E,
                                         const int32_t *W_l, const int32_t *L_l,
                                         const int32_t *K_l, int32_t max_iters);
int ann_search_layers(const ann_graph *const *graphs, int32_t n_layers, const ann_mlp *m,
                      const void *queries_dev, int32_t Q, const int32_t *entry_dev, int32_t E,
                      const int32_t *W_l, const int32_t *L_l, const int32_t *K_l,
                      int32_t max_iters, void *workspace_dev, size_t workspace_bytes,
                      int32_t *out_ids_dev, float *out_scores_dev, void *stream);

/*
 * Paper-literal inter-candidate search (Algorithm 1 read as independent search processes that
 * share one result container; Sec. 3.2), for comparison with the joint best-first rule of
 * ann_search.  One walker per distinct in-range seed (E <= 1024 and E * R <= 4096).  Per hop every live
 * walker scores the neighbours of its position that no walker of the query has scored before
 * (walkers in seed order, first occurrence wins; all walkers read their neighbours before any
 * moves) and moves to the best of its own newly scored neighbours (score descending, id
 * ascending); a walker without one stops.  After T >= 1 hops, or when every walker has
 * stopped, the k best of everything scored are returned, padded with (-1, -inf).
 * The call only enqueues work.  Counters as for ann_search (nodes_expanded counts walker
 * positions expanded).  Workspace: ann_search_walkers_workspace_bytes (0 on invalid arguments).
 */
size_t ann_search_walkers_workspace_bytes(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t E,
                                          int32_t T, int32_t k);
int ann_search_walkers(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q,
                       const int32_t *entry_dev, int32_t E, int32_t T, int32_t k,
                       void *workspace_dev, size_t workspace_bytes, int32_t *out_ids_dev,
                       float *out_scores_dev, void *stream);

/*
 * Continuous batching (Sec. 3.2, Q-HiPANNS and Algorithm 2: requests of different users arrive
 * and finish at different times and are aggregated into common batches).  Q_total queries are
 * served by `slots` search states: a query enters the first state that becomes free, in index
 * order, and leaves it when it has converged (or reached max_iters rounds), so every scoring
 * batch is filled by the queries that are running at that moment instead of thinning out while
 * the slowest query of a fixed batch finishes.  The result of every query is the one ann_search
 * gives for it (queries do not influence each other; only the grouping of pairs into scoring
 * batches differs, and a pair's relevance does not depend on that).
 *   queries_dev [Q_total][d_user], entry_dev [Q_total][E], out_ids_dev / out_scores_dev [Q_total][k]
 *   slots     : >= 1; more slots than queries leaves the surplus idle
 *   max_iters : rounds per query, 0 = until converged
 * The call follows the device's progress as ann_search with max_iters = 0 does (it has to learn
 * when the last query is done) and waits on `stream` at the end.
 * Workspace: ann_search_stream_workspace_bytes with the same arguments (0 on invalid ones); its
 * size grows with `slots`, plus 4 * first-hidden-width bytes per query.  ann_search_stats reads
 * the counters of all Q_total queries.
 */
size_t ann_search_stream_workspace_bytes(const ann_graph *g, const ann_mlp *m, int32_t Q_total,
                                         int32_t slots, int32_t E, int32_t W, int32_t L, int32_t k,
                                         int32_t max_iters);
int ann_search_stream(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q_total,
                      const int32_t *entry_dev, int32_t E, int32_t slots, int32_t W, int32_t L,
                      int32_t k, int32_t max_iters, void *workspace_dev, size_t workspace_bytes,
                      int32_t *out_ids_dev, float *out_scores_dev, void *stream);

/*
 * Open stream: continuous batching for queries that ARRIVE WHILE others are being searched (Sec. 3.2, Q-HiPANNS:
 * the scorer keeps listening for requests; Algorithm 2 batches whatever has arrived).  The caller owns four
 * device arrays of `capacity` rows (queries_dev [capacity][d_user], entry_dev [capacity][E], out_ids_dev and
 * out_scores_dev [capacity][k]); query number i of the stream's life lives in row i, and its result is written
 * to row i when it has converged (or reached max_iters rounds).  `slots` search states serve them as in
 * ann_search_stream, whose workspace size (with Q_total = capacity) applies.  All work goes to `stream`.
 *   ann_stream_submit : the next n rows of queries_dev / entry_dev are valid (written on `stream` before the
 *                       call, or otherwise complete); the queries join the search at the next round.  Only
 *                       enqueues two small kernels; may be called from another host thread than the one that
 *                       drives the rounds.  ANN_EINVAL beyond `capacity` (a stream does not reuse rows).
 *   ann_stream_step   : enqueues `rounds` rounds (admission of waiting queries into free states, packing,
 *                       scoring, list update) without looking at the device.
 *   ann_stream_drain  : enqueues rounds until every query submitted so far has its result, following the
 *                       device's progress as ann_search does, then waits on `stream`; queries submitted by
 *                       another thread meanwhile are served too.  ANN_EWORKSPACE / ANN_EDEVICE as ann_search.
 *   ann_stream_close  : waits on `stream` and frees the handle (the arrays and the workspace are the caller's).
 * The result of every query is the one ann_search gives for it, whenever it arrived.
 */
typedef struct ann_stream ann_stream; /* opaque */
int ann_stream_open(const ann_graph *g, const ann_mlp *m, int32_t capacity, int32_t slots, int32_t E, int32_t W,
                    int32_t L, int32_t k, int32_t max_iters, const void *queries_dev, const int32_t *entry_dev,
                    int32_t *out_ids_dev, float *out_scores_dev, void *workspace_dev, size_t workspace_bytes,
                    void *stream, ann_stream **out);
int ann_stream_submit(ann_stream *s, int32_t n);
int ann_stream_step(ann_stream *s, int32_t rounds);
int ann_stream_drain(ann_stream *s);
int ann_stream_close(ann_stream *s);

/*
 * Serendipity vector of the metric input (Eq. 5: the user half of the input is h_u + h~ with
 * h~ ~ N(0, I)): out_dev[q][c] = users_dev[q][c] + sigma * z(seed, draw, q * d + c), for the
 * caller to pass as `queries_dev` of a search.  sigma = 1 is the paper's distribution, 0 copies.
 * z is a pure function of its arguments (so the same vectors can be drawn again, anywhere):
 * Philox4x32-10 with counter (e / 4, draw) and key seed, uniforms (x + 1/2) / 2^32, Box-Muller on
 * the word pairs (0,1) and (2,3) with the cosine on the even element; the sum is formed in fp64 and
 * rounded to fp32 (then to bf16 or fp16, nearest even, for ANN_BF16 / ANN_F16).  `draw` tells independent draws with
 * one seed apart (one per batch of requests, say).
 *   users_dev, out_dev : [Q][d] device arrays of `dtype` (ANN_F32 / ANN_BF16 / ANN_F16); may be the same array
 * Only enqueues one kernel on `stream`; ANN_EINVAL on bad arguments (Q < 0, d < 1, negative or
 * non-finite sigma, null arrays with Q > 0).
 */
int ann_users_add_noise(const void *users_dev, void *out_dev, int32_t Q, int32_t d, int32_t dtype,
                        double sigma, uint64_t seed, uint64_t draw, void *stream);

/*
 * The 8-bit metric (Sec. 4.3's quantised deployment taken below 16 bits; e4m3 = the OCP 8-bit float
 * with 4 exponent and 3 mantissa bits, largest value 448, no infinities).
 * dtype = ANN_F8 means: the item table holds e4m3 bytes, [N][d] (ann_graph_load); users stay bf16;
 * ann_mlp_load takes bf16 weights as for ANN_BF16 and stores every matrix as e4m3(4 w) (the user
 * half of the first layer stays bf16 and is applied in fp32, once per query); products are
 * accumulated in fp32; the activations of hidden layer l are clamped to [0, 448 / 4^l] and rounded
 * to e4m3 at scale 4^l (nearest even); logits, sigmoid and the weighted sum are fp32.
 * Built for two shapes: 64-wide items with hidden widths 256 and 128, 128-wide items with hidden
 * widths 512 and 256, up to 8 heads (else ANN_ENOTIMPL);
 * ANN_EINVAL if a weight times 4 exceeds 448.
 *
 * ann_quantize_e4m3 makes such an item table: dst_dev[i] = e4m3(scale * src_dev[i]) (nearest even,
 * magnitudes above 448 clamped), src_dev of src_dtype ANN_F32 / ANN_BF16, n elements; the metric
 * above assumes scale = 1.  Only enqueues one kernel on `stream`.
 */
int ann_quantize_e4m3(const void *src_dev, int32_t src_dtype, int64_t n, float scale, uint8_t *dst_dev,
                      void *stream);

/*
 * Relevance (Eq. 5-8) of an explicit list of M pairs: out_dev[r] = relevance(user q_idx[r],
 * item item[r]).  q_idx_dev, item_dev: [M] int32; out_dev: [M] fp32.  Pairs whose indices
 * are out of range get NaN.  Uses the same kernels as the search.  `tile_rows` (0 = default)
 * sets how many pairs one batch of Algorithm 2 holds; results do not depend on it.
 * The call allocates and frees a small temporary on `stream`'s device and synchronises.
 */
int ann_score_pairs(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q,
                    int64_t M, const int32_t *q_idx_dev, const int32_t *item_dev, float *out_dev,
                    int32_t tile_rows, void *stream);

/*
 * Exhaustive search: the k most relevant items of the whole table for every query, under the same
 * relevance (Eq. 5-8) and the same scoring kernels the graph search uses: the ground truth that the recall
 * measure (Sec. 5.1.3) compares a search with, at the metric's own precision.
 * queries_dev: [Q][d_user]; out_ids_dev: [Q][k] int32, out_scores_dev: [Q][k] fp32, device memory, written.
 * Order: relevance descending, equal relevances by ascending id (the order of the search's results);
 * with k above the number of items the row ends with id -1 / relevance -inf.  1 <= k <= 2,048.
 * Cost: Q x N relevance scores (the adjacency of `g` is not used).
 * workspace_dev: device memory of at least ann_brute_force_workspace_bytes(g, m, Q, k) bytes (about 200 MB +
 * Q x k x 8 bytes + the per-query user terms), 256-byte aligned; the call then only enqueues kernels on `stream`
 * and the outputs are valid once they have run.  NULL: the call allocates and frees that temporary itself and
 * synchronises `stream`.
 * ANN_EINVAL for a null handle or pointer, a metric that does not match the graph, Q < 1, k out of range;
 * ANN_EWORKSPACE for a workspace that is too small; ANN_ENOMEM if the temporary cannot be allocated.
 * ann_brute_force_workspace_bytes returns 0 for arguments the call would refuse.
 */
size_t ann_brute_force_workspace_bytes(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t k);
int ann_brute_force(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q, int32_t k,
                    int32_t *out_ids_dev, float *out_scores_dev, void *workspace_dev, size_t workspace_bytes,
                    void *stream);

/*
 * Re-ranking: the k most relevant of each query's n candidate items under this metric.  Meant for the lists a
 * search returned under a cheaper metric (the 8-bit one of Sec. 4.3's quantised deployment): the traversal runs
 * in 8 bits, its best n candidates are scored once more in 16 bits, and the order of the result is the 16-bit
 * metric's.  The re-ranking itself is not in the paper; the relevance is Eq. 5-8, by the search's kernels.
 * cand_dev: [Q][n] int32 item ids, device memory, read only; entries outside [0, N) (the -1 padding of a search
 * result) are no candidates; an id that occurs several times is returned as often.  1 <= n <= 65,536.
 * Result as ann_brute_force: [Q][k], relevance descending, equal relevances by ascending id, -1 / -inf where
 * a query has fewer than k candidates.  1 <= k <= 2,048.
 * workspace_dev / workspace_bytes as for ann_brute_force, sized by ann_rerank_workspace_bytes(g, m, Q, n, k)
 * (8 bytes per candidate of a pass of at most 2^24 pairs, + Q x k x 8 + the per-query user terms); NULL = allocate,
 * free and synchronise.  Errors as ann_brute_force; ANN_EINVAL also for a null cand_dev or n out of range.
 */
size_t ann_rerank_workspace_bytes(const ann_graph *g, const ann_mlp *m, int32_t Q, int32_t n, int32_t k);
int ann_rerank(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q, const int32_t *cand_dev,
               int32_t n, int32_t k, int32_t *out_ids_dev, float *out_scores_dev, void *workspace_dev,
               size_t workspace_bytes, void *stream);

/*
 * ann_score_pairs for callers that cannot allocate device memory: code whose stream is being recorded
 * into a HIP graph, tight serving loops, harnesses that forbid allocation.  Same arguments and result as
 * ann_score_pairs (default batch size); the call makes no allocation of any kind and does not
 * synchronise: it only enqueues kernels on `stream`, and out_dev is valid once they have run.
 * What ann_score_pairs keeps in a temporary (the pair count the kernels read, the per-query user term of
 * the first layer, Q x first-hidden-width fp32) lives in a fixed array inside the library, 8 MiB + 384 bytes,
 * one copy on every GPU the library runs on, held until the process ends.
 * Limits: Q * first hidden width <= 2^21 (ANN_EINVAL beyond, with the reason in ann_last_error); the
 * metric's device must be the current device.
 * Every call on a GPU uses that GPU's one array: calls on the same stream follow each other and are safe;
 * calls that may overlap in time on one GPU (different streams, different host threads) race and give
 * wrong scores.  The array keeps the last call's contents; nothing in it needs clearing between calls.
 */
int ann_score_pairs_noalloc(const ann_graph *g, const ann_mlp *m, const void *queries_dev, int32_t Q,
                            int64_t M, const int32_t *q_idx_dev, const int32_t *item_dev, float *out_dev,
                            void *stream);

/*
 * Searches that run until every query has converged (ann_search / ann_search_layers with max_iters = 0,
 * ann_search_stream) follow the progress word their kernels store to pinned host memory every round.  This sets,
 * for the whole process, how long such a call waits for the NEXT report while `stream` stays busy before it gives
 * up with ANN_EDEVICE (default 600 s, 0 = wait for ever).  The limit counts from the last report seen, so work
 * the caller enqueued on the stream ahead of the search must finish within it too.  A call that gives up has
 * enqueued only complete rounds; its kernels end by themselves, nothing is left waiting on the device, and the
 * results are undefined.  While it waits the calling thread yields the core between looks at the word.
 */
int ann_set_progress_timeout(double seconds);

/* Waits for `stream`, then copies the counters of the last search run on workspace_dev. */
int ann_search_stats(const void *workspace_dev, ann_stats *out_host, void *stream);

/*
 * Stage timing for measurement runs.  While enabled on the calling host thread, ann_search and
 * ann_search_ragged bracket every kernel launch with two HIP events recorded on the search's
 * stream.  Stages: ANN_STAGE_SCORE = the MLP relevance kernel (Sec. 3.1), ANN_STAGE_ROUND =
 * seeding and the per-query round kernel (merge, choice of parents, neighbour gather, visited
 * filter; Algorithm 1), ANN_STAGE_PACK = prefix sum + packing of the ragged groups (Algorithm 2).
 * ann_profile_read waits for the recorded events, writes per stage the summed elapsed
 * milliseconds and the number of launches since the last read (arrays of ANN_STAGE_COUNT),
 * and forgets them.  Event pairs are created on demand and kept until the process ends.
 */
enum { ANN_STAGE_SCORE = 0, ANN_STAGE_ROUND = 1, ANN_STAGE_PACK = 2, ANN_STAGE_COUNT = 3 };
int ann_profile_enable(int on);
int ann_profile_read(double *ms_out, int64_t *launches_out);

/*
 * Plain device-to-device copy of `bytes` bytes (a multiple of 16, both pointers 16-byte aligned) by
 * a grid-stride kernel, enqueued on `stream`.  It exists for measurement only: it reads and writes
 * exactly `bytes` bytes of HBM, which gives hardware traffic counters (rocprofv3 FETCH_SIZE /
 * WRITE_SIZE) a reference of known size in the same run as the search kernels.
 */
int ann_profile_copy(void *dst_dev, const void *src_dev, size_t bytes, void *stream);

const char *ann_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* GMPGR_ANN_H */
