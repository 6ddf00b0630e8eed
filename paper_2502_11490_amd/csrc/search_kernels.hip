// Per-query search state machine of the joint best-first search (Sec. 3.2, Algorithm 1)
// and the packing of ragged survivor groups into one dense pair list (Algorithm 2).
//
// One workgroup owns one query in every kernel here: its sorted candidate list (the shared
// container of Algorithm 1), its exact visited table and its survivors of the current round.
// Per round:   scan_compact -> (MLP kernel) -> round
//   round       : merge the scores of the previous round into the list, test termination,
//                 pick <= W unexpanded entries among the first L ranks, read their adjacency
//                 rows, drop out-of-range / repeated / already scored ids, keep the rest as
//                 this query's survivors
//   scan_compact: exclusive prefix sum of the survivor counts over all queries and a stable
//                 copy of every group into the dense pair list (query-major, first-found
//                 first), which the MLP kernel cuts into fixed-size batches
#include "common.h"
#include "keys.h"

namespace gmpgr {

// Threads per query in the per-query kernels (seeding, round, output).
#ifndef QUERY_BLOCK
#define QUERY_BLOCK 256
#endif
constexpr int BLOCK = QUERY_BLOCK;     // largest workgroup of the per-query kernels (launch bound, LDS sizing)
constexpr int WAVES = BLOCK / 64;
// The functions below are templates over the workgroup size BLK: the round kernel is also built for
// half-size workgroups (see launch_round).
#ifndef ROUND_BIG_FROM
#define ROUND_BIG_FROM 512   // candidates per query and round above which the round kernel runs larger workgroups
#endif
#ifndef FILTER_CHUNK
#define FILTER_CHUNK 1024   // candidates of a round that pass the visited filter together
#endif
#ifndef ROUND_TILE_MAX
#define ROUND_TILE_MAX 4096   // most list entries held in LDS at a time during the merge
#endif
#ifndef ROUND_WAVES_MIN
#define ROUND_WAVES_MIN 8     // waves per SIMD the round kernel is compiled for (8: at most 64 registers per lane)
#endif
#ifndef ROUND_BIG_BLOCK
#define ROUND_BIG_BLOCK 512
#endif
constexpr int SCAN_BLOCK = 256;
constexpr int SCAN_WAVES = SCAN_BLOCK / 64;

// Phase timing of the round kernel for measurement builds (-DROUND_TIMING): thread 0 of every
// 64th workgroup adds the shader-clock ticks of each phase to counters 8..15 of the stats block
// (every workgroup doing so would serialise on those few addresses and distort what is measured).
#ifdef ROUND_TIMING
#define PHASE_MARK(k)                                                                          \
    do {                                                                                       \
        if (threadIdx.x == 0 && (blockIdx.x & 63) == 0) {                                      \
            long long now_ = clock64();                                                        \
            atomicAdd((unsigned long long *)&stats[8 + (k)], (unsigned long long)(now_ - t_)); \
            t_ = now_;                                                                         \
        }                                                                                      \
    } while (0)
#define PHASE_START long long t_ = clock64();
#else
#define PHASE_MARK(k)
#define PHASE_START
#endif

__device__ __forceinline__ uint32_t hash_id(uint32_t id) { return id * 0x9E3779B1u; }

// Exclusive prefix count of `flag` over the workgroup in thread order; *total = block sum.
// wave_sums: LDS int[WAVES + 1].  Contains two barriers.
template <int BLK>
__device__ __forceinline__ int block_excl_count(bool flag, int *wave_sums, int *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long b = __ballot(flag);
    int excl = __popcll(b & ((1ull << lane) - 1ull));
    if (lane == 0) wave_sums[wave] = __popcll(b);
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < (BLK >> 6); ++w) {
        int c = wave_sums[w];
        if (w < wave) base += c;
        tot += c;
    }
    __syncthreads();
    *total = tot;
    return base + excl;
}

// Sorts keys[0..m), 1 <= m <= BLK, ascending, by counting: the keys are distinct, so the rank of a key is the
// number of smaller ones.  The count for key j is shared by BLK / m_pad threads (m_pad: m rounded up to a power
// of two), each over its share of the keys, which a wave reads as LDS broadcasts, one after the other without
// waiting; the shares meet in an LDS counter.  Three barriers and m * m_pad / BLK independent reads per
// thread, where the bitonic network makes log2(m)^2 / 2 dependent trips to the LDS with most threads idle.
//   cnt : LDS uint32[m_pad], any contents.   All threads of the workgroup call; ends with a barrier.
template <int BLK>
__device__ void rank_sort(uint64_t *keys, int m, uint32_t *cnt) {
    int shift = 0;
    while ((1 << shift) < m) ++shift;
    const int m_pad = 1 << shift, groups = BLK >> shift;
    const int j = threadIdx.x & (m_pad - 1), part = threadIdx.x >> shift;
    if ((int)threadIdx.x < m_pad) cnt[threadIdx.x] = 0;
    __syncthreads();  // the keys are all written, the counters are zero
    const uint64_t key = j < m ? keys[j] : 0;
    const int per = (m + groups - 1) / groups;
    const int i0 = part * per, i1 = min(m, i0 + per);
    uint32_t smaller = 0;
    for (int i = i0; i < i1; ++i) smaller += keys[i] < key ? 1u : 0u;
    if (j < m && smaller) atomicAdd(&cnt[j], smaller);
    __syncthreads();  // every count is complete and nobody reads the unsorted keys any more
    if (part == 0 && j < m) keys[cnt[j]] = key;
    __syncthreads();
}

// Drops ids that are out of range, repeated inside cand[0..n_cand) (first occurrence kept)
// or already in this query's visited table; inserts the rest into the table and writes them,
// in their order of occurrence, to out[0..n_new).  Returns n_new (same in every thread).
//   cand          : LDS int32[n_cand]
//   dd_key/dd_pos : LDS uint32[dd_n] each, dd_n a power of two >= 2 * n_cand (dedupe by id)
//   bk_key/bk_cnt : LDS uint32[dd_n] each (arrivals per bucket in this pass)
//   out_tag       : global uint16[n_new]: (tag_base + candidate position) / tag_div of every survivor
//   table         : global uint32[hash_cap]: hash_cap/16 buckets of 16 slots (one 64-byte line);
//                   a bucket is filled from slot 0 up, EMPTY_SLOT = free.  An id lives in its home
//                   bucket or, if that one is full, in the next ones up to the first bucket that
//                   is not full.  The caller guarantees n_visited + n_cand <= hash_cap / 2.
//
// The table of a query is touched by one workgroup only, so it needs no global atomics (they
// cost three times a plain access here): every candidate reads its whole bucket once (one line),
// decides "seen / room / full" from that snapshot, and the candidates that arrive at the same
// bucket in the same pass take consecutive free slots by a rank drawn from an LDS counter.
// Stores of a pass become visible to the next pass through a workgroup-scope fence + barrier.
template <int BLK>
__device__ int filter_and_insert(const int32_t *cand, int n_cand, uint32_t *dd_key, uint32_t *dd_pos,
                                 uint32_t *bk_key, uint32_t *bk_cnt, int dd_n, uint32_t *table, int hash_cap,
                                 int64_t N, int32_t *out, int *wave_sums, uint16_t *out_tag, int tag_div,
                                 int tag_base = 0) {
    const int n_buckets = hash_cap >> 4;
    const uint32_t bmask = (uint32_t)n_buckets - 1u;
    const int bshift = 32 - (31 - __clz(n_buckets));  // n_buckets = 2^b (b >= 2) -> top b bits
    for (int i = threadIdx.x; i < dd_n; i += BLK) {
        dd_key[i] = EMPTY_SLOT;
        dd_pos[i] = 0xFFFFFFFFu;
    }
    __syncthreads();
    const uint32_t dd_mask = (uint32_t)dd_n - 1u;
    // pass 1: smallest position of every distinct id
    for (int p = threadIdx.x; p < n_cand; p += BLK) {
        int32_t v = cand[p];
        if (v < 0 || (int64_t)v >= N) continue;
        uint32_t s = hash_id((uint32_t)v) & dd_mask;
        for (;;) {
            uint32_t old = atomicCAS(&dd_key[s], EMPTY_SLOT, (uint32_t)v);
            if (old == EMPTY_SLOT || old == (uint32_t)v) {
                atomicMin(&dd_pos[s], (uint32_t)p);
                break;
            }
            s = (s + 1u) & dd_mask;
        }
    }
    __syncthreads();
    // pass 2: first occurrences look themselves up in the visited table and enter it if absent
    int n_new = 0;
    for (int p0 = 0; p0 < n_cand; p0 += BLK) {
        const int p = p0 + threadIdx.x;
        bool fresh = false, active = false;
        int32_t v = -1;
        uint32_t bkt = 0;
        if (p < n_cand) {
            v = cand[p];
            if (v >= 0 && (int64_t)v < N) {
                uint32_t s = hash_id((uint32_t)v) & dd_mask;
                while (dd_key[s] != (uint32_t)v) s = (s + 1u) & dd_mask;
                active = (dd_pos[s] == (uint32_t)p);
                bkt = hash_id((uint32_t)v) >> bshift;
            }
        }
        for (;;) {
            for (int i = threadIdx.x; i < dd_n; i += BLK) {
                bk_key[i] = EMPTY_SLOT;
                bk_cnt[i] = 0u;
            }
            // snapshot of the bucket: every read of this pass completes before any store of it
            bool found = false;
            int cnt = 0;
            if (active) {
                // (Requesting the home buckets before the dedupe, so that the lines travel meanwhile, keeps 16
                // registers busy across it: in a kernel held to 64 they spill, which cost C4 a quarter of its time.)
                const uint4 *line = (const uint4 *)(table + (size_t)bkt * 16);
                const uint4 q0 = line[0], q1 = line[1], q2 = line[2], q3 = line[3];
                const uint32_t w[16] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w,
                                        q2.x, q2.y, q2.z, q2.w, q3.x, q3.y, q3.z, q3.w};
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    found |= (w[i] == (uint32_t)v);
                    cnt += (w[i] != EMPTY_SLOT);
                }
            }
            __syncthreads();
            if (active) {
                if (found) {
                    active = false;  // scored in an earlier round
                } else if (cnt == 16) {
                    bkt = (bkt + 1u) & bmask;  // full: the id can only be further on
                } else {
                    uint32_t s = hash_id(bkt) & dd_mask;
                    for (;;) {
                        uint32_t old = atomicCAS(&bk_key[s], EMPTY_SLOT, bkt);
                        if (old == EMPTY_SLOT || old == bkt) break;
                        s = (s + 1u) & dd_mask;
                    }
                    const int slot = cnt + (int)atomicAdd(&bk_cnt[s], 1u);
                    if (slot < 16) {
                        table[(size_t)bkt * 16 + slot] = (uint32_t)v;
                        fresh = true;
                        active = false;
                    } else {
                        bkt = (bkt + 1u) & bmask;  // filled up by this pass: try the next bucket
                    }
                }
            }
            const bool more = (p0 + BLK < n_cand);
            if (!__syncthreads_or(active ? 1 : 0)) {
                if (more) {
                    __threadfence_block();
                    __syncthreads();
                }
                break;
            }
            // This pass's stores must be seen by the next pass's bucket reads.  A table belongs to one workgroup,
            // whose waves share a compute unit and its vector cache: workgroup scope is enough, and a device-scope
            // fence would write the whole L2 slice back.
            __threadfence_block();
            __syncthreads();
        }
        int tot;
        int pos = block_excl_count<BLK>(fresh, wave_sums, &tot);
        if (fresh) {
            out[n_new + pos] = v;
            out_tag[n_new + pos] = (uint16_t)((tag_base + p) / tag_div);  // the parent (or seed) it came from
        }
        n_new += tot;
    }
    return n_new;
}

// The same filter over a bitmap of the item ids (one bit per item, N / 8 bytes per query) instead of the hash
// table: chosen where the bitmap is the smaller of the two (long lists on a moderate item count), because the
// probes of all queries then fall into a much smaller address range and seeding has much less to clear.
//   bits : global uint32[ceil(N / 32) rounded up to 64 words], all zero at the start of a search
// Every first occurrence reads its word (4 bytes); the ones whose bit is clear are new.  New ids that share a
// word meet in an LDS table keyed by the word index, OR their bits together there, and the one that opened the
// entry stores word | bits: plain loads and stores, the bitmap belongs to this workgroup alone.
//   cand_rank : LDS int32[n_cand] or nullptr: the bit that stands for candidate p is cand_rank[p] instead of its id
//               (a permutation of the ids chosen so that ids the graph joins lie in the same 64-byte lines)
template <int BLK>
__device__ int filter_and_mark(const int32_t *cand, const int32_t *cand_rank, int n_cand, uint32_t *dd_key,
                               uint32_t *dd_pos, uint32_t *bk_key, uint32_t *bk_cnt, int dd_n, uint32_t *bits, int64_t N,
                               int32_t *out, int *wave_sums, uint16_t *out_tag, int tag_div, int tag_base) {
    uint32_t pre = 0;  // the first BLK candidates request their word right away (nothing is stored before pass 2)
    if ((int)threadIdx.x < n_cand) {
        const int32_t v = cand[threadIdx.x];
        if (v >= 0 && (int64_t)v < N) pre = bits[(uint32_t)(cand_rank ? cand_rank[threadIdx.x] : v) >> 5];
    }
    for (int i = threadIdx.x; i < dd_n; i += BLK) {
        dd_key[i] = EMPTY_SLOT;
        dd_pos[i] = 0xFFFFFFFFu;
        bk_key[i] = EMPTY_SLOT;
        bk_cnt[i] = 0u;
    }
    __syncthreads();
    const uint32_t dd_mask = (uint32_t)dd_n - 1u;
    // pass 1: smallest position of every distinct id
    for (int p = threadIdx.x; p < n_cand; p += BLK) {
        int32_t v = cand[p];
        if (v < 0 || (int64_t)v >= N) continue;
        uint32_t s = hash_id((uint32_t)v) & dd_mask;
        for (;;) {
            uint32_t old = atomicCAS(&dd_key[s], EMPTY_SLOT, (uint32_t)v);
            if (old == EMPTY_SLOT || old == (uint32_t)v) {
                atomicMin(&dd_pos[s], (uint32_t)p);
                break;
            }
            s = (s + 1u) & dd_mask;
        }
    }
    __syncthreads();
    // pass 2: first occurrences test their bit; the new ones set it
    int n_new = 0;
    for (int p0 = 0; p0 < n_cand; p0 += BLK) {
        const int p = p0 + threadIdx.x;
        bool fresh = false, owner = false;
        int32_t v = -1;
        uint32_t word = 0, old_word = 0, slot = 0, bit = 0;
        if (p < n_cand) {
            v = cand[p];
            if (v >= 0 && (int64_t)v < N) {
                uint32_t s = hash_id((uint32_t)v) & dd_mask;
                while (dd_key[s] != (uint32_t)v) s = (s + 1u) & dd_mask;
                if (dd_pos[s] == (uint32_t)p) {
                    bit = (uint32_t)(cand_rank ? cand_rank[p] : v);
                    word = bit >> 5;
                    old_word = (p0 == 0) ? pre : bits[word];
                    fresh = ((old_word >> (bit & 31)) & 1u) == 0u;
                }
            }
        }
        if (fresh) {
            slot = hash_id(word) & dd_mask;
            for (;;) {
                uint32_t old = atomicCAS(&bk_key[slot], EMPTY_SLOT, word);
                if (old == EMPTY_SLOT || old == word) {
                    owner = (old == EMPTY_SLOT);
                    break;
                }
                slot = (slot + 1u) & dd_mask;
            }
            atomicOr(&bk_cnt[slot], 1u << (bit & 31));
        }
        __syncthreads();  // every new bit of this pass has reached its LDS entry
        if (owner) bits[word] = old_word | bk_cnt[slot];
        int tot;
        const int pos = block_excl_count<BLK>(fresh, wave_sums, &tot);
        if (fresh) {
            out[n_new + pos] = v;
            out_tag[n_new + pos] = (uint16_t)((tag_base + p) / tag_div);
        }
        n_new += tot;
        if (p0 + BLK < n_cand) {
            // the words stored above must be seen by the next pass; its ids open fresh LDS entries
            for (int i = threadIdx.x; i < dd_n; i += BLK) {
                bk_key[i] = EMPTY_SLOT;
                bk_cnt[i] = 0u;
            }
            __threadfence_block();
            __syncthreads();
        }
    }
    return n_new;
}

// Either form of the visited set: table_cap > 0 = hash table of that many entries, table_cap < 0 = bitmap in a
// region of -table_cap words.
template <int BLK>
__device__ __forceinline__ int visited_filter(const int32_t *cand, const int32_t *cand_rank, int n_cand, uint32_t *dd_key,
                                              uint32_t *dd_pos, uint32_t *bk_key, uint32_t *bk_cnt, int dd_n,
                                              uint32_t *table, int table_cap, int64_t N, int32_t *out, int *wave_sums,
                                              uint16_t *out_tag, int tag_div, int tag_base) {
    if (table_cap < 0)
        return filter_and_mark<BLK>(cand, cand_rank, n_cand, dd_key, dd_pos, bk_key, bk_cnt, dd_n, table, N, out, wave_sums,
                                    out_tag, tag_div, tag_base);
    return filter_and_insert<BLK>(cand, n_cand, dd_key, dd_pos, bk_key, bk_cnt, dd_n, table, table_cap, N, out, wave_sums,
                                  out_tag, tag_div, tag_base);
}

// Counters and control block start at zero (a kernel, not a memset, so that a caller may
// capture the launch sequence into a HIP graph).
// stats[5], stats[6]: bytes of one adjacency row and of one item row, from which ann_search_stats derives the
// algorithmic bytes of the gather stages.
__global__ void zero_stats_kernel(int64_t *stats, Ctrl *ctrl, int Q, int keep_stats, int adj_row_bytes,
                                  int item_row_bytes) {
    if (threadIdx.x < 16 && !keep_stats)
        stats[threadIdx.x] = threadIdx.x == 4 ? Q : threadIdx.x == 5 ? adj_row_bytes : threadIdx.x == 6 ? item_row_bytes : 0;
    if (threadIdx.x < 16) ((int32_t *)ctrl)[threadIdx.x] = 0;
}

// ------------------------------------------------------------------------------------------
// Seeding: clear the visited table, keep the distinct in-range entry ids as the survivors of
// "round 0" (they are scored by the first MLP launch and merged by the first round kernel).
// `slot` names the search state that is set up, `query` the row of entries / per-query parameters.
template <int BLK>
__device__ void seed_slot(int slot, int query, const int32_t *__restrict__ entries, const int32_t *__restrict__ rank,
                          int E, int64_t N, QState *state, uint32_t *hash, int hash_cap, int32_t *cand_g, int slots,
                          int32_t *counts,
                          const int32_t *W_q, const int32_t *L_q, const int32_t *cap_q, int W, int L, int cap,
                          int W_max, int L_max, int cap_max, int64_t *stats, unsigned char *smem, uint16_t *tag_g) {
    int dd_n = 2;
    while (dd_n < 2 * E) dd_n <<= 1;
    int32_t *cand = (int32_t *)smem;                 // [E]
    int32_t *cand_rank = rank ? cand + ((E + 3) & ~3) : nullptr;   // [E] the seeds' places in the visited bitmap
    uint32_t *dd_key = (uint32_t *)(cand + (rank ? 2 : 1) * ((E + 3) & ~3));
    uint32_t *dd_pos = dd_key + dd_n;
    uint32_t *bk_key = dd_pos + dd_n;
    uint32_t *bk_cnt = bk_key + dd_n;
    int *wave_sums = (int *)(bk_cnt + dd_n);

    const int table_words = hash_cap < 0 ? -hash_cap : hash_cap;  // a multiple of 64, the table 256-byte aligned
    uint32_t *table = hash + (size_t)slot * table_words;
    {
        uint4 *t4 = (uint4 *)table;
        const uint32_t e = hash_cap < 0 ? 0u : EMPTY_SLOT;  // bitmap: no bit set; hash table: every slot free
        const uint4 e4 = make_uint4(e, e, e, e);
        for (int i = threadIdx.x; i < table_words / 4; i += BLK) t4[i] = e4;
    }
    for (int i = threadIdx.x; i < E; i += BLK) {
        const int32_t v = entries[(size_t)query * E + i];
        cand[i] = v;
        if (rank) cand_rank[i] = (v >= 0 && (int64_t)v < N) ? rank[v] : -1;
    }
    __threadfence_block();
    __syncthreads();
    int n = visited_filter<BLK>(cand, cand_rank, E, dd_key, dd_pos, bk_key, bk_cnt, dd_n, table, hash_cap, N,
                                cand_g + (size_t)slot * slots, wave_sums, tag_g + (size_t)slot * slots, 1, 0);
    if (threadIdx.x == 0) {
        QState s;
        s.t = 0;
        s.done = 0;
        s.n_list = 0;
        s.n_visited = n;
        int w = W_q ? W_q[query] : W, l = L_q ? L_q[query] : L, c = cap_q ? cap_q[query] : cap;
        s.W = min(max(w, 1), W_max);
        s.L = min(max(l, 1), L_max);
        s.cap = cap_max > 0 ? min(max(c, 1), cap_max) : max(c, 0);
        s.n_expanded = 0;
        s.first_open = 0;
        s.pad[0] = s.pad[1] = s.pad[2] = 0;
        state[slot] = s;
        counts[slot] = n;
    }
}

__global__ void __launch_bounds__(BLOCK)
init_kernel(const int32_t *__restrict__ entries, const int32_t *__restrict__ rank, int E, int64_t N, QState *state,
            uint32_t *hash,
            int hash_cap, int32_t *cand_g, int slots, int32_t *counts, const int32_t *W_q,
            const int32_t *L_q, const int32_t *cap_q, int W, int L, int cap, int W_max, int L_max,
            int cap_max, int64_t *stats, uint16_t *tag_g) {
    extern __shared__ __align__(16) unsigned char smem[];
    seed_slot<BLOCK>(blockIdx.x, blockIdx.x, entries, rank, E, N, state, hash, hash_cap, cand_g, slots, counts, W_q, L_q, cap_q, W,
              L, cap, W_max, L_max, cap_max, stats, smem, tag_g);
}

// A query's counters join the totals once, when its result is written: every workgroup adding to the
// same few words in every round made those additions, which the memory side performs one after the
// other (about 10 ns each), the longest part of a round.  One lane calls this with sums over a
// group of queries.
__device__ __forceinline__ void add_to_totals(int64_t *stats, long long scored, long long expanded, int rounds,
                                              int overflowed) {
    atomicAdd((unsigned long long *)&stats[0], (unsigned long long)scored);
    atomicAdd((unsigned long long *)&stats[1], (unsigned long long)expanded);
    atomicMax((unsigned long long *)&stats[2], (unsigned long long)rounds);
    if (overflowed) atomicAdd((unsigned long long *)&stats[3], (unsigned long long)overflowed);
}

// First k entries of a slot's list to row `row` of the outputs, padded with (-1, -inf).
template <int BLK>
__device__ void emit_row(const QState *state, const uint64_t *pool_g, int C, int k, int slot, int64_t row,
                         int32_t *out_ids, float *out_scores) {
    const int n = state[slot].n_list;
    const uint64_t *pool = pool_g + (size_t)slot * C;
    for (int i = threadIdx.x; i < k; i += BLK) {
        int32_t id = -1;
        float sc = -INFINITY;
        if (i < n) {
            uint64_t key = pool[i];
            id = key_id(key);
            sc = key_score(key);
        }
        out_ids[(size_t)row * k + i] = id;
        out_scores[(size_t)row * k + i] = sc;
    }
}

// ------------------------------------------------------------------------------------------
// Continuous batching (Sec. 3.2, Q-HiPANNS: requests arrive and finish at different times and are
// aggregated into common batches).  The search state lives in slots; a slot whose query has
// finished writes that query's result and takes the next waiting query, in index order (a
// counter is the queue).  Runs before the packing step of every round.
__global__ void stream_reset_kernel(int64_t *stats, Ctrl *ctrl, QState *state, int32_t *counts, int32_t *slot_query,
                                    int S, int Q_total, int adj_row_bytes, int item_row_bytes) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 16) {
        stats[i] = i == 4 ? max(Q_total, 0) : i == 5 ? adj_row_bytes : i == 6 ? item_row_bytes : 0;
        ((int32_t *)ctrl)[i] = 0;
    }
    if (i < S) {
        QState s = {};
        s.done = 1;
        state[i] = s;
        counts[i] = -1;
        slot_query[i] = -1;
    }
}

// Open stream: queries [0, avail) have arrived (their rows in the query, entry and user-term arrays are valid).
// A kernel, so that the word changes in stream order behind the work that made the rows valid.
__global__ void stream_publish_kernel(Ctrl *ctrl, int64_t *stats, int avail) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        ctrl->avail = avail;
        stats[4] = avail;
    }
}

__global__ void __launch_bounds__(BLOCK)
admit_kernel(const int32_t *__restrict__ entries, const int32_t *__restrict__ rank, int E, int64_t N, QState *state,
             uint32_t *hash, int hash_cap,
             int32_t *cand_g, int slots, int32_t *counts, const int32_t *W_q, const int32_t *L_q,
             const int32_t *cap_q, int W, int L, int cap, int W_max, int L_max, int cap_max, int64_t *stats,
             Ctrl *ctrl, int32_t *slot_query, int Q_total, const uint64_t *pool_g, int C, int k, int32_t *out_ids,
             float *out_scores, uint16_t *tag_g) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int next_s;
    const int slot = blockIdx.x;
    if (!state[slot].done) return;  // still searching
    const int served = slot_query[slot];
    if (served >= 0) {
        emit_row<BLOCK>(state, pool_g, C, k, slot, served, out_ids, out_scores);
        if (threadIdx.x == 0) {
            const QState st = state[slot];
            add_to_totals(stats, st.n_visited, st.n_expanded, st.t, (st.done & 2) ? 1 : 0);
        }
    }
    __syncthreads();  // every wave has read which query the slot served before thread 0 names the next one
    if (threadIdx.x == 0) {
        int next;
        if (Q_total >= 0) {
            next = Q_total;
            // the counter only grows; once it has passed the total nobody needs to touch it again
            if (*(volatile int32_t *)&ctrl->next_query < Q_total) next = atomicAdd(&ctrl->next_query, 1);
            next = next < Q_total ? next : -1;
        } else {
            // open stream: the number of queries that have arrived (ctrl->avail) grows while the search runs, so
            // the counter must never pass it: a query index claimed before its query exists would be lost
            const int avail = *(volatile int32_t *)&ctrl->avail;
            int cur = *(volatile int32_t *)&ctrl->next_query;
            next = -1;
            while (cur < avail) {
                const int seen = atomicCAS(&ctrl->next_query, cur, cur + 1);
                if (seen == cur) {
                    next = cur;
                    break;
                }
                cur = seen;
            }
        }
        next_s = next;
        slot_query[slot] = next_s;
        if (next_s < 0) counts[slot] = -1;  // idle: contributes no pairs, is not counted as running
    }
    __syncthreads();  // also: the list of the served query has been read before the slot is re-seeded
    const int next = next_s;
    if (next < 0) return;
    seed_slot<BLOCK>(slot, next, entries, rank, E, N, state, hash, hash_cap, cand_g, slots, counts, W_q, L_q, cap_q, W, L, cap,
              W_max, L_max, cap_max, stats, smem, tag_g);
}

// ------------------------------------------------------------------------------------------
// Exclusive scan of survivor counts + stable packing into the dense pair list (Algorithm 2).
// A workgroup owns SCAN_QPB consecutive queries (4 or 8: few, so that many workgroups share the
// copying).  It first sums the counts of all earlier queries (every workgroup re-reads them from
// L2: O(Q^2 / SCAN_QPB) four-byte reads in total, no waiting on other workgroups, the same result
// every run), then scans its own counts and copies its groups, one wave per query at a time.
template <int SCAN_QPB>  // queries per workgroup, a multiple of 4
__global__ void __launch_bounds__(SCAN_BLOCK)
scan_compact_kernel(const int32_t *__restrict__ counts, int Q, const int32_t *__restrict__ cand_g, int slots,
                    int32_t *offsets, int32_t *pair_q, int32_t *pair_id, Ctrl *ctrl,
                    const int32_t *__restrict__ slot_query, uint64_t *mailbox, uint64_t mail_word, int Q_total) {
    __shared__ int red[SCAN_WAVES];
    __shared__ int red_active[SCAN_WAVES];
    __shared__ int loc_off[SCAN_QPB + 1];
    __shared__ int loc_cnt[SCAN_QPB];
    const int q0 = blockIdx.x * SCAN_QPB;
    const bool last = (blockIdx.x == gridDim.x - 1);
    // pairs of all earlier queries (and, in the last workgroup, the number of running queries)
    int sum = 0, act = 0;
    const int lim = last ? Q : q0;
    // q0 is a multiple of 4 and the array is 256-byte aligned: four counts per load up to q0
    const int4 *counts4 = (const int4 *)counts;
    for (int i4 = threadIdx.x; i4 < (q0 >> 2); i4 += SCAN_BLOCK) {
        const int4 c = counts4[i4];
        sum += max(c.x, 0) + max(c.y, 0) + max(c.z, 0) + max(c.w, 0);
        act += (c.x >= 0) + (c.y >= 0) + (c.z >= 0) + (c.w >= 0);
    }
    for (int i = q0 + threadIdx.x; i < lim; i += SCAN_BLOCK) act += (counts[i] >= 0);  // last workgroup only
    for (int o = 32; o > 0; o >>= 1) {
        sum += __shfl_down(sum, o);
        act += __shfl_down(act, o);
    }
    if ((threadIdx.x & 63) == 0) {
        red[threadIdx.x >> 6] = sum;
        red_active[threadIdx.x >> 6] = act;
    }
    __syncthreads();
    int prefix = 0, n_active = 0;
    for (int w = 0; w < SCAN_WAVES; ++w) {
        prefix += red[w];
        n_active += red_active[w];
    }
    if (threadIdx.x < 64) {
        int q = q0 + threadIdx.x;
        int c = (threadIdx.x < SCAN_QPB && q < Q) ? max(counts[q], 0) : 0;
        int inc = c;
        for (int o = 1; o < SCAN_QPB; o <<= 1) {
            int v = __shfl_up(inc, o);
            if ((int)threadIdx.x >= o) inc += v;
        }
        if (threadIdx.x < SCAN_QPB) {
            loc_cnt[threadIdx.x] = c;
            loc_off[threadIdx.x] = prefix + inc - c;
            if (threadIdx.x == SCAN_QPB - 1) loc_off[SCAN_QPB] = prefix + inc;
            if (q < Q) offsets[q] = prefix + inc - c;
        }
    }
    __syncthreads();
    if (last && threadIdx.x == 0) {
        ctrl->M = loc_off[SCAN_QPB];
        ctrl->n_active = n_active;
        if (mailbox) {
            // progress for the enqueuing host thread: one store to pinned host memory, nobody waits for it
            // nothing running and nothing waiting (open stream, Q_total < 0: nothing that has arrived so far)
            const int waiting_until = Q_total >= 0 ? Q_total : *(volatile int32_t *)&ctrl->avail;
            const bool finished = n_active == 0 && (Q_total == 0 || ctrl->next_query >= waiting_until);
            __hip_atomic_store(mailbox, mail_word | (finished ? 1ull : 0ull), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = wave; i < SCAN_QPB; i += SCAN_WAVES) {
        int q = q0 + i;
        if (q >= Q) break;
        int c = loc_cnt[i], off = loc_off[i];
        const int32_t *src = cand_g + (size_t)q * slots;
        const int32_t user = slot_query ? slot_query[q] : q;  // whose user vector scores this group
        for (int j = lane; j < c; j += 64) {
            pair_id[off + j] = src[j];
            pair_q[off + j] = user;
        }
    }
}

// ------------------------------------------------------------------------------------------
// One round of one query.
//
// The list (a6) lives in global memory, sorted; LDS holds only the new entries of the round and one
// tile of the list at a time, so the list may be as long as the workspace allows.
//
// Merge.  Only new entries that can enter the list are kept (better than the current worst entry once
// the list is full) and sorted on their own (<= W*R keys).  The list is then walked in tiles from its
// END towards the front: a tile of old entries is read into LDS, every old entry moves up by the number
// of new entries that precede it, every new entry that falls behind the tile's first entry goes to its
// own index plus the number of old entries that precede it (one binary search per entry in each
// direction), and the walk stops at the tile that takes the smallest new entry: the ranks in front of
// it do not change and are neither read nor written.  Moving entries towards the end while walking
// towards the front never overwrites an entry that has not been read yet, so the merge is in place.
// Keys are unique (an id is scored once per query), so the destinations are a permutation.
//
// Choice of parents.  The state keeps `first_open`, a rank below which every entry has been expanded
// (a lower bound of the first unexpanded rank: it falls to the first insertion point of a round and
// otherwise only grows).  The scan for the first <= W unexpanded entries among the first L ranks starts
// there, reading the list in pieces of one entry per thread (four per thread after the first piece).
// Eight workgroups of 256 threads fill a CU's wave slots; that needs no more than 64 registers per lane.
// BITMAP: the visited set is one bit per item (hash_cap < 0), else the hash table.  PIECES: a round may bring more
// candidates than pass the filter at once (both are compile-time so that each build holds one filter, once, in
// its 64 registers).  RESIDENT: the whole list fits one tile (C <= tile_keys); it is then requested at the very
// start, together with the state, merged into a second LDS copy, and the parents are chosen from that copy: two
// dependent trips to memory fewer per round than the tiled walk, which is what short lists are bound by.
template <int BLK, bool BITMAP, bool PIECES, bool RESIDENT>
__global__ void __launch_bounds__(BLK) __attribute__((amdgpu_waves_per_eu(ROUND_WAVES_MIN, 8)))
round_kernel(const int32_t *__restrict__ adj, const int32_t *__restrict__ adj_rank, int R, int64_t N, QState *state,
             uint64_t *pool_g, int C,
             uint32_t *hash, int hash_cap, int32_t *cand_g, int slots, int32_t *counts,
             const int32_t *__restrict__ offsets, const float *__restrict__ scores, int new_cap,
             int W_max, int64_t *stats, uint16_t *tag_g, int walkers, int tile_keys, int chunk) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int q = blockIdx.x;
    PHASE_START
    // LDS: parents and scan scratch first; then one region used twice: by the new entries and the list
    // tile during the merge, by the candidate ids and the dedupe tables afterwards
    int32_t *parents = (int32_t *)smem;                       // [W_max]
    int *wave_sums = parents + ((W_max + 3) & ~3);            // [16] one per wave
    int *shared_i = wave_sums + 16;                           // [8] values one thread hands to all
    uint64_t *newk = (uint64_t *)(shared_i + 8);              // [new_cap]   new entries, sorted
    uint64_t *best = newk + new_cap;                          // [W_max]     walkers: best new child of each
    uint64_t *tile = best + ((W_max + 1) & ~1);               // [tile_keys] a piece of the stored list
    uint64_t *merged = tile + tile_keys;                      // [C]         RESIDENT only: the list after the merge
    int32_t *cand = (int32_t *)newk;                          // [min(slots, FILTER_CHUNK)]
    uint64_t *pool = pool_g + (size_t)q * C;
    int32_t *cand_q = cand_g + (size_t)q * slots;
    uint16_t *tag_q = tag_g + (size_t)q * slots;

    // Everything the round needs first is requested at once, before any of it is looked at: the
    // workgroups of a launch start together, and every dependent trip to memory costs them all a few
    // microseconds.  (The worst entry is read whether or not the list is full: C >= 1.)
    const int n_prev = __builtin_amdgcn_readfirstlane(counts[q]);
    QState st = state[q];
    const int off = __builtin_amdgcn_readfirstlane(offsets[q]);
    const uint64_t stored_worst = RESIDENT ? 0 : pool[C - 1];
    if (n_prev < 0) return;  // finished or idle: counts[q] stays -1
    // the state is the same in every lane: kept in scalar registers, it leaves the vector registers to the filter
    st.t = __builtin_amdgcn_readfirstlane(st.t);
    st.done = __builtin_amdgcn_readfirstlane(st.done);
    st.n_list = __builtin_amdgcn_readfirstlane(st.n_list);
    st.n_visited = __builtin_amdgcn_readfirstlane(st.n_visited);
    st.W = __builtin_amdgcn_readfirstlane(st.W);
    st.L = __builtin_amdgcn_readfirstlane(st.L);
    st.cap = __builtin_amdgcn_readfirstlane(st.cap);
    st.n_expanded = __builtin_amdgcn_readfirstlane(st.n_expanded);
    st.first_open = __builtin_amdgcn_readfirstlane(st.first_open);
    if (RESIDENT) {  // the whole list, not only its n_list valid entries: requested before the state has arrived
#pragma unroll 4
        for (int i = threadIdx.x; i < C; i += BLK) tile[i] = pool[i];
    }
    if (st.done) {
        if (threadIdx.x == 0) counts[q] = -1;
        return;
    }
    // chunk: candidates that go through the visited filter together; with a bitmap addressed by rank their ranks
    // (adj_rank holds the rank of every adjacency entry, row for row) sit behind them
    int dd_n = 2;
    while (dd_n < 2 * chunk) dd_n <<= 1;
    int32_t *cand_rank = (BITMAP && adj_rank) ? cand + ((chunk + 3) & ~3) : nullptr;
    uint32_t *dd_key = (uint32_t *)(cand + (cand_rank ? 2 : 1) * ((chunk + 3) & ~3));
    uint32_t *dd_pos = dd_key + dd_n;
    uint32_t *bk_key = dd_pos + dd_n;
    uint32_t *bk_cnt = bk_key + dd_n;

    if (walkers)
        for (int i = threadIdx.x; i < W_max; i += BLK) best[i] = KEY_SENTINEL;
    if (threadIdx.x == 0) shared_i[0] = 0x7fffffff;  // rank of the first inserted entry
    __syncthreads();
    PHASE_MARK(0);  // state load

    // 1. the scores of the previous round (or of the seeds) become keys; those that cannot enter are dropped
    const bool full = (st.n_list == C);
    const uint64_t worst = full ? (RESIDENT ? tile[C - 1] : stored_worst) : KEY_SENTINEL;
    int m = 0;
    for (int j0 = 0; j0 < n_prev; j0 += BLK) {
        int j = j0 + threadIdx.x;
        uint64_t key = KEY_SENTINEL;
        bool keep = false;
        if (j < n_prev) {
            key = make_key(scores[off + j], cand_q[j], 0u);
            keep = key < worst;
            // walkers: the best newly scored neighbour of each walker, whether it enters the list or not
            if (walkers) atomicMin((unsigned long long *)&best[tag_q[j]], (unsigned long long)key);
        }
        int tot;
        int pos = block_excl_count<BLK>(keep, wave_sums, &tot);
        if (keep) newk[m + pos] = key;
        m += tot;
    }
    PHASE_MARK(1);  // new keys: scores load + filter
    int n_list = st.n_list;
    if (m > 0) {
        if (m <= BLK && 2 * tile_keys >= BLK && (!RESIDENT || 2 * C >= BLK)) {
            // scratch: a buffer that is free until the merge below
            rank_sort<BLK>(newk, m, (uint32_t *)(RESIDENT ? merged : tile));
        } else {
            int m2 = 2;
            while (m2 < m) m2 <<= 1;
            for (int i = m + threadIdx.x; i < m2; i += BLK) newk[i] = KEY_SENTINEL;
            __syncthreads();
            bitonic_sort<BLK>(newk, m2);
        }
        PHASE_MARK(6);  // sort of the new keys
        // 1b. merge into the stored list
        if (RESIDENT) {
            // by rank, into the second copy: an entry's position is its index in its own sequence plus the number
            // of entries of the other sequence in front of it
            for (int i = threadIdx.x; i < st.n_list + m; i += BLK) {
                uint64_t key;
                int pos;
                if (i < st.n_list) {
                    key = tile[i];
                    pos = i + lower_bound_keys(newk, m, key);
                } else {
                    key = newk[i - st.n_list];
                    pos = (i - st.n_list) + lower_bound_keys(tile, st.n_list, key);
                    if (i == st.n_list) shared_i[0] = pos;  // rank of the first inserted entry
                }
                if (pos < C) merged[pos] = key;
            }
        }
        // tile by tile from the end
        int hi = st.n_list, rem = RESIDENT ? 0 : m;
        while (rem > 0) {
            const int lo = max(0, hi - tile_keys), cnt = hi - lo;
            for (int i = threadIdx.x; i < cnt; i += BLK) tile[i] = pool[lo + i];
            __syncthreads();
            // new entries [0, nlo) precede the tile's first entry: they belong to tiles further front
            const int nlo = (lo == 0) ? 0 : lower_bound_keys(newk, rem, tile[0]);
            for (int i = threadIdx.x; i < cnt; i += BLK) {
                const uint64_t key = tile[i];
                const int lb = nlo + lower_bound_keys(newk + nlo, rem - nlo, key);
                const int dest = lo + i + lb;
                if (lb > 0 && dest < C) pool[dest] = key;  // lb = 0: the entry stays where it is
            }
            for (int j = nlo + threadIdx.x; j < rem; j += BLK) {
                const uint64_t key = newk[j];
                const int dest = j + lo + lower_bound_keys(tile, cnt, key);
                if (dest < C) pool[dest] = key;
                if (j == 0) shared_i[0] = dest;
            }
            __syncthreads();  // the tile buffer is free again
            hi = lo;
            rem = nlo;
        }
        n_list = min(C, st.n_list + m);
        // the scan below reads entries this workgroup has just stored
        if (!RESIDENT) __threadfence_block();
        __syncthreads();
    }
    PHASE_MARK(2);  // rank merge
    // RESIDENT: the list as it stands now, in LDS
    uint64_t *lw = RESIDENT ? (m > 0 ? merged : tile) : nullptr;

    // 2. termination test and choice of the parents
    int n_par = 0, n_live = 0;
    const bool capped = (st.cap > 0 && st.t >= st.cap);
    const int lim = walkers ? 0 : min(st.L, n_list);
    int first_open = min(st.first_open, shared_i[0]);
    if (walkers && !capped) {
        // Paper-literal variant (Alg. 1 read as independent walkers): walker s moves to the best of the
        // neighbours it scored last round (round 0: to its seed); a walker without one is dead (-1) and
        // contributes R invalid candidates, so that candidate position / R keeps naming the walker.
        for (int s0 = 0; s0 < st.W; s0 += BLK) {
            const int sl = s0 + threadIdx.x;
            const bool live = sl < st.W && best[sl] != KEY_SENTINEL;
            if (sl < st.W) parents[sl] = live ? key_id(best[sl]) : -1;
            int tot;
            (void)block_excl_count<BLK>(live, wave_sums, &tot);
            n_live += tot;
        }
        n_par = n_live > 0 ? st.W : 0;
    }
    if (!capped && !walkers) {
        int i0 = first_open;
        bool first_piece = true;
        while (i0 < lim && n_par < st.W) {
            // one entry per thread in the first piece (the parents are nearly always found there), four in the
            // later ones: all four are requested before the first is looked at
            const int per = first_piece ? 1 : 4;
            uint64_t e[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * BLK + (int)threadIdx.x;
                e[u] = (u < per && i < lim) ? (RESIDENT ? lw[i] : pool[i]) : KEY_SENTINEL;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (u >= per || i0 >= lim || n_par >= st.W) break;  // uniform over the workgroup
                const int i = i0 + (int)threadIdx.x;
                const bool open = (i < lim) && !key_expanded(e[u]);
                int tot;
                const int pos = block_excl_count<BLK>(open, wave_sums, &tot);
                if (open && n_par + pos < st.W) {
                    parents[n_par + pos] = key_id(e[u]);
                    pool[i] = e[u] | 1ull;
                    if (RESIDENT) lw[i] = e[u] | 1ull;  // the ranks from the first inserted entry on are stored below
                    if (n_par + pos == st.W - 1) shared_i[1] = i + 1;  // everything in front of it is expanded now
                }
                first_open = (n_par + tot >= st.W) ? -1 : min(i0 + BLK, lim);  // -1: taken from shared_i[1] below
                n_par = min(st.W, n_par + tot);
                i0 += BLK;
            }
            first_piece = false;
        }
    }
    __syncthreads();
    if (first_open < 0) first_open = shared_i[1];
    if (RESIDENT && m > 0)  // what the merge moved: the ranks from the first inserted entry on
        for (int i = shared_i[0] + threadIdx.x; i < n_list; i += BLK) pool[i] = lw[i];
    // a visited table that could not take this round's ids ends the query
    bool overflow = false;
    if (!BITMAP && n_par > 0 && (int64_t)st.n_visited + (int64_t)n_par * R > (int64_t)(hash_cap / 2)) {
        overflow = true;
        n_par = 0;
    }
    if (n_par == 0) {
        if (threadIdx.x == 0) {
            state[q].n_list = n_list;
            state[q].first_open = first_open;
            state[q].done = overflow ? 3 : 1;
            counts[q] = -1;
        }
        return;
    }

    if (RESIDENT) __syncthreads();  // the LDS copies of the list are dead from here on; their space is reused
    // 3. neighbour gather: one adjacency row per parent, consecutive lanes read consecutive ids;
    // 4. visited filter, 5. survivors of this query for the next MLP launch.
    // A round's candidates go through in pieces of at most `chunk` (what the dedupe tables in LDS hold).  An id
    // that comes again in a later piece is dropped there because the earlier piece has entered it into the
    // visited table: the first occurrence still wins, in candidate order.
    PHASE_MARK(3);  // selection
    const int n_cand = n_par * R;
    int n_new = 0;
    for (int c0 = 0; c0 < (PIECES ? n_cand : 1); c0 += chunk) {
        const int nc = PIECES ? min(chunk, n_cand - c0) : n_cand;
        if (PIECES && c0 > 0) {  // the table stores of the piece before must be seen by this piece's reads
            __threadfence_block();
            __syncthreads();
        }
        for (int j = threadIdx.x; j < nc; j += BLK) {
            const int p = (c0 + j) / R, s = (c0 + j) - p * R;
            cand[j] = parents[p] >= 0 ? adj[(size_t)parents[p] * R + s] : -1;
            if (BITMAP && cand_rank) cand_rank[j] = parents[p] >= 0 ? adj_rank[(size_t)parents[p] * R + s] : -1;
        }
        __syncthreads();
        if (BITMAP)
            n_new += filter_and_mark<BLK>(cand, cand_rank, nc, dd_key, dd_pos, bk_key, bk_cnt, dd_n, hash + (size_t)q * (size_t)(-hash_cap),
                                          N, cand_q + n_new, wave_sums, tag_q + n_new, R, PIECES ? c0 : 0);
        else
            n_new += filter_and_insert<BLK>(cand, nc, dd_key, dd_pos, bk_key, bk_cnt, dd_n, hash + (size_t)q * hash_cap,
                                            hash_cap, N, cand_q + n_new, wave_sums, tag_q + n_new, R, PIECES ? c0 : 0);
    }
    PHASE_MARK(5);  // adjacency gather, dedupe + visited table
    if (threadIdx.x == 0) {
        state[q].n_list = n_list;
        state[q].first_open = first_open;
        state[q].t = st.t + 1;
        state[q].n_visited = st.n_visited + n_new;
        state[q].n_expanded = st.n_expanded + (walkers ? n_live : n_par);
        counts[q] = n_new;
    }
}

// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(BLOCK)
emit_kernel(const QState *__restrict__ state, const uint64_t *__restrict__ pool_g, int C, int k,
            int32_t *out_ids, float *out_scores, int64_t *stats, int Q) {
    emit_row<BLOCK>(state, pool_g, C, k, blockIdx.x, blockIdx.x, out_ids, out_scores);
    // counters: every 64th workgroup sums those of 64 consecutive queries in its first wave
    if ((blockIdx.x & 63) == 0 && threadIdx.x < 64) {
        const int q = blockIdx.x + threadIdx.x;
        long long scored = 0, expanded = 0;
        int rounds = 0, overflowed = 0;
        if (q < Q) {
            const QState st = state[q];
            scored = st.n_visited, expanded = st.n_expanded, rounds = st.t, overflowed = (st.done & 2) ? 1 : 0;
        }
        for (int o = 32; o > 0; o >>= 1) {
            scored += __shfl_down(scored, o);
            expanded += __shfl_down(expanded, o);
            rounds = max(rounds, __shfl_down(rounds, o));
            overflowed += __shfl_down(overflowed, o);
        }
        if (threadIdx.x == 0) add_to_totals(stats, scored, expanded, rounds, overflowed);
    }
}

// ------------------------------------------------------------------------------------------
// What the kernels take as `hash_cap`: the hash table's entries, or minus the bitmap's words.
static int table_cap_arg(const Plan &p) { return p.bitmap_words > 0 ? -p.bitmap_words : p.hash_cap; }

static int item_row_bytes(const ann_graph *g) {
    return g->d * (g->dtype == ANN_F32 ? 4 : g->dtype == ANN_F8 ? 1 : 2);
}

static int new_cap_of(const Plan &p) {
    int n = 2;
    while (n < p.slots) n <<= 1;
    return n;
}

// Entries of the stored list that the round kernel holds in LDS at a time during the merge: the whole list
// when it is short, a quarter of a long one, at most 4,096 (32 KB).
static int tile_keys_of(const Plan &p) {
    int t = 1024;
    while (t < ROUND_TILE_MAX && 4 * t < p.C) t <<= 1;
    return t;
}

// Does the visited bitmap of this search go by the graph's locality order?
static bool ranked(const ann_graph *g, const Plan &p) { return p.bitmap_words > 0 && g->adj_rank != nullptr; }

// Candidates that go through the visited filter together.  With ranks beside the ids the pieces are half as
// large, so that the filter's LDS stays below what the merge needs anyway (the piece size does not show in the
// kernel's time).
static int filter_chunk(const ann_graph *g, const Plan &p) {
    const int most = ranked(g, p) ? FILTER_CHUNK / 2 : FILTER_CHUNK;
    return p.slots < most ? p.slots : most;
}

// list_keys: list entries held in LDS (0: one tile)
static size_t round_smem(const ann_graph *g, const Plan &p, int list_keys = 0) {
    const int chunk = filter_chunk(g, p);
    int dd_n = 2;
    while (dd_n < 2 * chunk) dd_n <<= 1;
    size_t lists = (size_t)(new_cap_of(p) + ((p.W_max + 1) & ~1) + (list_keys > 0 ? list_keys : tile_keys_of(p))) * 8;
    size_t filt = (size_t)((chunk + 3) & ~3) * 4 * (ranked(g, p) ? 2 : 1) + (size_t)dd_n * 16;
    return (size_t)((p.W_max + 3) & ~3) * 4 + 24 * 4 + (lists > filt ? lists : filt);
}

static size_t seed_smem(const ann_graph *g, const Plan &p) {
    int dd_n = 2;
    while (dd_n < 2 * p.E) dd_n <<= 1;
    return (size_t)((p.E + 3) & ~3) * 4 * (ranked(g, p) ? 2 : 1) + (size_t)dd_n * 16 + (WAVES + 1) * 4;
}

int launch_init(const SearchArgs &a) {
    const Plan &p = a.plan;
    size_t smem = seed_smem(a.g, p);
    int64_t *stats = (int64_t *)(a.ws + p.off_stats);
    hipLaunchKernelGGL(zero_stats_kernel, dim3(1), dim3(64), 0, a.stream, stats, (Ctrl *)(a.ws + p.off_ctrl), p.Q,
                       a.keep_stats ? 1 : 0, p.R * 4, item_row_bytes(a.g));
    hipLaunchKernelGGL(init_kernel, dim3(p.Q), dim3(BLOCK), smem, a.stream, a.entries,
                       ranked(a.g, p) ? a.g->rank : nullptr, p.E, a.g->N,
                       (QState *)(a.ws + p.off_state), (uint32_t *)(a.ws + p.off_hash), table_cap_arg(p),
                       (int32_t *)(a.ws + p.off_cand), p.slots, (int32_t *)(a.ws + p.off_counts), a.W_q,
                       a.L_q, a.cap_q, a.W, a.L, a.cap, p.W_max, p.L_max, p.max_iters_max, stats,
                       (uint16_t *)(a.ws + p.off_tag));
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

int launch_stream_reset(const SearchArgs &a) {
    const Plan &p = a.plan;
    const int n = p.Q > 16 ? p.Q : 16;
    hipLaunchKernelGGL(stream_reset_kernel, dim3((n + 255) / 256), dim3(256), 0, a.stream,
                       (int64_t *)(a.ws + p.off_stats), (Ctrl *)(a.ws + p.off_ctrl), (QState *)(a.ws + p.off_state),
                       (int32_t *)(a.ws + p.off_counts), a.slot_query, p.Q, a.Q_total, p.R * 4, item_row_bytes(a.g));
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

int launch_stream_publish(const SearchArgs &a, int avail) {
    const Plan &p = a.plan;
    hipLaunchKernelGGL(stream_publish_kernel, dim3(1), dim3(64), 0, a.stream, (Ctrl *)(a.ws + p.off_ctrl),
                       (int64_t *)(a.ws + p.off_stats), avail);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

int launch_admit(const SearchArgs &a) {
    const Plan &p = a.plan;
    hipLaunchKernelGGL(admit_kernel, dim3(p.Q), dim3(BLOCK), seed_smem(a.g, p), a.stream, a.entries,
                       ranked(a.g, p) ? a.g->rank : nullptr, p.E, a.g->N,
                       (QState *)(a.ws + p.off_state), (uint32_t *)(a.ws + p.off_hash), table_cap_arg(p),
                       (int32_t *)(a.ws + p.off_cand), p.slots, (int32_t *)(a.ws + p.off_counts), a.W_q, a.L_q,
                       a.cap_q, a.W, a.L, a.cap, p.W_max, p.L_max, p.max_iters_max, (int64_t *)(a.ws + p.off_stats),
                       (Ctrl *)(a.ws + p.off_ctrl), a.slot_query, a.Q_total, (const uint64_t *)(a.ws + p.off_pool), p.C,
                       p.k, a.out_ids, a.out_scores, (uint16_t *)(a.ws + p.off_tag));
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

int launch_scan_compact(const SearchArgs &a) {
    const Plan &p = a.plan;
    // every workgroup reads the counts of all earlier queries: with very many queries fewer, larger workgroups
    const int qpb = p.Q <= 8192 ? 4 : 8;
    const int blocks = (p.Q + qpb - 1) / qpb;
    auto fn = qpb == 4 ? scan_compact_kernel<4> : scan_compact_kernel<8>;
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(SCAN_BLOCK), 0, a.stream,
                       (const int32_t *)(a.ws + p.off_counts), p.Q, (const int32_t *)(a.ws + p.off_cand),
                       p.slots, (int32_t *)(a.ws + p.off_offsets), (int32_t *)(a.ws + p.off_pair_q),
                       (int32_t *)(a.ws + p.off_pair_id), (Ctrl *)(a.ws + p.off_ctrl), a.slot_query, a.mailbox,
                       a.mail_tag | ((uint64_t)(uint32_t)(a.round_index + 1) << 1), a.Q_total);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

int launch_round(const SearchArgs &a) {
    const Plan &p = a.plan;
    size_t smem = round_smem(a.g, p);
    // Workgroups of 128 threads when a round has at most 128 candidates per query and the batch is far larger
    // than what a chip holds at once (2,048 workgroups of 256): twice as many queries are then resident, and
    // the candidates still go through the visited filter in one pass.  (C4: 33 -> 28 ms per step; with few
    // queries the shorter path of the larger workgroup wins: C2 3.9 against 4.2 ms.)
    // Workgroups of 1,024 threads when a round brings more than 512 candidates per query: the candidates pass the
    // visited filter in one sweep, and the sort and the merge have a quarter of the work per thread.
    const bool half = (p.slots <= 128 && p.Q >= 8192);
    const bool big = p.slots > ROUND_BIG_FROM;  // several filter pieces only occur here: slots > FILTER_CHUNK / 2
    const int which = half ? 1 : big ? 2 : 0;
    const int threads = half ? 128 : big ? ROUND_BIG_BLOCK : BLOCK;
    const bool bm = p.bitmap_words > 0;
    const int chunk = filter_chunk(a.g, p);
    const bool pieces = p.slots > chunk;
    const bool resident = !big && p.C <= tile_keys_of(p);
    const int tile_keys = resident ? ((p.C + 1) & ~1) : tile_keys_of(p);  // resident: the list itself, twice
    if (resident) smem = round_smem(a.g, p, tile_keys + p.C);
    using Fn = decltype(&round_kernel<BLOCK, false, false, false>);
    Fn fn;
    if (big)
        fn = pieces ? (bm ? round_kernel<ROUND_BIG_BLOCK, true, true, false> : round_kernel<ROUND_BIG_BLOCK, false, true, false>)
                    : (bm ? round_kernel<ROUND_BIG_BLOCK, true, false, false> : round_kernel<ROUND_BIG_BLOCK, false, false, false>);
    else if (half)
        fn = resident ? (bm ? round_kernel<128, true, false, true> : round_kernel<128, false, false, true>)
                      : (bm ? round_kernel<128, true, false, false> : round_kernel<128, false, false, false>);
    else
        fn = resident ? (bm ? round_kernel<BLOCK, true, false, true> : round_kernel<BLOCK, false, false, true>)
                      : (bm ? round_kernel<BLOCK, true, false, false> : round_kernel<BLOCK, false, false, false>);
    if (smem > 48 * 1024) {
        static std::atomic<uint32_t> raised[24];
        if (int rc = raise_lds_limit((const void *)fn, 128 * 1024, a.m->device,
                                     raised[8 * which + (bm ? 4 : 0) + (pieces ? 2 : 0) + (resident ? 1 : 0)]);
            rc != ANN_OK)
            return rc;
    }
    hipLaunchKernelGGL(fn, dim3(p.Q), dim3(threads), smem, a.stream, a.g->adj,
                       ranked(a.g, p) ? a.g->adj_rank : nullptr, p.R, a.g->N,
                       (QState *)(a.ws + p.off_state), (uint64_t *)(a.ws + p.off_pool), p.C,
                       (uint32_t *)(a.ws + p.off_hash), table_cap_arg(p), (int32_t *)(a.ws + p.off_cand), p.slots,
                       (int32_t *)(a.ws + p.off_counts), (const int32_t *)(a.ws + p.off_offsets),
                       (const float *)(a.ws + p.off_scores), new_cap_of(p), p.W_max,
                       (int64_t *)(a.ws + p.off_stats), (uint16_t *)(a.ws + p.off_tag), a.walkers ? 1 : 0,
                       tile_keys, chunk);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

int launch_emit(const SearchArgs &a) {
    const Plan &p = a.plan;
    hipLaunchKernelGGL(emit_kernel, dim3(p.Q), dim3(BLOCK), 0, a.stream, (const QState *)(a.ws + p.off_state),
                       (const uint64_t *)(a.ws + p.off_pool), p.C, p.k, a.out_ids, a.out_scores,
                       (int64_t *)(a.ws + p.off_stats), p.Q);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

}  // namespace gmpgr
