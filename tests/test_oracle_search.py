"""Pins for the oracle's search (Sec. 3.2, Algorithm 1) and brute force (Sec. 5.1.3).

None of the expected values below comes from the oracle's own search loop:
hand-derived ring trajectories (tests/golden/ring_trajectories.json), exhaustive
ranking by numpy, an independently written priority-queue best-first search,
and invariants that hold for any correct implementation.
"""
import heapq
import json
import os

import numpy as np
import pytest

import oracle
from workloads import PRESETS, make_workload, random_mlp, scaled, to_host

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def _rank_all(emb, users, mlp, k):
    """Exhaustive ranking with numpy's lexsort on per-pair scores (score desc, id asc)."""
    N, Q = emb.shape[0], users.shape[0]
    ids = np.empty((Q, k), np.int32)
    sc = np.empty((Q, k), np.float32)
    for q in range(Q):
        s = oracle.score_pairs(emb, users, mlp, np.full(N, q), np.arange(N))
        order = np.lexsort((np.arange(N), -s.astype(np.float64)))[:k]
        ids[q, : len(order)] = order
        sc[q, : len(order)] = s[order]
    return ids, sc


def _tiny(seed, N=300, d=8, R=6, Q=6, hidden=(12,), J=3, n_clusters=5, E=2):
    cfg = scaled(PRESETS["C1"], N, n_clusters=n_clusters, Q=Q)
    from dataclasses import replace

    cfg = replace(cfg, d=d, R=R, hidden=hidden, head_w=(0.5, 0.3, 0.2)[:J], E=E)
    wl = to_host(make_workload(cfg, seed=seed))
    Ws, bs = random_mlp(cfg.dims, seed + 100, "f32", bias_scale=0.2)
    mlp = oracle.Mlp([w.numpy() for w in Ws], [b.numpy() for b in bs], np.asarray(cfg.head_w, np.float32))
    return wl, mlp


def _monotone_problem(N, R, direction):
    """Ring graph and a one-layer metric strictly monotone in the item id."""
    adj = (np.arange(N)[:, None] + np.arange(1, R + 1)[None, :]) % N
    emb = np.zeros((N, 2), np.float32)
    emb[:, 0] = np.arange(N) / N
    a = 4.0 if direction == "increasing" else -4.0
    # concat(user[2], item[2]); only item coordinate 0 matters
    mlp = oracle.Mlp([np.array([[0, 0, a, 0]], np.float32)], [np.zeros(1, np.float32)], np.ones(1, np.float32))
    return adj.astype(np.int32), emb, mlp


# ----------------------------------------------------------------------------- golden trajectories
@pytest.mark.parametrize("case", json.load(open(os.path.join(GOLD, "ring_trajectories.json")))["cases"],
                         ids=lambda c: c["name"])
def test_ring_trajectory_by_hand(case):
    adj, emb, mlp = _monotone_problem(case["N"], case["R"], case["monotone"])
    users = np.zeros((1, 2), np.float32)
    entries = np.asarray([case["seed"]], np.int32)
    r = oracle.search(emb, adj, users, mlp, entries, case["W"], case["L"], case["k"], case["max_iters"],
                      trace=True, visited_cap=256, trace_cap=64)
    assert r["ids"][0].tolist() == case["expected_ids"]
    vis = case["expected_visited_in_order"]
    want = list(range(*vis["range"])) if "range" in vis else vis["list"]
    got = [v for v in r["visited"][0].tolist() if v >= 0]
    assert got == want
    assert int(r["n_expanded"][0]) == case["n_expanded"]
    assert int(r["n_scored"][0]) == case["n_scored"]
    assert int(r["n_iters"][0]) == case["n_iters"]
    # scores returned are those of the returned ids
    s = oracle.score_pairs(emb, users, mlp, np.zeros(case["k"], np.int32), r["ids"][0])
    assert np.array_equal(s, r["scores"][0])


# ----------------------------------------------------------------------------- layer-by-layer search
def _ring(n, R):
    return ((np.arange(n)[:, None] + np.arange(1, R + 1)[None, :]) % n).astype(np.int32)


@pytest.mark.parametrize("case", json.load(open(os.path.join(GOLD, "layered_trajectories.json")))["cases"],
                         ids=lambda c: c["name"])
def test_layered_trajectory_by_hand(case):
    N_l, R = case["N_l"], case["R"]
    _, emb, mlp = _monotone_problem(N_l[-1], R, case["monotone"])
    adjs = [_ring(n, R) for n in N_l]
    users = np.zeros((1, 2), np.float32)
    entries = np.asarray([case["seed"]], np.int32)
    # the oracle's layer loop, with the per-layer traces taken from separate calls so that the
    # visited order can be checked too
    r = oracle.search_layers(emb, adjs, users, mlp, entries, case["W_l"], case["L_l"], case["K_l"],
                             case["max_iters"], trace=True)
    seeds = entries
    for l, n in enumerate(N_l):
        lay = r["layers"][l]
        assert lay["ids"][0].tolist() == case["expected_ids_per_layer"][l]
        assert int(lay["n_scored"][0]) == case["n_scored_per_layer"][l]
        assert int(lay["n_expanded"][0]) == case["n_expanded_per_layer"][l]
        assert int(lay["n_iters"][0]) == case["n_iters_per_layer"][l]
        one = oracle.search(emb[:n], adjs[l], users, mlp, seeds, case["W_l"][l], case["L_l"][l], case["K_l"][l],
                            case["max_iters"], trace=True, visited_cap=64)
        vis = case["expected_visited_per_layer"][l]
        want = list(range(*vis["range"])) if "range" in vis else vis["list"]
        assert [v for v in one["visited"][0].tolist() if v >= 0] == want
        seeds = np.asarray([case["expected_ids_per_layer"][l]], np.int32)
    assert r["ids"][0].tolist() == case["expected_ids_per_layer"][-1]
    assert int(r["n_scored"][0]) == sum(case["n_scored_per_layer"])


def _nested_layers(wl, sizes, R, seed):
    """Random nested graphs over the first sizes[l] items (valid ids only, no self loops)."""
    rng = np.random.default_rng(seed)
    adjs = []
    for n in sizes:
        a = rng.integers(0, n - 1, size=(n, R))
        a = a + (a >= np.arange(n)[:, None])     # skip the node itself
        adjs.append(a.astype(np.int32))
    return adjs


def test_one_layer_is_the_flat_search():
    wl, mlp = _tiny(21)
    a = oracle.search(wl["emb"], wl["adj"], wl["users"], mlp, wl["entries"], 2, 12, 9)
    b = oracle.search_layers(wl["emb"], [wl["adj"]], wl["users"], mlp, wl["entries"], [2], [12], [9])
    assert np.array_equal(a["ids"], b["ids"]) and np.array_equal(a["scores"], b["scores"])


def test_layers_chain_through_their_result_lists():
    # an independent statement of the outer loop: best-first search (written separately below)
    # per layer with W = 1, the k best of a layer being the seeds of the next
    wl, mlp = _tiny(22, N=400, Q=4, E=1)
    sizes = [40, 150, 400]
    adjs = _nested_layers(wl, sizes, 5, 7)
    ef, K = [6, 8, 10], [3, 4, 7]
    entries = (wl["entries"] % sizes[0]).astype(np.int32)
    got = oracle.search_layers(wl["emb"], adjs, wl["users"], mlp, entries, [1, 1, 1], ef, K)
    for q in range(4):
        s = oracle.score_pairs(wl["emb"], wl["users"], mlp, np.full(400, q), np.arange(400)).astype(np.float64)
        seeds = [int(entries[q, 0])]
        for l, n in enumerate(sizes):
            seeds = _best_first_multi(s[:n], adjs[l], seeds, ef[l], K[l])
        assert got["ids"][q].tolist() == seeds + [-1] * (K[-1] - len(seeds))


def test_complete_layers_equal_brute_force():
    wl, mlp = _tiny(23, N=120, Q=5, E=2)
    sizes = [15, 50, 120]
    adjs = []
    for n in sizes:
        a = np.arange(n - 1)[None, :] + (np.arange(n - 1)[None, :] >= np.arange(n)[:, None])
        adjs.append(a.astype(np.int32))
    entries = (wl["entries"] % sizes[0]).astype(np.int32)
    got = oracle.search_layers(wl["emb"], adjs, wl["users"], mlp, entries, [2, 3, 2], [4, 6, 5], [5, 8, 11])
    ids, sc = _rank_all(wl["emb"], wl["users"], mlp, 11)
    assert np.array_equal(got["ids"], ids)
    assert np.array_equal(got["scores"], sc)


# ----------------------------------------------------------------------------- walkers (paper-literal variant)
@pytest.mark.parametrize("case", json.load(open(os.path.join(GOLD, "walker_trajectories.json")))["cases"],
                         ids=lambda c: c["name"])
def test_walker_trajectory_by_hand(case):
    adj, emb, mlp = _monotone_problem(case["N"], case["R"], case["monotone"])
    users = np.zeros((1, 2), np.float32)
    entries = np.asarray([case["seed"]], np.int32)
    r = oracle.search_walkers(emb, adj, users, mlp, entries, case["T"], case["k"], trace=True, visited_cap=64)
    assert r["ids"][0].tolist() == case["expected_ids"]
    vis = case["expected_visited_in_order"]
    want = list(range(*vis["range"])) if "range" in vis else vis["list"]
    assert [v for v in r["visited"][0].tolist() if v >= 0] == want
    assert int(r["n_scored"][0]) == case["n_scored"]
    assert int(r["n_expanded"][0]) == case["n_expanded"]
    assert int(r["n_iters"][0]) == case["n_iters"]


def _walkers_reference(scores, adj, seeds, T, k):
    """The walker search written independently with dicts: returns the k best visited ids."""
    seen, where = {}, []
    for s in seeds:
        if 0 <= s < len(scores) and s not in seen:
            seen[s] = scores[s]
            where.append(s)
        else:
            where.append(None)
    for _ in range(T):
        if all(w is None for w in where):
            break
        moves = []
        for w in where:
            mine = []
            if w is not None:
                for v in adj[w]:
                    v = int(v)
                    if v not in seen:
                        seen[v] = scores[v]
                        mine.append(v)
            moves.append(min(mine, key=lambda v: (-scores[v], v)) if mine else None)
        where = moves
    return sorted(seen, key=lambda v: (-seen[v], v))[:k]


def test_walkers_equal_an_independent_implementation():
    wl, mlp = _tiny(31, N=500, Q=5, E=4, R=6)
    entries = wl["entries"].copy()
    entries[1, 2] = entries[1, 0]      # a repeated seed starts no second walker
    entries[2, 1] = -5                 # nor does an invalid one
    for T, k in ((1, 10), (4, 25), (12, 60)):
        got = oracle.search_walkers(wl["emb"], wl["adj"], wl["users"], mlp, entries, T, k)
        for q in range(5):
            s = oracle.score_pairs(wl["emb"], wl["users"], mlp, np.full(500, q), np.arange(500)).astype(np.float64)
            want = _walkers_reference(s, wl["adj"], [int(e) for e in entries[q]], T, k)
            assert got["ids"][q].tolist() == want + [-1] * (k - len(want))


def test_walkers_on_a_complete_graph_find_the_best_items_in_one_hop():
    wl, mlp = _tiny(32, N=60, Q=4, E=3)
    n = 60
    adj = (np.arange(n - 1)[None, :] + (np.arange(n - 1)[None, :] >= np.arange(n)[:, None])).astype(np.int32)
    got = oracle.search_walkers(wl["emb"], adj, wl["users"], mlp, wl["entries"] % n, 1, 12)
    ids, sc = _rank_all(wl["emb"], wl["users"], mlp, 12)
    assert np.array_equal(got["ids"], ids) and np.array_equal(got["scores"], sc)


def test_single_walker_on_monotone_scores_is_the_flat_search_with_w1():
    # with strictly increasing relevance along the ring, greedy hops and best-first expansion coincide
    adj, emb, mlp = _monotone_problem(300, 8, "increasing")
    users = np.zeros((1, 2), np.float32)
    entries = np.asarray([[7]], np.int32)
    a = oracle.search_walkers(emb, adj, users, mlp, entries, 9, 20)
    b = oracle.search(emb, adj, users, mlp, entries, 1, 4, 20, 9)
    assert np.array_equal(a["ids"], b["ids"])


# ----------------------------------------------------------------------------- brute force
def test_brute_force_is_the_exhaustive_ranking():
    wl, mlp = _tiny(11)
    got = oracle.brute_force(wl["emb"], wl["users"], mlp, 17, n_threads=2)
    ids, sc = _rank_all(wl["emb"], wl["users"], mlp, 17)
    assert np.array_equal(got["ids"], ids)
    assert np.array_equal(got["scores"], sc)


def test_brute_force_pads_when_k_exceeds_n():
    emb = np.random.default_rng(0).standard_normal((3, 2)).astype(np.float32)
    users = np.zeros((1, 2), np.float32)
    mlp = oracle.Mlp([np.ones((1, 4), np.float32)], [np.zeros(1, np.float32)], np.ones(1, np.float32))
    r = oracle.brute_force(emb, users, mlp, 5)
    assert r["ids"][0, 3:].tolist() == [-1, -1] and np.all(np.isneginf(r["scores"][0, 3:]))
    assert sorted(r["ids"][0, :3].tolist()) == [0, 1, 2]


def test_rerank_of_every_item_is_brute_force_and_of_a_subset_its_restriction():
    wl, mlp = _tiny(12)
    N, Q = wl["emb"].shape[0], wl["users"].shape[0]
    rng = np.random.default_rng(3)
    everything = np.stack([rng.permutation(N) for _ in range(Q)]).astype(np.int32)
    bf = oracle.brute_force(wl["emb"], wl["users"], mlp, 17)
    rr = oracle.rerank(wl["emb"], wl["users"], mlp, everything, 17)
    assert np.array_equal(rr["ids"], bf["ids"]) and np.array_equal(rr["scores"], bf["scores"])
    # a subset, with padding and out-of-range ids among the candidates: the exhaustive ranking restricted to it
    full = oracle.brute_force(wl["emb"], wl["users"], mlp, N)
    sub = everything[:, : N // 3].copy()
    cand = np.concatenate([sub, np.full((Q, 2), -1, np.int32), np.full((Q, 1), N, np.int32)], axis=1)
    rr = oracle.rerank(wl["emb"], wl["users"], mlp, cand, N // 3 + 4)
    for q in range(Q):
        keep = [v for v in full["ids"][q] if v in set(sub[q].tolist())]
        assert rr["ids"][q, : len(keep)].tolist() == keep
        assert np.all(rr["ids"][q, len(keep):] == -1) and np.all(np.isneginf(rr["scores"][q, len(keep):]))
    # a repeated candidate is kept as often as it occurs
    twice = np.concatenate([sub[:, :5], sub[:, :1]], axis=1)
    rr = oracle.rerank(wl["emb"], wl["users"], mlp, twice, 6)
    for q in range(Q):
        assert sorted(rr["ids"][q].tolist()) == sorted(twice[q].tolist())


def test_complete_graph_search_equals_brute_force():
    # one expansion of the seed reaches every item
    wl, mlp = _tiny(12, N=120, R=6)
    N = 120
    adj = np.stack([np.delete(np.arange(N), i) for i in range(N)]).astype(np.int32)
    for W, L, k in ((1, 4, 10), (3, 16, 5), (2, 1, 30)):
        r = oracle.search(wl["emb"], adj, wl["users"], mlp, wl["entries"], W, L, k, 0)
        bf = oracle.brute_force(wl["emb"], wl["users"], mlp, k)
        assert np.array_equal(r["ids"], bf["ids"])
        assert np.array_equal(r["scores"], bf["scores"])


def _reachable(adj, seeds):
    seen = set(int(s) for s in seeds)
    todo = list(seen)
    while todo:
        v = todo.pop()
        for w in adj[v]:
            if int(w) not in seen:
                seen.add(int(w))
                todo.append(int(w))
    return seen


def test_pool_as_large_as_the_graph_equals_brute_force():
    wl, mlp = _tiny(13, N=250, R=8, Q=5)
    N = 250
    for q in range(5):
        assert len(_reachable(wl["adj"], wl["entries"][q])) == N  # every node reachable from the seeds
    for W in (1, 4):
        r = oracle.search(wl["emb"], wl["adj"], wl["users"], mlp, wl["entries"], W, N, 20, 0, trace=True)
        bf = oracle.brute_force(wl["emb"], wl["users"], mlp, 20)
        assert np.array_equal(r["ids"], bf["ids"])
        assert np.array_equal(r["scores"], bf["scores"])
        assert np.all(r["n_scored"] == N) and np.all(r["n_expanded"] == N)


# ----------------------------------------------------------------------------- invariants
@pytest.mark.parametrize("W,L,k,E,cap", [(2, 32, 10, 1, 0), (4, 16, 40, 3, 0), (1, 8, 8, 2, 5), (8, 24, 100, 4, 3)])
def test_invariants_on_clustered_graph(W, L, k, E, cap):
    cfg = scaled(PRESETS["C1"], 3000, n_clusters=8, Q=24)
    from dataclasses import replace

    cfg = replace(cfg, E=E)
    wl = to_host(make_workload(cfg, seed=77))
    mlp = oracle.Mlp(wl["W"], wl["b"], wl["head_w"])
    R = wl["adj"].shape[1]
    r = oracle.search(wl["emb"], wl["adj"], wl["users"], mlp, wl["entries"], W, L, k, cap, trace=True,
                      visited_cap=4096, trace_cap=512, n_threads=4)
    for q in range(cfg.Q):
        vis = r["visited"][q]
        vis = vis[vis >= 0]
        assert len(vis) == r["n_scored"][q] == len(set(vis.tolist()))  # each id scored once
        t = int(r["n_iters"][q])
        assert len(vis) <= E + t * W * R
        if cap:
            assert t <= cap
        # result = best k of everything that was scored, in (score desc, id asc) order
        s = oracle.score_pairs(wl["emb"], wl["users"], mlp, np.full(len(vis), q), vis)
        order = np.lexsort((vis, -s.astype(np.float64)))[:k]
        want_ids = np.full(k, -1, np.int32)
        want_ids[: len(order)] = vis[order]
        assert np.array_equal(r["ids"][q], want_ids)
        valid = r["ids"][q] >= 0
        assert len(set(r["ids"][q][valid].tolist())) == valid.sum()
        assert np.array_equal(r["scores"][q][valid], s[order])
        assert np.all(np.isneginf(r["scores"][q][~valid]))
        # score at rank L never decreases; -inf while fewer than L were scored
        w = r["worst"][q][: t + 1]
        assert not np.any(np.isnan(w))
        assert np.all(w[1:] >= w[:-1])
        assert np.all(np.isnan(r["worst"][q][t + 1:]))


def test_all_equal_scores_fall_back_to_smallest_ids():
    N, R = 64, 5
    rng = np.random.default_rng(3)
    adj = np.stack([rng.choice(np.delete(np.arange(N), i), R, replace=False) for i in range(N)]).astype(np.int32)
    emb = rng.standard_normal((N, 4)).astype(np.float32)
    users = rng.standard_normal((3, 4)).astype(np.float32)
    mlp = oracle.Mlp([np.zeros((2, 8), np.float32)], [np.zeros(2, np.float32)], np.array([0.5, 0.5], np.float32))
    entries = np.array([[7], [20], [63]], np.int32)
    r = oracle.search(emb, adj, users, mlp, entries, 2, 6, 9, 3, trace=True, visited_cap=128)
    for q in range(3):
        vis = sorted(v for v in r["visited"][q].tolist() if v >= 0)
        want = (vis + [-1] * 9)[:9]
        assert r["ids"][q].tolist() == want
    # complete graph: the k smallest ids overall
    adjc = np.stack([np.delete(np.arange(N), i) for i in range(N)]).astype(np.int32)
    r = oracle.search(emb, adjc, users, mlp, entries, 1, 4, 9, 0)
    assert all(r["ids"][q].tolist() == list(range(9)) for q in range(3))


# ----------------------------------------------------------------------------- W = E = 1 is best-first search
def _best_first(scores, adj, seed, ef, k):
    """Textbook greedy best-first graph search with a bounded result set (ef), written with
    heaps; `scores` holds the relevance of every item for this query."""
    visited = {seed}
    cand = [(-scores[seed], seed)]  # max-heap on score, ties to the smaller id
    res = [(scores[seed], -seed)]  # min-heap: worst result on top (lower score, then larger id)
    while cand:
        neg, c = heapq.heappop(cand)
        worst_s, worst_negid = res[0]
        if len(res) >= ef and (-neg, -c) < (worst_s, worst_negid):
            break
        for v in adj[c]:
            v = int(v)
            if v in visited:
                continue
            visited.add(v)
            if len(res) < ef or (scores[v], -v) > res[0]:
                heapq.heappush(cand, (-scores[v], v))
                heapq.heappush(res, (scores[v], -v))
                if len(res) > ef:
                    heapq.heappop(res)
    out = sorted(res, key=lambda t: (-t[0], -t[1]))[:k]
    return [-i for _, i in out], visited


def _best_first_multi(scores, adj, seeds, ef, k):
    """The same textbook search started from several entry points (all of them in the candidate
    and result heaps from the start), as a hierarchical index runs it on every layer."""
    visited, cand, res = set(), [], []
    for s in seeds:
        if s in visited:
            continue
        visited.add(s)
        heapq.heappush(cand, (-scores[s], s))
        heapq.heappush(res, (scores[s], -s))
        if len(res) > ef:
            heapq.heappop(res)
    while cand:
        neg, c = heapq.heappop(cand)
        if len(res) >= ef and (-neg, -c) < res[0]:
            break
        for v in adj[c]:
            v = int(v)
            if v in visited:
                continue
            visited.add(v)
            if len(res) < ef or (scores[v], -v) > res[0]:
                heapq.heappush(cand, (-scores[v], v))
                heapq.heappush(res, (scores[v], -v))
                if len(res) > ef:
                    heapq.heappop(res)
    out = sorted(res, key=lambda t: (-t[0], -t[1]))[:k]
    return [-i for _, i in out]


def test_single_walker_is_classic_best_first_search():
    cfg = scaled(PRESETS["C1"], 2000, n_clusters=6, Q=16)
    wl = to_host(make_workload(cfg, seed=91))
    mlp = oracle.Mlp(wl["W"], wl["b"], wl["head_w"])
    N = 2000
    for L, k in ((8, 8), (24, 10), (64, 33)):
        r = oracle.search(wl["emb"], wl["adj"], wl["users"], mlp, wl["entries"], 1, L, k, 0, trace=True,
                          visited_cap=N)
        for q in range(cfg.Q):
            s = oracle.score_pairs(wl["emb"], wl["users"], mlp, np.full(N, q), np.arange(N)).astype(np.float64)
            ids, visited = _best_first(s, wl["adj"], int(wl["entries"][q, 0]), L, k)
            assert r["ids"][q].tolist() == (ids + [-1] * k)[:k]
            assert set(v for v in r["visited"][q].tolist() if v >= 0) == visited


# ----------------------------------------------------------------------------- symmetries
def test_entry_order_batch_order_and_threading_do_not_matter():
    cfg = scaled(PRESETS["C1"], 4000, n_clusters=8, Q=20)
    from dataclasses import replace

    cfg = replace(cfg, E=4)
    wl = to_host(make_workload(cfg, seed=5))
    mlp = oracle.Mlp(wl["W"], wl["b"], wl["head_w"])
    base = oracle.search(wl["emb"], wl["adj"], wl["users"], mlp, wl["entries"], 3, 20, 15, 0)
    # shared container: which seed found an item is irrelevant
    rev = oracle.search(wl["emb"], wl["adj"], wl["users"], mlp, wl["entries"][:, ::-1].copy(), 3, 20, 15, 0)
    assert np.array_equal(base["ids"], rev["ids"]) and np.array_equal(base["scores"], rev["scores"])
    # queries are independent
    perm = np.random.default_rng(1).permutation(cfg.Q)
    p = oracle.search(wl["emb"], wl["adj"], wl["users"][perm], mlp, wl["entries"][perm], 3, 20, 15, 0, n_threads=3)
    assert np.array_equal(base["ids"][perm], p["ids"])
    sub = oracle.search(wl["emb"], wl["adj"], wl["users"][:3], mlp, wl["entries"][:3], 3, 20, 15, 0)
    assert np.array_equal(base["ids"][:3], sub["ids"])


def test_relabelling_the_items_relabels_the_result():
    """The cluster-ordered labelling of the workload generator is the same problem: the search visits the same
    items in the same order (relevances are distinct, so the tie rule by id never decides)."""
    cfg = scaled(PRESETS["C1"], 3000, n_clusters=8, Q=10)
    a = make_workload(cfg, seed=13)
    b = make_workload(cfg, seed=13, contiguous_ids=True)
    relabel = b["relabel"].numpy()
    a, b = to_host(a), to_host(b)
    cluster = b["cluster"]
    assert np.all(cluster[1:] >= cluster[:-1])
    mlp = oracle.Mlp(a["W"], a["b"], a["head_w"])
    ra = oracle.search(a["emb"], a["adj"], a["users"], mlp, a["entries"], 3, 40, 15, 0, trace=True)
    rb = oracle.search(b["emb"], b["adj"], b["users"], mlp, b["entries"], 3, 40, 15, 0, trace=True)
    assert np.array_equal(relabel[ra["ids"]], rb["ids"]) and np.array_equal(ra["scores"], rb["scores"])
    assert np.array_equal(ra["n_scored"], rb["n_scored"])


def test_per_query_parameters_equal_separate_runs():
    cfg = scaled(PRESETS["C1"], 3000, n_clusters=8, Q=6)
    wl = to_host(make_workload(cfg, seed=8))
    mlp = oracle.Mlp(wl["W"], wl["b"], wl["head_w"])
    Wq = np.array([1, 2, 3, 4, 5, 16], np.int32)
    Lq = np.array([16, 40, 8, 64, 5, 33], np.int32)
    cq = np.array([0, 8, 3, 0, 64, 2], np.int32)
    r = oracle.search(wl["emb"], wl["adj"], wl["users"], mlp, wl["entries"], Wq, Lq, 12, cq)
    for q in range(6):
        one = oracle.search(wl["emb"], wl["adj"], wl["users"][q:q + 1], mlp, wl["entries"][q:q + 1],
                            int(Wq[q]), int(Lq[q]), 12, int(cq[q]))
        assert np.array_equal(one["ids"][0], r["ids"][q])


def test_more_search_effort_never_lowers_recall_on_average():
    # not an exact law per query, but on a batch recall grows from tiny L to L >= N (where it is 1)
    cfg = scaled(PRESETS["C1"], 1500, n_clusters=4, Q=24)
    wl = to_host(make_workload(cfg, seed=21))
    mlp = oracle.Mlp(wl["W"], wl["b"], wl["head_w"])
    bf = oracle.brute_force(wl["emb"], wl["users"], mlp, 10, n_threads=4)
    rec = []
    for L in (10, 200, 1500):
        r = oracle.search(wl["emb"], wl["adj"], wl["users"], mlp, wl["entries"], 2, L, 10, 0, n_threads=4)
        rec.append(oracle.recall_at(r["ids"], bf["ids"], 10))
    assert rec[0] <= rec[1] <= rec[2] == 1.0


def test_recall_definition():
    # Sec. 5.1.3: share of the true top-k among the first k returned
    found = np.array([[1, 2, 3, 4], [9, 8, -1, -1]], np.int32)
    truth = np.array([[4, 3, 7, 6], [8, 5, 9, 1]], np.int32)
    assert oracle.recall_at(found, truth, 4) == pytest.approx((2 + 2) / 8)
    assert oracle.recall_at(found, truth, 2) == pytest.approx((0 + 1) / 4)


def test_argument_checks():
    wl, mlp = _tiny(1)
    with pytest.raises(ValueError):
        oracle.search(wl["emb"], wl["adj"], wl["users"], mlp, wl["entries"], 0, 4, 4, 0)
    with pytest.raises(ValueError):
        oracle.search(wl["emb"], wl["adj"], wl["users"], mlp, wl["entries"], 1, 0, 4, 0)
    with pytest.raises(ValueError):
        oracle.search(wl["emb"], wl["adj"], wl["users"], mlp, wl["entries"], 1, 4, 0, 0)
