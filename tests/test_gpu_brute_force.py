"""ann_brute_force (the exhaustive search that the recall measure of Sec. 5.1.3 compares with) against the
oracle's brute force, through the C ABI.

fp32 metric: ids equal to the oracle's, in order, relevances to 1e-5.  16-bit metrics: the kernels' relevances
differ from the exact ones in the last bits, so near-ties may swap; what is unique is checked exactly (the
result is the top k of the device's own relevances, which ann_score_pairs returns for every item and whose
parity with the oracle has its own tests), and the agreement with the oracle is bounded."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_11490_amd as ann
from tests.gpu_util import open_handles, oracle_mlp
from workloads import PRESETS, make_workload, scaled, to_host

pytestmark = pytest.mark.gpu


def _device_top_k(g, m, users, N, k, rows):
    """Top k by (relevance descending, id ascending) of the relevances ann_score_pairs gives for every item."""
    ids = np.full((len(rows), k), -1, np.int32)
    sc = np.full((len(rows), k), -np.inf, np.float32)
    items = torch.arange(N, dtype=torch.int32, device="cuda")
    for r, q in enumerate(rows):
        s = ann.ann_score_pairs(g, m, users, torch.full((N,), q, dtype=torch.int32, device="cuda"), items).cpu().numpy()
        order = np.lexsort((np.arange(N), -s.astype(np.float64)))[:k]
        ids[r, :len(order)] = order
        sc[r, :len(order)] = s[order]
    return ids, sc


@pytest.mark.parametrize("N,Q,k", [(50, 3, 64), (700, 9, 25), (5000, 6, 100), (70001, 3, 100), (2100, 2, 2048)])
def test_brute_force_fp32_equals_oracle(N, Q, k):
    cfg = scaled(PRESETS["C1"], N, n_clusters=3, Q=Q)
    wl = make_workload(cfg, seed=N)
    g, m, dev = open_handles(wl)
    ids, sc = ann.ann_brute_force(g, m, dev["users"], k)
    h = to_host(wl)
    bf = oracle.brute_force(h["emb"], h["users"], oracle_mlp(h), k, n_threads=8)
    assert np.array_equal(ids.cpu().numpy(), bf["ids"])
    got = sc.cpu().numpy()
    held = bf["ids"] >= 0
    np.testing.assert_allclose(got[held], bf["scores"][held], rtol=1e-5)
    assert np.all(np.isneginf(got[~held])) and np.all(ids.cpu().numpy()[~held] == -1)


@pytest.mark.parametrize("preset,N,Q,k", [("C2", 3000, 5, 100), ("C3", 3000, 5, 100), ("C4", 3000, 5, 100),
                                          ("C3", 66000, 300, 50)])
def test_brute_force_16bit_is_the_top_k_of_the_kernels_relevances(preset, N, Q, k):
    """Several item chunks with a ragged last one (66,000 items) and several query blocks (300 queries of
    66,000 items are two blocks of pairs)."""
    cfg = scaled(PRESETS[preset], N, n_clusters=8, Q=Q)
    wl = make_workload(cfg, seed=11)
    g, m, dev = open_handles(wl)
    assert ann.ann_mlp_uses_mfma(m)
    ids, sc = ann.ann_brute_force(g, m, dev["users"], k)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    rows = sorted({0, 1, Q // 2, Q - 2, Q - 1})
    want_ids, want_sc = _device_top_k(g, m, dev["users"], N, k, rows)
    assert np.array_equal(ids[rows], want_ids)
    assert np.array_equal(sc[rows], want_sc)
    # against the oracle: exact relevances within the 16-bit budget, and nearly the same set
    h = to_host(wl)
    sub = rows[:3]
    users = np.ascontiguousarray(h["users"][sub])
    bf = oracle.brute_force(h["emb"], users, oracle_mlp(h), k, n_threads=8)
    exact = oracle.score_pairs(h["emb"], users, oracle_mlp(h), np.repeat(np.arange(len(sub)), k).astype(np.int32),
                               ids[sub].reshape(-1).astype(np.int32), n_threads=8).reshape(len(sub), k)
    assert np.max(np.abs(sc[sub] - exact)) <= 1e-2
    shared = np.mean([len(set(ids[q]) & set(bf["ids"][i])) / k for i, q in enumerate(sub)])
    assert shared >= 0.9, shared


def test_brute_force_rows_do_not_depend_on_the_batch():
    cfg = scaled(PRESETS["C2"], 4000, n_clusters=8, Q=40)
    wl = make_workload(cfg, seed=5)
    g, m, dev = open_handles(wl)
    ids, sc = ann.ann_brute_force(g, m, dev["users"], 30)
    part_ids, part_sc = ann.ann_brute_force(g, m, dev["users"][17:23].contiguous(), 30)
    assert torch.equal(ids[17:23], part_ids) and torch.equal(sc[17:23], part_sc)


def _reaches_everything(adj: np.ndarray, seeds) -> bool:
    seen = {int(v) for v in seeds if 0 <= v < adj.shape[0]}
    todo = list(seen)
    while todo:
        for w in adj[todo.pop()]:
            if int(w) not in seen:
                seen.add(int(w))
                todo.append(int(w))
    return len(seen) == adj.shape[0]


def test_brute_force_is_what_a_search_that_scores_everything_returns():
    """A list as long as the table: for every query whose seeds reach all items the search's result is the
    exhaustive one, id for id and bit for bit (same kernels, same order)."""
    N = 900
    cfg = scaled(PRESETS["C2"], N, n_clusters=4, Q=12)
    wl = make_workload(cfg, seed=8)
    g, m, dev = open_handles(wl)
    s_ids, s_sc = ann.ann_search(g, m, dev["users"], dev["entries"], 4, N, 40, 0)
    b_ids, b_sc = ann.ann_brute_force(g, m, dev["users"], 40)
    h = to_host(wl)
    full = [q for q in range(cfg.Q) if _reaches_everything(h["adj"], h["entries"][q])]
    assert len(full) >= cfg.Q // 2
    assert torch.equal(s_ids[full], b_ids[full]) and torch.equal(s_sc[full], b_sc[full])


def test_brute_force_argument_errors():
    cfg = scaled(PRESETS["C1"], 500, n_clusters=2, Q=4)
    wl = make_workload(cfg)
    g, m, dev = open_handles(wl)
    for k in (0, 2049):
        with pytest.raises(ann.AnnError):
            ann.ann_brute_force(g, m, dev["users"], k)
    with pytest.raises(ValueError):
        ann.ann_brute_force(g, m, dev["users"], 5, out_ids=torch.empty(4, 6, dtype=torch.int32, device="cuda"))


def test_brute_force_full_size_c3():
    """10 M items: 153 item chunks per query.  One query is checked id for id against the top k of the
    relevances ann_score_pairs gives for all 10 M items, the sample against the independent fp32 ranking and
    the returned relevances against the exact oracle."""
    import os
    import sys
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    from bench import recall_at, torch_ground_truth

    cfg = PRESETS["C3"]
    wl = make_workload(cfg, device="cuda:0")
    g = ann.ann_graph_load(wl["adj"], wl["emb"])
    m = ann.ann_mlp_load(wl["W"], wl["b"], wl["head_w"], cfg.d, ann.ANN_BF16)
    q_sel = [3, 1000, 4095] + list(range(2000, 2013))
    users = wl["users"][q_sel].contiguous()
    k = 100
    ids, sc = ann.ann_brute_force(g, m, users, k)
    want_ids, want_sc = _device_top_k(g, m, users, cfg.N, k, [0])
    assert np.array_equal(ids[:1].cpu().numpy(), want_ids) and np.array_equal(sc[:1].cpu().numpy(), want_sc)
    ids_h, sc_h = ids.cpu().numpy(), sc.cpu().numpy()
    assert np.all(sc_h[:, :-1] >= sc_h[:, 1:]) and ids_h.min() >= 0 and ids_h.max() < cfg.N
    truth = torch_ground_truth(wl, q_sel, k).cpu()
    agreement = recall_at(ids.cpu(), truth, k)
    print(f"exhaustive search in bf16 against the fp32 ranking: shared top-{k} {agreement:.4f}")
    assert agreement >= 0.95
    h = to_host({n: wl[n] for n in ("emb", "W", "b", "head_w")})
    hu = to_host({"users": users})
    exact = oracle.score_pairs(h["emb"], hu["users"], oracle.Mlp(h["W"], h["b"], h["head_w"]),
                               np.repeat(np.arange(len(q_sel)), k).astype(np.int32), ids_h.reshape(-1), n_threads=16)
    assert np.max(np.abs(sc_h.reshape(-1) - exact)) <= 1e-2


# ----------------------------------------------------------------------------- re-ranking of candidate lists
def _candidates(N, Q, n, seed, with_junk=True):
    rng = np.random.default_rng(seed)
    cand = np.stack([rng.choice(N, size=n, replace=False) for _ in range(Q)]).astype(np.int32)
    if with_junk and n >= 8:
        cand[:, 3] = -1           # the padding of a search result
        cand[0, 5] = N            # out of range
        cand[1 % Q, 6] = cand[1 % Q, 7]   # a repeated id
    if with_junk and n >= 2500 and Q > 2:
        cand[2, n // 2:] = cand[2, :n - n // 2]   # every id twice, far enough apart to meet a copy already merged
    return cand


@pytest.mark.parametrize("N,Q,n,k", [(900, 7, 40, 10), (5000, 5, 3000, 100), (5000, 3, 30, 64), (70000, 260, 65536, 20)])
def test_rerank_fp32_equals_oracle(N, Q, n, k):
    """The last case is two passes (260 queries of 65,536 candidates) at the largest n."""
    cfg = scaled(PRESETS["C1"], N, n_clusters=3, Q=Q)
    wl = make_workload(cfg, seed=N + n)
    g, m, dev = open_handles(wl)
    cand = _candidates(N, Q, n, seed=k)
    ids, sc = ann.ann_rerank(g, m, dev["users"], torch.from_numpy(cand).cuda(), k)
    h = to_host(wl)
    rows = list(range(Q)) if Q <= 16 else [0, 1, 2, 255, 256, 257, Q - 1]
    want = oracle.rerank(h["emb"], np.ascontiguousarray(h["users"][rows]), oracle_mlp(h), cand[rows], k, n_threads=8)
    got_ids, got_sc = ids.cpu().numpy()[rows], sc.cpu().numpy()[rows]
    assert np.array_equal(got_ids, want["ids"])
    held = want["ids"] >= 0
    np.testing.assert_allclose(got_sc[held], want["scores"][held], rtol=1e-5)
    assert np.all(np.isneginf(got_sc[~held]))


@pytest.mark.parametrize("preset", ["C2", "C3", "C4"])
def test_rerank_16bit_is_the_top_k_of_the_kernels_relevances(preset):
    N, Q, n, k = 20000, 6, 5000, 100
    cfg = scaled(PRESETS[preset], N, n_clusters=8, Q=Q)
    wl = make_workload(cfg, seed=17)
    g, m, dev = open_handles(wl)
    assert ann.ann_mlp_uses_mfma(m)
    cand = _candidates(N, Q, n, seed=2)
    cand_d = torch.from_numpy(cand).cuda()
    ids, sc = ann.ann_rerank(g, m, dev["users"], cand_d, k)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    for q in range(Q):
        ok = (cand[q] >= 0) & (cand[q] < N)
        c = cand[q][ok]
        s = ann.ann_score_pairs(g, m, dev["users"], torch.full((c.size,), q, dtype=torch.int32, device="cuda"),
                                torch.from_numpy(c).cuda()).cpu().numpy()
        order = np.lexsort((c, -s.astype(np.float64)))[:k]
        assert np.array_equal(ids[q], c[order]) and np.array_equal(sc[q], s[order])
    h = to_host(wl)
    want = oracle.rerank(h["emb"], h["users"], oracle_mlp(h), cand, k, n_threads=8)
    exact = oracle.score_pairs(h["emb"], h["users"], oracle_mlp(h), np.repeat(np.arange(Q), k).astype(np.int32),
                               ids.reshape(-1), n_threads=8).reshape(Q, k)
    assert np.max(np.abs(sc - exact)) <= 1e-2
    shared = np.mean([len(set(ids[q]) & set(want["ids"][q])) / len(set(want["ids"][q])) for q in range(Q)])
    assert shared >= 0.95, shared


def test_rerank_of_an_8bit_search_recovers_the_16bit_ranking():
    """Traversal under the 8-bit metric, its best 512 scored again under the 16-bit metric: the first 100 are
    then, up to a point of recall, those of the 16-bit search with the same parameters."""
    cfg = scaled(PRESETS["C3"], 200_000, n_clusters=256, Q=64)
    wl = make_workload(cfg, seed=23)
    g, m, dev = open_handles(wl)
    emb8 = ann.ann_quantize_e4m3(dev["emb"])
    g8 = ann.ann_graph_load(dev["adj"], emb8)
    m8 = ann.ann_mlp_load(wl["W"], wl["b"], wl["head_w"], cfg.d, ann.ANN_F8)
    W, L = 8, 1024
    ids16, _ = ann.ann_search(g, m, dev["users"], dev["entries"], W, L, 100, 0)
    ids8, _ = ann.ann_search(g8, m8, dev["users"], dev["entries"], W, L, 512, 0)
    ids_rr, sc_rr = ann.ann_rerank(g, m, dev["users"], ids8, 100)
    truth, _ = ann.ann_brute_force(g, m, dev["users"], 100)
    rec = lambda found: float(np.mean([len(set(a.tolist()) & set(b.tolist()) - {-1}) / 100
                                       for a, b in zip(found.cpu().numpy(), truth.cpu().numpy())]))
    r16, r8, rrr = rec(ids16), rec(ids8[:, :100]), rec(ids_rr)
    print(f"recall@100 against the 16-bit exhaustive ranking: 16-bit search {r16:.4f}, 8-bit search {r8:.4f}, "
          f"8-bit search re-ranked {rrr:.4f}")
    assert rrr >= r16 - 0.01 and rrr >= r8
    s = sc_rr.cpu().numpy()
    assert np.all(s[:, :-1] >= s[:, 1:])


def test_rerank_argument_errors():
    cfg = scaled(PRESETS["C1"], 500, n_clusters=2, Q=4)
    wl = make_workload(cfg)
    g, m, dev = open_handles(wl)
    cand = torch.zeros(4, 8, dtype=torch.int32, device="cuda")
    with pytest.raises(ann.AnnError):
        ann.ann_rerank(g, m, dev["users"], cand, 0)
    with pytest.raises(ann.AnnError):
        ann.ann_rerank(g, m, dev["users"], torch.zeros(4, 65537, dtype=torch.int32, device="cuda"), 5)
    with pytest.raises(ValueError):
        ann.ann_rerank(g, m, dev["users"], cand[:3].contiguous(), 5)
    with pytest.raises(TypeError):
        ann.ann_rerank(g, m, dev["users"], cand.long(), 5)


def test_caller_workspace_form_only_enqueues_and_gives_the_same_result():
    """With a caller's workspace the two calls allocate nothing, do not synchronise and return what the allocating
    form returns; a workspace that is too small is refused before anything runs."""
    cfg = scaled(PRESETS["C2"], 30000, n_clusters=8, Q=50)
    wl = make_workload(cfg, seed=31)
    g, m, dev = open_handles(wl)
    k, n = 40, 700
    cand = torch.from_numpy(_candidates(cfg.N, cfg.Q, n, seed=4)).cuda()
    want_b = ann.ann_brute_force(g, m, dev["users"], k)
    want_r = ann.ann_rerank(g, m, dev["users"], cand, k)
    ws_b = torch.empty(ann.ann_brute_force_workspace_bytes(g, m, cfg.Q, k), dtype=torch.uint8, device="cuda")
    ws_r = torch.empty(ann.ann_rerank_workspace_bytes(g, m, cfg.Q, n, k), dtype=torch.uint8, device="cuda")
    ids = torch.empty(cfg.Q, k, dtype=torch.int32, device="cuda")
    sc = torch.empty(cfg.Q, k, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    allocations = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]
    for _ in range(2):   # the workspace keeps the last call's contents: a second call must not see them
        before = allocations()
        ann.ann_brute_force(g, m, dev["users"], k, out_ids=ids, out_scores=sc, workspace=ws_b)
        assert allocations() == before
        torch.cuda.synchronize()
        assert torch.equal(ids, want_b[0]) and torch.equal(sc, want_b[1])
        before = allocations()
        ann.ann_rerank(g, m, dev["users"], cand, k, out_ids=ids, out_scores=sc, workspace=ws_r)
        assert allocations() == before
        torch.cuda.synchronize()
        assert torch.equal(ids, want_r[0]) and torch.equal(sc, want_r[1])
    with pytest.raises(ann.AnnError) as e:
        ann.ann_rerank(g, m, dev["users"], cand, k, workspace=ws_r[:4096])
    assert e.value.code == -5
