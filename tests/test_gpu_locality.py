"""ann_graph_set_locality: the visited bitmap addressed by a rank of the ids instead of the ids.  It may change
where a search keeps its bits and nothing else: every case compares the search with a rank (a random permutation,
the worst there is, and the order the generator package derives from the adjacency) with the same search without
one, id for id, relevance for relevance and counter for counter, and one case with the oracle."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_2502_11490_amd as ann
from tests.gpu_util import open_handles, oracle_mlp, same_list_fraction
from workloads import PRESETS, locality_rank, make_workload, scaled, to_host

pytestmark = pytest.mark.gpu


def _ranks(adj, seed):
    N = adj.shape[0]
    g = torch.Generator().manual_seed(seed)
    return {"random": torch.randperm(N, generator=g).to(torch.int32).cuda(),
            "graph": locality_rank(adj)[0].cuda()}


def _stats(ws):
    st = ann.ann_search_stats(ws)
    return (st.pairs_scored, st.nodes_expanded, st.max_query_iters, st.visited_overflow, st.queries)


@pytest.mark.parametrize("preset,W,L,k,E,cap", [("C1", 4, 64, 20, 3, 0), ("C1", 24, 300, 50, 5, 0), ("C1", 64, 2500, 100, 8, 0),
                                                ("C1", 128, 300, 50, 5, 3), ("C2", 8, 512, 100, 4, 0), ("C3", 40, 3000, 100, 8, 0)])
def test_search_with_a_locality_order_is_the_same_search(preset, W, L, k, E, cap, monkeypatch):
    """Short resident lists; 384, 1,024 (several filter pieces only with ranks beside the ids), 1,280 and 2,048
    candidates per round; the fp32 and the 16-bit kernels; seeds that are invalid or repeated."""
    monkeypatch.setenv("GMPGR_VISITED_SET", "bitmap")
    cfg = replace(scaled(PRESETS[preset], 6000, n_clusters=12, Q=48), E=E)
    wl = make_workload(cfg, seed=41)
    ent = wl["entries"].clone()
    ent[0, 0] = -1
    ent[1, E - 1] = ent[1, 0]
    ent[2, 0] = cfg.N
    wl["entries"] = ent
    g, m, dev = open_handles(wl)
    assert ann.ann_search_visited_set_is_bitmap(g, m, cfg.Q, E, W, L, k, cap)
    size = ann.ann_search_workspace_bytes(g, m, cfg.Q, E, W, L, k, cap)
    ws = torch.empty(size, dtype=torch.uint8, device="cuda")
    want_ids, want_sc = ann.ann_search(g, m, dev["users"], dev["entries"], W, L, k, cap, workspace=ws)
    want_ids, want_sc, want = want_ids.clone(), want_sc.clone(), _stats(ws)
    for name, rank in _ranks(wl["adj"], 5).items():
        ann.ann_graph_set_locality(g, rank)
        assert ann.ann_search_workspace_bytes(g, m, cfg.Q, E, W, L, k, cap) == size
        ids, sc = ann.ann_search(g, m, dev["users"], dev["entries"], W, L, k, cap, workspace=ws)
        assert torch.equal(ids, want_ids) and torch.equal(sc, want_sc), name
        assert _stats(ws) == want, name
    ann.ann_graph_set_locality(g, None)
    ids, sc = ann.ann_search(g, m, dev["users"], dev["entries"], W, L, k, cap, workspace=ws)
    assert torch.equal(ids, want_ids) and _stats(ws) == want
    if preset == "C1":   # and it is the oracle's search
        h = to_host(wl)
        ref = oracle.search(h["emb"], h["adj"], h["users"], oracle_mlp(h), h["entries"], W, L, k, cap, n_threads=8)
        assert same_list_fraction(want_ids.cpu().numpy(), ref["ids"]) >= 0.99


def test_locality_order_in_the_other_entry_points(monkeypatch):
    """Continuous batching (a slot's bitmap is cleared and re-seeded), per-query parameters and the walker rule."""
    monkeypatch.setenv("GMPGR_VISITED_SET", "bitmap")
    cfg = replace(scaled(PRESETS["C5"], 8000, n_clusters=16, Q=60), E=4)
    wl = make_workload(cfg, seed=43)
    g, m, dev = open_handles(wl)
    W, L, k = 6, 200, 40
    runs = {
        "stream": lambda: ann.ann_search_stream(g, m, dev["users"], dev["entries"], 9, W, L, k, 0),
        "ragged": lambda: ann.ann_search_ragged(g, m, dev["users"], dev["entries"], dev["W_q"], dev["L_q"], dev["cap_q"],
                                                cfg.W_range[1], cfg.L_range[1], k, cfg.cap_range[1]),
        "walkers": lambda: ann.ann_search_walkers(g, m, dev["users"], dev["entries"], 12, k),
    }
    want = {n: tuple(t.clone() for t in f()) for n, f in runs.items()}
    for name, rank in _ranks(wl["adj"], 6).items():
        ann.ann_graph_set_locality(g, rank)
        for n, f in runs.items():
            ids, sc = f()
            assert torch.equal(ids, want[n][0]) and torch.equal(sc, want[n][1]), (name, n)


def test_rank_must_be_a_permutation():
    cfg = scaled(PRESETS["C1"], 2000, n_clusters=4, Q=4)
    wl = make_workload(cfg)
    g, m, dev = open_handles(wl)
    good = torch.randperm(cfg.N).to(torch.int32).cuda()
    ann.ann_graph_set_locality(g, good)
    twice = good.clone()
    twice[7] = twice[8]
    beyond = good.clone()
    beyond[3] = cfg.N
    for bad in (twice, beyond):
        with pytest.raises(ann.AnnError) as e:
            ann.ann_graph_set_locality(g, bad)
        assert e.value.code == -1
    with pytest.raises(ValueError):
        ann.ann_graph_set_locality(g, good[:-1].contiguous())
    with pytest.raises(TypeError):
        ann.ann_graph_set_locality(g, good.long())
    assert not ann.ann_search_visited_set_is_bitmap(g, m, cfg.Q, cfg.E, 2, 16, 5, 0)   # a short list: the hash table
    with pytest.raises(ann.AnnError):
        ann.ann_search_visited_set_is_bitmap(g, m, cfg.Q, cfg.E, 0, 16, 5, 0)
    # a refused rank leaves the graph without one: the search still runs and gives the plain result
    ids, _ = ann.ann_search(g, m, dev["users"], dev["entries"], 2, 16, 5, 0)
    ann.ann_graph_set_locality(g, None)
    ids0, _ = ann.ann_search(g, m, dev["users"], dev["entries"], 2, 16, 5, 0)
    assert torch.equal(ids, ids0)
