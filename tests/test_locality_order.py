"""The locality order the generator package derives from an adjacency (workloads/locality.py): a permutation,
found from the graph alone, that puts the members of a community next to each other."""
import numpy as np
import torch

from workloads import PRESETS, locality_rank, make_workload, scaled
from workloads.locality import common_neighbour_counts, lines_per_row


def test_common_neighbour_counts_by_hand():
    # two triangles joined by one edge; rows padded with the node itself
    adj = torch.tensor([[1, 2, 0], [0, 2, 1], [0, 1, 3], [4, 5, 2], [3, 5, 4], [3, 4, 5]], dtype=torch.int32)
    c = common_neighbour_counts(adj)
    brute = [[len(set(adj[u].tolist()) & set(adj[int(v)].tolist())) for v in adj[u]] for u in range(6)]
    assert c.tolist() == brute


def test_two_cliques_become_two_runs_of_ranks():
    n = 40
    rows = []
    for u in range(2 * n):
        base = 0 if u < n else n
        rows.append([base + (u - base + j) % n for j in range(1, 9)])
    adj = torch.tensor(rows, dtype=torch.int32)
    adj[3, 0] = n + 5           # a few long-range edges between the two
    adj[n + 7, 1] = 2
    perm = torch.randperm(2 * n, generator=torch.Generator().manual_seed(1))
    inv = torch.empty_like(perm)
    inv[perm] = torch.arange(2 * n)
    shuffled = torch.empty_like(adj)
    shuffled[perm] = perm[adj.long()].to(torch.int32)        # the same graph under shuffled labels
    rank, info = locality_rank(shuffled)
    assert sorted(rank.tolist()) == list(range(2 * n)) and info["groups"] == 2
    side = (inv[torch.argsort(rank.long())] >= n).long()     # which clique each rank position belongs to
    assert int((side[1:] != side[:-1]).sum()) == 1


def test_order_of_a_clustered_workload_keeps_a_row_in_fewer_bitmap_lines():
    cfg = scaled(PRESETS["C2"], 60000, n_clusters=96, Q=4)
    wl = make_workload(cfg, seed=3)
    rank, info = locality_rank(wl["adj"])
    assert np.array_equal(np.sort(rank.numpy()), np.arange(cfg.N))
    by_id = lines_per_row(wl["adj"], torch.arange(cfg.N))
    assert info["bitmap_lines_per_row"] == round(lines_per_row(wl["adj"], rank.long()), 2)
    assert info["bitmap_lines_per_row"] < 0.7 * by_id
    # the hidden clusters are what it found, from the edges alone: along the order the cluster changes rarely
    cluster = wl["cluster"].long()[torch.argsort(rank.long())]
    assert int((cluster[1:] != cluster[:-1]).sum()) < cfg.N // 20
