"""A locality order of the items derived from the adjacency alone (input preparation: no arithmetic of the
retrieval method; plain torch, runs on whatever device the adjacency is on).

Edges between items of one community of the graph have common neighbours, the long-range edges have next to none.
Items joined by edges with at least `min_common` common neighbours are put into one group (label propagation with
pointer jumping over those edges, in both directions) and groups are numbered one after the other, so that the
members of a group get consecutive ranks.  Too low a threshold lets a few chance triangles chain the communities
together, too high a one splits them; the threshold is chosen by what the order is for: the number of 64-byte
lines of a one-bit-per-item bitmap that the entries of an adjacency row fall into, averaged over the rows.
The result is what ann_graph_set_locality takes: it changes where a search keeps its visited bits, not what it
returns."""
from __future__ import annotations

from typing import Optional, Tuple

import torch


def common_neighbour_counts(adj: torch.Tensor, chunk: int = 4096) -> torch.Tensor:
    """[N, R] uint8: for every edge (u, adj[u][j]) the number of ids the two adjacency rows share."""
    N, R = adj.shape
    a = adj.long().clamp(min=0, max=N - 1)
    out = torch.empty(N, R, dtype=torch.uint8, device=adj.device)
    for s in range(0, N, chunk):
        A = a[s:s + chunk]                      # [c, R]
        B = a[A]                                # [c, R, R]: the rows of the neighbours
        out[s:s + chunk] = (A[:, None, :, None] == B[:, :, None, :]).any(-1).sum(-1).to(torch.uint8)
    return out


def _groups(adj: torch.Tensor, counts: torch.Tensor, min_common: int) -> torch.Tensor:
    N = adj.shape[0]
    us, vs = [], []
    step = 1 << 22                               # rows at a time: a mask over all N * R entries at once may pass 2^31
    for s in range(0, N, step):
        a = adj[s:s + step].long()
        keep = (counts[s:s + step] >= min_common) & (a >= 0) & (a < N)
        us.append(torch.arange(s, s + a.shape[0], device=adj.device)[:, None].expand_as(a)[keep])
        vs.append(a[keep])
    u, v = torch.cat(us), torch.cat(vs)
    lab = torch.arange(N, device=adj.device)
    for _ in range(10_000):
        new = lab.clone()
        new.scatter_reduce_(0, u, lab[v], "amin")
        new.scatter_reduce_(0, v, lab[u], "amin")
        new = new[new]
        if torch.equal(new, lab):
            break
        lab = new
    return lab


def _rank_of(lab: torch.Tensor) -> torch.Tensor:
    N = lab.shape[0]
    order = torch.argsort(lab, stable=True)     # position -> id: groups by their smallest id, members by id
    rank = torch.empty(N, dtype=torch.long, device=lab.device)
    rank[order] = torch.arange(N, device=lab.device)
    return rank


def lines_per_row(adj: torch.Tensor, rank: torch.Tensor, line_bits: int = 512, chunk: int = 1 << 20) -> float:
    """Mean number of distinct bitmap lines (line_bits ranks each) that the entries of one adjacency row fall
    into: what a search pays per expanded node for its visited bits."""
    N, R = adj.shape
    total = 0
    shift = line_bits.bit_length() - 1
    for s in range(0, N, chunk):
        lines = rank[adj[s:s + chunk].long().clamp(min=0, max=N - 1)] >> shift
        srt = torch.sort(lines, dim=1).values
        total += int((srt[:, 1:] != srt[:, :-1]).sum()) + srt.shape[0]
    return total / N


def locality_rank(adj: torch.Tensor, min_common: Optional[int] = None, chunk: int = 4096) -> Tuple[torch.Tensor, dict]:
    """rank [N] int32 (a permutation of the ids) and a dict with the threshold used and what it achieves.
    Without a given threshold, the one whose order leaves an adjacency row in the fewest 64-byte bitmap lines."""
    N = adj.shape[0]
    counts = common_neighbour_counts(adj, chunk)
    best = None
    for t in ([min_common] if min_common is not None else [1, 2, 3, 4, 6, 8]):
        lab = _groups(adj, counts, t)
        rank = _rank_of(lab)
        cost = lines_per_row(adj, rank)
        if best is None or cost < best[0]:
            best = (cost, t, rank, lab)
    cost, t, rank, lab = best
    sizes = torch.bincount(torch.unique(lab, return_inverse=True)[1])
    info = {"min_common": int(t), "groups": int(sizes.numel()), "largest_group": int(sizes.max()),
            "bitmap_lines_per_row": round(cost, 2),
            "bitmap_lines_per_row_by_id": round(lines_per_row(adj, torch.arange(N, device=adj.device)), 2)}
    return rank.to(torch.int32), info
