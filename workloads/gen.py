"""Seeded synthetic workloads shaped like the paper's retrieval setting.

The paper searches a proximity graph over learned item embeddings with a small
multi-head MLP as the relevance metric (Sec. 3.1, Sec. 3.2).  Its data sets are
private, so every input here is synthetic and seeded:

* items: Gaussian mixture (cluster means ~N(0,1) per coordinate, isotropic
  noise sigma), cluster sizes uniform or Zipf;
* graph: fixed degree R, int32 adjacency; R/2 L2-nearest neighbours inside the
  item's own cluster plus R/2 uniform random long-range edges (no self loops,
  no repeats inside a row);
* item ids: a seeded random permutation of the cluster-sorted order, so that
  ids carry no locality;
* MLP: He-initialised affine layers ([out][in] row-major), zero biases, fixed
  head-combination weights;
* users ~N(0,1); optionally half of them near a few "hot" cluster means;
* entry points: E distinct uniform-random item ids per query.

Only input construction lives here; no scoring and no search.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

SEED_BASE = 250211490
# seed streams: +1 means, +2 assignments, +3 noise, +4 random edges, +5 id permutation,
# +6 MLP, +7 users, +8 entry points, +9 per-query W/L/caps


@dataclass(frozen=True)
class Config:
    name: str
    N: int
    d: int
    dtype: str  # "f32" | "bf16"
    n_clusters: int
    R: int
    hidden: Tuple[int, ...]
    head_w: Tuple[float, ...]
    Q: int
    E: int
    W: int
    L: int
    k: int
    sigma: float = 0.3
    zipf_s: float = 0.0  # 0 = uniform cluster sizes
    ragged: bool = False  # per-query W / L / iteration caps
    hot_clusters: int = 0  # >0: half of the users sit near this many cluster means
    L_range: Tuple[int, int] = (16, 256)
    W_range: Tuple[int, int] = (1, 16)
    cap_range: Tuple[int, int] = (8, 64)

    @property
    def J(self) -> int:
        return len(self.head_w)

    @property
    def dims(self) -> Tuple[int, ...]:
        return (2 * self.d,) + tuple(self.hidden) + (self.J,)


W3 = (0.5, 0.3, 0.2)
W4 = (0.4, 0.3, 0.2, 0.1)

PRESETS: Dict[str, Config] = {
    "C1": Config("C1", 10_000, 32, "f32", 16, 16, (64,), W3, 64, 1, 2, 32, 10),
    "C2": Config("C2", 1_000_000, 64, "bf16", 1024, 32, (256, 128), W3, 1024, 4, 4, 64, 100),
    "C3": Config("C3", 10_000_000, 128, "bf16", 16384, 32, (512, 256), W4, 4096, 8, 8, 128, 200),
    "C4": Config("C4", 100_000_000, 64, "bf16", 65536, 32, (256,), W3, 16384, 4, 4, 64, 100),
    "C5": Config("C5", 10_000_000, 64, "bf16", 8192, 32, (256, 128), W3, 8192, 4, 8, 128, 100,
                 zipf_s=1.1, ragged=True, hot_clusters=10),
}


def scaled(cfg: Config, N: int, n_clusters: Optional[int] = None, Q: Optional[int] = None,
           name: Optional[str] = None) -> Config:
    """Same recipe at a smaller item count (keeps items-per-cluster when n_clusters is None)."""
    if n_clusters is None:
        n_clusters = max(1, int(round(cfg.n_clusters * N / cfg.N)))
    return replace(cfg, N=N, n_clusters=n_clusters, Q=cfg.Q if Q is None else Q,
                   name=name or f"{cfg.name}@{N}")


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _round_dtype(x: torch.Tensor, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return x.to(torch.bfloat16)
    if dtype == "f32":
        return x.to(torch.float32)
    raise ValueError(f"dtype {dtype!r}")


def random_mlp(dims: Sequence[int], seed: int, dtype: str = "f32", bias_scale: float = 0.0,
               device="cpu") -> Tuple[List[torch.Tensor], List[torch.Tensor]]:
    """He-initialised layers W[l] ~ N(0, 2/fan_in), shape [dims[l+1], dims[l]]; biases
    bias_scale * N(0,1) in fp32 (zero by default)."""
    g = _gen(device, seed)
    Ws, bs = [], []
    for l in range(len(dims) - 1):
        fan_in, fan_out = dims[l], dims[l + 1]
        w = torch.randn(fan_out, fan_in, generator=g, device=device) * math.sqrt(2.0 / fan_in)
        b = torch.randn(fan_out, generator=g, device=device) * bias_scale
        Ws.append(_round_dtype(w, dtype).contiguous())
        bs.append(b.to(torch.float32).contiguous())
    return Ws, bs


def _cluster_assign(cfg: Config, device, seed: int) -> torch.Tensor:
    g = _gen(device, seed + 2)
    if cfg.zipf_s > 0:
        ranks = torch.arange(1, cfg.n_clusters + 1, device=device, dtype=torch.float64)
        p = ranks.pow(-cfg.zipf_s)
        p = (p / p.sum()).to(torch.float32)
        out = torch.empty(cfg.N, dtype=torch.int64, device=device)
        step = 1 << 22
        for s in range(0, cfg.N, step):
            n = min(step, cfg.N - s)
            out[s:s + n] = torch.multinomial(p, n, replacement=True, generator=g)
        return out
    return torch.randint(0, cfg.n_clusters, (cfg.N,), generator=g, device=device)


def _knn_in_clusters(x: torch.Tensor, starts: torch.Tensor, counts: torch.Tensor, K: int,
                     budget: int = 1 << 26) -> torch.Tensor:
    """x: [N,d] fp32 in cluster-sorted order.  Returns [N,K] int64 positions of the K
    L2-nearest other members of each item's cluster (-1 where the cluster is too small)."""
    N, d = x.shape
    dev = x.device
    out = torch.full((N, K), -1, dtype=torch.int64, device=dev)
    sq = (x * x).sum(1)
    order = torch.argsort(counts)
    cs = counts[order].tolist()
    ss = starts[order].tolist()
    i, C = 0, len(cs)
    while i < C:
        if cs[i] == 0:
            i += 1
            continue
        if cs[i] > 4096:
            # one big cluster at a time, row-chunked
            s0, n = ss[i], cs[i]
            xb = x[s0:s0 + n]
            sqb = sq[s0:s0 + n]
            rows = max(1, (budget << 3) // n)  # a few GB of distances at a time on the big clusters
            for r0 in range(0, n, rows):
                r1 = min(n, r0 + rows)
                dist = sqb[r0:r1, None] + sqb[None, :] - 2.0 * (xb[r0:r1] @ xb.T)
                ar = torch.arange(r0, r1, device=dev)
                dist[ar - r0, ar] = float("inf")
                kk = min(K, n - 1)
                if kk > 0:
                    idx = torch.topk(dist, kk, dim=1, largest=False).indices
                    out[s0 + r0:s0 + r1, :kk] = idx + s0
            i += 1
            continue
        # batch of small clusters, padded to the largest in the batch
        j = i
        P = max(cs[i], K + 1)
        while j < C and cs[j] <= 4096:
            Pn = max(cs[j], K + 1)
            if (j - i + 1) * Pn * Pn > budget and j > i:
                break
            P = Pn
            j += 1
        B = j - i
        st = torch.tensor(ss[i:j], device=dev, dtype=torch.int64)
        ct = torch.tensor(cs[i:j], device=dev, dtype=torch.int64)
        ar = torch.arange(P, device=dev, dtype=torch.int64)
        valid = ar[None, :] < ct[:, None]  # [B,P]
        pos = (st[:, None] + ar[None, :]).clamp_(max=N - 1)
        xb = x[pos]  # [B,P,d]
        sqb = sq[pos]
        dist = sqb[:, :, None] + sqb[:, None, :] - 2.0 * torch.bmm(xb, xb.transpose(1, 2))
        dist.masked_fill_(~valid[:, None, :], float("inf"))
        dist[:, ar, ar] = float("inf")
        top = torch.topk(dist, K, dim=2, largest=False)
        idx = top.indices + st[:, None, None]
        idx = torch.where(torch.isinf(top.values), torch.full_like(idx, -1), idx)
        out[pos[valid]] = idx[valid]
        i = j
    return out


def _build_graph(x_sorted: torch.Tensor, starts, counts, R: int, seed: int) -> torch.Tensor:
    N = x_sorted.shape[0]
    dev = x_sorted.device
    K = R // 2
    adj = torch.full((N, R), -1, dtype=torch.int64, device=dev)
    adj[:, :K] = _knn_in_clusters(x_sorted, starts, counts, K)
    g = _gen(dev, seed + 4)
    _fill_random_edges(adj, g)
    return adj


def _fill_random_edges(adj: torch.Tensor, gen: torch.Generator, chunk: int = 1 << 20) -> None:
    """adj: [N,R] int64 with -1 where a uniform random edge is wanted.  Fills those slots in
    place so that no row holds its own index or a repeated value; the slots that already
    hold a neighbour are never changed."""
    N, R = adj.shape
    dev = adj.device
    if N <= R:
        raise ValueError("need N > R for rows without repeats or self loops")
    for s in range(0, N, chunk):
        e = min(N, s + chunk)
        a = adj[s:e]
        rows = torch.arange(s, e, device=dev)[:, None]
        is_random = a < 0  # slots this routine owns
        need = is_random.clone()
        for _ in range(256):
            n_need = int(need.sum())
            if n_need == 0:
                break
            a[need] = torch.randint(0, N, (n_need,), generator=gen, device=dev)
            # flag every copy of a repeated value except the first in slot order
            srt, perm = torch.sort(a, dim=1, stable=True)
            dup_sorted = torch.zeros_like(a, dtype=torch.bool)
            dup_sorted[:, 1:] = srt[:, 1:] == srt[:, :-1]
            dup = torch.zeros_like(dup_sorted)
            dup.scatter_(1, perm, dup_sorted)
            need = (dup | (a == rows)) & is_random
        else:
            raise RuntimeError("random edge fill did not converge")


def make_workload(cfg: Config, device="cpu", seed: int = SEED_BASE, with_graph: bool = True,
                  contiguous_ids: bool = False) -> Dict:
    """Builds every input of one configuration on `device`.

    contiguous_ids: the same items, graph, users and seeds with the items labelled in cluster order (the members
    of a cluster have consecutive ids) instead of by the seeded random permutation; `relabel` [N] int64 then
    maps an id of the standard labelling to the id of the same item here.  A variant for measurements of what
    id locality is worth; every test and the timed step use the standard labelling.

    Returns a dict of torch tensors:
      emb [N,d] (f32|bf16), adj [N,R] int32, W (list, f32|bf16), b (list, f32), head_w [J] f32,
      users [Q,d] (f32|bf16), entries [Q,E] int32, and for ragged configs W_q, L_q, cap_q [Q] int32.
    """
    dev = torch.device(device)
    N, d = cfg.N, cfg.d
    means = torch.randn(cfg.n_clusters, d, generator=_gen(dev, seed + 1), device=dev)
    assign = _cluster_assign(cfg, dev, seed)
    assign_sorted, _ = torch.sort(assign)
    counts = torch.bincount(assign_sorted, minlength=cfg.n_clusters)
    starts = torch.cumsum(counts, 0) - counts
    g_noise = _gen(dev, seed + 3)
    x = torch.empty(N, d, dtype=torch.float32, device=dev)
    step = 1 << 20
    for s in range(0, N, step):
        e = min(N, s + step)
        x[s:e] = means[assign_sorted[s:e]] + cfg.sigma * torch.randn(e - s, d, generator=g_noise, device=dev)
    perm = torch.randperm(N, generator=_gen(dev, seed + 5), device=dev)  # position -> id
    out: Dict = {"cfg": cfg, "seed": seed}
    relabel = None
    if contiguous_ids:
        relabel = torch.empty(N, dtype=torch.int64, device=dev)
        relabel[perm] = torch.arange(N, device=dev)  # standard id -> position = id in this labelling
        perm = torch.arange(N, device=dev)
        out["relabel"] = relabel
    if with_graph:
        adj_pos = _build_graph(x, starts, counts, cfg.R, seed)  # positions
        adj = torch.empty(N, cfg.R, dtype=torch.int32, device=dev)
        for s in range(0, N, step):
            e = min(N, s + step)
            adj[perm[s:e]] = perm[adj_pos[s:e]].to(torch.int32)
        del adj_pos
        out["adj"] = adj
    emb = torch.empty(N, d, dtype=torch.bfloat16 if cfg.dtype == "bf16" else torch.float32, device=dev)
    emb[perm] = _round_dtype(x, cfg.dtype)
    del x
    out["emb"] = emb
    cluster_of_id = torch.empty(N, dtype=torch.int32, device=dev)
    cluster_of_id[perm] = assign_sorted.to(torch.int32)
    out["cluster"] = cluster_of_id

    Ws, bs = random_mlp(cfg.dims, seed + 6, cfg.dtype, 0.0, dev)
    out["W"], out["b"] = Ws, bs
    out["head_w"] = torch.tensor(cfg.head_w, dtype=torch.float32, device=dev)
    out["dims"] = list(cfg.dims)

    g_u = _gen(dev, seed + 7)
    users = torch.randn(cfg.Q, d, generator=g_u, device=dev)
    if cfg.hot_clusters > 0:
        half = cfg.Q // 2
        hot = torch.randint(0, cfg.hot_clusters, (half,), generator=g_u, device=dev)
        # hot clusters = the most populated ones
        big = torch.argsort(counts, descending=True)[: cfg.hot_clusters]
        users[:half] = means[big[hot]] + cfg.sigma * torch.randn(half, d, generator=g_u, device=dev)
    out["users"] = _round_dtype(users, cfg.dtype).contiguous()

    g_e = _gen(dev, seed + 8)
    ent = torch.randint(0, N, (cfg.Q, cfg.E), generator=g_e, device=dev)
    for _ in range(256):
        srt, p = torch.sort(ent, dim=1, stable=True)
        dup_s = torch.zeros_like(ent, dtype=torch.bool)
        dup_s[:, 1:] = srt[:, 1:] == srt[:, :-1]
        dup = torch.zeros_like(dup_s)
        dup.scatter_(1, p, dup_s)
        n = int(dup.sum())
        if n == 0:
            break
        ent[dup] = torch.randint(0, N, (n,), generator=g_e, device=dev)
    if relabel is not None:
        ent = relabel[ent]
    out["entries"] = ent.to(torch.int32).contiguous()

    if cfg.ragged:
        g_r = _gen(dev, seed + 9)
        out["L_q"] = torch.randint(cfg.L_range[0], cfg.L_range[1] + 1, (cfg.Q,), generator=g_r, device=dev).to(torch.int32)
        out["W_q"] = torch.randint(cfg.W_range[0], cfg.W_range[1] + 1, (cfg.Q,), generator=g_r, device=dev).to(torch.int32)
        out["cap_q"] = torch.randint(cfg.cap_range[0], cfg.cap_range[1] + 1, (cfg.Q,), generator=g_r, device=dev).to(torch.int32)
    return out


def _knn_global(x: torch.Tensor, K: int, budget: int = 1 << 27) -> torch.Tensor:
    """x: [n,d] fp32.  [n,K] int64 indices of the K L2-nearest other rows, by exhaustive distances."""
    n = x.shape[0]
    dev = x.device
    sq = (x * x).sum(1)
    out = torch.empty((n, K), dtype=torch.int64, device=dev)
    rows = max(1, budget // n)
    for r0 in range(0, n, rows):
        r1 = min(n, r0 + rows)
        dist = sq[r0:r1, None] + sq[None, :] - 2.0 * (x[r0:r1] @ x.T)
        ar = torch.arange(r0, r1, device=dev)
        dist[ar - r0, ar] = float("inf")
        out[r0:r1] = torch.topk(dist, K, dim=1, largest=False).indices
    return out


def layer_sizes(N: int, n_layers: int, growth: int, R: int) -> List[int]:
    """Item counts of the nested layers, coarsest first: each layer `growth` times the one above
    (the paper's fourth table, the appendix table of HNSW layer sizes: four layers, about 17x per layer); layers too small to give every
    node R distinct neighbours are left out."""
    sizes = [-(-N // growth ** (n_layers - 1 - l)) for l in range(n_layers)]
    return [n for n in sizes if n > R]


def make_layers(wl: Dict, n_layers: int = 4, growth: int = 17) -> Dict:
    """Nested graphs over the workload's items for the layer-by-layer search: layer l holds the
    items with ids 0 .. sizes[l] - 1 (ids are a random permutation, so this is a uniform sample,
    as the level draw of an HNSW index gives), the base layer is the workload's own graph.  An
    upper layer has the same recipe as the base layer, R/2 L2-nearest neighbours + R/2 uniform
    random ones without repeats or self loops; where a layer is too sparse for in-cluster
    neighbours (fewer than R + 2 items per cluster on average) the nearest neighbours are taken
    among all items of the layer.  Returns {"sizes", "adjs" (int32, coarsest first), "entries"
    [Q,E] int32 distinct ids of the coarsest layer}."""
    cfg = wl["cfg"]
    seed = wl["seed"]
    dev = wl["emb"].device
    R, K = cfg.R, cfg.R // 2
    sizes = layer_sizes(cfg.N, n_layers, growth, R)
    adjs = []
    for l, n in enumerate(sizes[:-1]):
        x = wl["emb"][:n].to(torch.float32)
        adj = torch.full((n, R), -1, dtype=torch.int64, device=dev)
        if n >= cfg.n_clusters * (R + 2):
            cl = wl["cluster"][:n].to(torch.int64)
            order = torch.argsort(cl, stable=True)  # position -> id
            counts = torch.bincount(cl, minlength=cfg.n_clusters)
            starts = torch.cumsum(counts, 0) - counts
            pos = _knn_in_clusters(x[order], starts, counts, K)
            ids = torch.where(pos >= 0, order[pos.clamp(min=0)], pos)
            adj[order, :K] = ids
        else:
            adj[:, :K] = _knn_global(x, K)
        _fill_random_edges(adj, _gen(dev, seed + 20 + l))
        adjs.append(adj.to(torch.int32).contiguous())
    adjs.append(wl["adj"])
    g_e = _gen(dev, seed + 19)
    E = min(cfg.E, sizes[0])
    if sizes[0] <= 8192:  # distinct ids per query: the E smallest of sizes[0] random keys
        ent = torch.rand(cfg.Q, sizes[0], generator=g_e, device=dev).topk(E, dim=1, largest=False).indices
    else:                 # repeats are possible and harmless (a repeated seed is ignored)
        ent = torch.randint(0, sizes[0], (cfg.Q, E), generator=g_e, device=dev)
    return {"sizes": sizes, "adjs": adjs, "entries": ent.to(torch.int32).contiguous()}


def _np(t: torch.Tensor) -> np.ndarray:
    t = t.detach().to("cpu").contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def to_host(wl: Dict) -> Dict:
    """Host copies as numpy arrays; bf16 tensors become uint16 arrays holding the raw bits."""
    out = {}
    for key, v in wl.items():
        if isinstance(v, torch.Tensor):
            out[key] = _np(v)
        elif isinstance(v, list) and v and isinstance(v[0], torch.Tensor):
            out[key] = [_np(t) for t in v]
        else:
            out[key] = v
    return out
