"""CPU oracle (test infrastructure): ctypes front end of gmp_oracle.c.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may import
this package.  It shares nothing with the HIP library.  The wrapper marshals
arguments (numpy arrays, bf16 passed as raw uint16 bits) and does no arithmetic
of the method itself; weights in bf16 are widened to fp32, which is exact.
Two functions are written out here rather than in C, each a few lines over the
C routines: search_layers (a loop of searches, one per layer) and rerank
(relevances by score_pairs, then numpy's lexsort for the search's order; pinned
to brute_force in tests/test_oracle_search.py).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gmp_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile gmp_oracle.c with gcc -O2 -fopenmp into oracle/liboracle.so."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
        for name in ("oracle_score_pairs", "oracle_search", "oracle_search_walkers", "oracle_brute_force",
                     "oracle_users_add_noise"):
            getattr(_lib, name).restype = ctypes.c_int
        _lib.oracle_e4m3_encode.restype = ctypes.c_int64
        _lib.oracle_e4m3_quantize.restype = ctypes.c_int64
        _lib.oracle_noise_element.restype = ctypes.c_double
        _lib.oracle_philox4x32_10.restype = None
        _lib.oracle_f16_round.restype = None
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> the same values as fp32 (exact)."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _as_f32(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return widen_bf16(a)
    # fp16 arrays widen exactly too (the cast below); they are then ordinary fp32 inputs
    return np.ascontiguousarray(a, dtype=np.float32)


class Mlp:
    """Flat fp32 copy of the layers: W[l] is [dims[l+1], dims[l]] row-major."""

    def __init__(self, W: Sequence[np.ndarray], b: Sequence[np.ndarray], head_w: np.ndarray):
        self.n_layers = len(W)
        dims = [int(W[0].shape[1])] + [int(w.shape[0]) for w in W]
        for l, w in enumerate(W):
            assert w.shape == (dims[l + 1], dims[l]), "layer shapes must chain"
            assert b[l].shape == (dims[l + 1],)
        assert len(head_w) == dims[-1]
        self.dims = np.asarray(dims, dtype=np.int32)
        self.W = np.concatenate([_as_f32(w).ravel() for w in W]).astype(np.float32)
        self.b = np.concatenate([_as_f32(x).ravel() for x in b]).astype(np.float32)
        self.head_w = np.ascontiguousarray(head_w, dtype=np.float32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _table(a: np.ndarray):
    """(array, dtype code) for an embedding / user table given as fp32 or raw bf16 bits."""
    if a.dtype == np.uint16:
        return np.ascontiguousarray(a), BF16
    return np.ascontiguousarray(a, dtype=np.float32), F32   # fp16 tables widen exactly


def score_pairs(emb: np.ndarray, users: np.ndarray, mlp: Mlp, q_idx: np.ndarray, item: np.ndarray,
                act_round: int = 0, n_threads: int = 1) -> np.ndarray:
    lib = _load()
    emb, dt = _table(emb)
    users, dtu = _table(users)
    assert dt == dtu, "users and items must share a dtype"
    q_idx = np.ascontiguousarray(q_idx, dtype=np.int32)
    item = np.ascontiguousarray(item, dtype=np.int32)
    M = q_idx.shape[0]
    out = np.empty(M, dtype=np.float32)
    rc = lib.oracle_score_pairs(
        _ptr(emb), dt, ctypes.c_int64(emb.shape[0]), int(emb.shape[1]), _ptr(users),
        int(users.shape[1]), ctypes.c_int64(users.shape[0]), mlp.n_layers, _ptr(mlp.dims),
        _ptr(mlp.W), _ptr(mlp.b), _ptr(mlp.head_w), int(act_round), ctypes.c_int64(M),
        _ptr(q_idx), _ptr(item), _ptr(out), int(n_threads))
    if rc != 0:
        raise ValueError(f"oracle_score_pairs failed rc={rc}")
    return out


def _per_query(v, Q: int) -> np.ndarray:
    a = np.asarray(v, dtype=np.int32)
    if a.ndim == 0:
        a = np.full(Q, int(a), dtype=np.int32)
    assert a.shape == (Q,)
    return np.ascontiguousarray(a)


def search(emb: np.ndarray, adj: np.ndarray, users: np.ndarray, mlp: Mlp, entries: np.ndarray,
           W, L, k: int, max_iters=0, act_round: int = 0, n_threads: int = 1,
           trace: bool = False, visited_cap: int = 0, trace_cap: int = 0) -> Dict:
    """Runs the synchronous search for every query.  W, L, max_iters: scalars or [Q] arrays.
    Returns ids [Q,k], scores [Q,k] and, with trace=True, n_scored / n_expanded / n_iters,
    visited [Q,visited_cap] and worst [Q,trace_cap]."""
    lib = _load()
    emb, dt = _table(emb)
    users, dtu = _table(users)
    assert dt == dtu
    adj = np.ascontiguousarray(adj, dtype=np.int32)
    entries = np.ascontiguousarray(entries, dtype=np.int32)
    Q, E = entries.shape
    assert users.shape[0] == Q
    Wq, Lq, cq = _per_query(W, Q), _per_query(L, Q), _per_query(max_iters, Q)
    ids = np.empty((Q, k), dtype=np.int32)
    scores = np.empty((Q, k), dtype=np.float32)
    n_scored = np.zeros(Q, dtype=np.int64) if trace else None
    n_expanded = np.zeros(Q, dtype=np.int64) if trace else None
    n_iters = np.zeros(Q, dtype=np.int32) if trace else None
    visited = np.empty((Q, visited_cap), dtype=np.int32) if trace and visited_cap > 0 else None
    worst = np.empty((Q, trace_cap), dtype=np.float32) if trace and trace_cap > 0 else None
    rc = lib.oracle_search(
        _ptr(emb), dt, ctypes.c_int64(emb.shape[0]), int(emb.shape[1]), _ptr(adj),
        int(adj.shape[1]), _ptr(users), int(users.shape[1]), ctypes.c_int64(Q), mlp.n_layers,
        _ptr(mlp.dims), _ptr(mlp.W), _ptr(mlp.b), _ptr(mlp.head_w), int(act_round),
        _ptr(entries), int(E), _ptr(Wq), _ptr(Lq), _ptr(cq), int(k), _ptr(ids), _ptr(scores),
        _ptr(n_scored), _ptr(n_expanded), _ptr(n_iters), _ptr(visited),
        ctypes.c_int64(visited_cap if visited is not None else 0), _ptr(worst),
        int(trace_cap if worst is not None else 0), int(n_threads))
    if rc != 0:
        raise ValueError(f"oracle_search failed rc={rc}")
    out = {"ids": ids, "scores": scores}
    if trace:
        out.update(n_scored=n_scored, n_expanded=n_expanded, n_iters=n_iters, visited=visited,
                   worst=worst)
    return out


def search_walkers(emb: np.ndarray, adj: np.ndarray, users: np.ndarray, mlp: Mlp, entries: np.ndarray,
                   T: int, k: int, act_round: int = 0, n_threads: int = 1, trace: bool = False,
                   visited_cap: int = 0) -> Dict:
    """Paper-literal inter-candidate search (Algorithm 1 read as independent walkers): one walker
    per seed, T greedy hops each (a walker moves to the best of the neighbours it has newly scored
    and dies when it has none), one shared visited set and one shared result list per query.
    Returns ids [Q,k], scores [Q,k] and, with trace=True, n_scored / n_expanded / n_iters and
    visited [Q,visited_cap]."""
    lib = _load()
    emb, dt = _table(emb)
    users, dtu = _table(users)
    assert dt == dtu
    adj = np.ascontiguousarray(adj, dtype=np.int32)
    entries = np.ascontiguousarray(entries, dtype=np.int32)
    Q, E = entries.shape
    assert users.shape[0] == Q
    ids = np.empty((Q, k), dtype=np.int32)
    scores = np.empty((Q, k), dtype=np.float32)
    n_scored = np.zeros(Q, dtype=np.int64) if trace else None
    n_expanded = np.zeros(Q, dtype=np.int64) if trace else None
    n_iters = np.zeros(Q, dtype=np.int32) if trace else None
    visited = np.empty((Q, visited_cap), dtype=np.int32) if trace and visited_cap > 0 else None
    rc = lib.oracle_search_walkers(
        _ptr(emb), dt, ctypes.c_int64(emb.shape[0]), int(emb.shape[1]), _ptr(adj),
        int(adj.shape[1]), _ptr(users), int(users.shape[1]), ctypes.c_int64(Q), mlp.n_layers,
        _ptr(mlp.dims), _ptr(mlp.W), _ptr(mlp.b), _ptr(mlp.head_w), int(act_round),
        _ptr(entries), int(E), int(T), int(k), _ptr(ids), _ptr(scores), _ptr(n_scored),
        _ptr(n_expanded), _ptr(n_iters), _ptr(visited),
        ctypes.c_int64(visited_cap if visited is not None else 0), int(n_threads))
    if rc != 0:
        raise ValueError(f"oracle_search_walkers failed rc={rc}")
    out = {"ids": ids, "scores": scores}
    if trace:
        out.update(n_scored=n_scored, n_expanded=n_expanded, n_iters=n_iters, visited=visited)
    return out


def search_layers(emb: np.ndarray, adjs, users: np.ndarray, mlp: Mlp, entries: np.ndarray,
                  W_l, L_l, K_l, max_iters=0, act_round: int = 0, n_threads: int = 1,
                  trace: bool = False) -> Dict:
    """Layer-by-layer search (Sec. 3.2; the outer loop over HNSW layers of Algorithm 1): adjs[l]
    is the graph of layer l over the items 0 .. len(adjs[l]) - 1, coarsest layer first; the
    K_l[l] items a layer returns, in rank order, are the seeds of the next layer, which starts
    from an empty candidate list and an empty visited set.  Returns the last layer's result
    and, with trace=True, `layers`: the per-layer results (ids, scores, n_scored, ...)."""
    assert len(adjs) == len(W_l) == len(L_l) == len(K_l) >= 1
    seeds = np.ascontiguousarray(entries, dtype=np.int32)
    layers = []
    for adj, W, L, K in zip(adjs, W_l, L_l, K_l):
        n = adj.shape[0]
        res = search(emb[:n], adj, users, mlp, seeds, W, L, int(K), max_iters=max_iters,
                     act_round=act_round, n_threads=n_threads, trace=trace)
        layers.append(res)
        seeds = res["ids"]      # padding (-1) is an absent seed for the next layer
    out = dict(layers[-1])
    if trace:
        out["layers"] = layers
        out["n_scored"] = sum(r["n_scored"] for r in layers)
        out["n_expanded"] = sum(r["n_expanded"] for r in layers)
    return out


def brute_force(emb: np.ndarray, users: np.ndarray, mlp: Mlp, k: int, act_round: int = 0,
                n_threads: int = 1) -> Dict:
    lib = _load()
    emb, dt = _table(emb)
    users, dtu = _table(users)
    assert dt == dtu
    Q = users.shape[0]
    ids = np.empty((Q, k), dtype=np.int32)
    scores = np.empty((Q, k), dtype=np.float32)
    rc = lib.oracle_brute_force(
        _ptr(emb), dt, ctypes.c_int64(emb.shape[0]), int(emb.shape[1]), _ptr(users),
        int(users.shape[1]), ctypes.c_int64(Q), mlp.n_layers, _ptr(mlp.dims), _ptr(mlp.W),
        _ptr(mlp.b), _ptr(mlp.head_w), int(act_round), int(k), _ptr(ids), _ptr(scores),
        int(n_threads))
    if rc != 0:
        raise ValueError(f"oracle_brute_force failed rc={rc}")
    return {"ids": ids, "scores": scores}


def rerank(emb: np.ndarray, users: np.ndarray, mlp: Mlp, cand: np.ndarray, k: int, act_round: int = 0,
           n_threads: int = 1) -> Dict:
    """The k most relevant of each query's candidates cand [Q][n] (relevance of Eq. 5-8 by score_pairs, then the
    search's order: relevance descending, equal relevances by ascending id; numpy's lexsort is the sort).  Ids
    outside the table are no candidates; an id that occurs several times is kept as often.  Rows with fewer than
    k candidates end with id -1 / relevance -inf.  All ids of the table as candidates is brute_force."""
    cand = np.asarray(cand)
    Q, n = cand.shape
    N = emb.shape[0]
    ids = np.full((Q, k), -1, dtype=np.int32)
    scores = np.full((Q, k), -np.inf, dtype=np.float32)
    for q in range(Q):
        c = cand[q][(cand[q] >= 0) & (cand[q] < N)].astype(np.int32)
        if c.size == 0:
            continue
        s = score_pairs(emb, users, mlp, np.full(c.size, q, dtype=np.int32), c, act_round=act_round,
                        n_threads=n_threads)
        order = np.lexsort((c, -s.astype(np.float64)))[:k]
        ids[q, :order.size] = c[order]
        scores[q, :order.size] = s[order]
    return {"ids": ids, "scores": scores}


def recall_at(found_ids: np.ndarray, truth_ids: np.ndarray, k: int) -> float:
    """Rec@k of Sec. 5.1.3: share of the true top-k found among the first k returned."""
    hits = 0
    for f, t in zip(found_ids[:, :k], truth_ids[:, :k]):
        hits += len(set(int(v) for v in f if v >= 0) & set(int(v) for v in t))
    return hits / float(truth_ids.shape[0] * k)


def philox4x32_10(ctr, key):
    """One Philox4x32-10 block: ctr = 4 words, key = 2 words -> 4 output words."""
    c = (ctypes.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    out = (ctypes.c_uint32 * 4)()
    _load().oracle_philox4x32_10(c, k, out)
    return [int(x) for x in out]


def noise_element(seed: int, stream: int, e: int) -> float:
    """The standard normal variate that element e of a [Q][d] user array receives (Eq. 5)."""
    return float(_load().oracle_noise_element(ctypes.c_uint64(seed), ctypes.c_uint64(stream), ctypes.c_uint64(e)))


def users_add_noise(users: np.ndarray, sigma: float, seed: int, stream: int = 0) -> np.ndarray:
    """users + sigma * h~ with h~ ~ N(0, I) (Eq. 5: the serendipity vector added to the user half of the
    metric input), drawn by the counter-based generator described in gmp_oracle.c; same dtype as `users`
    (fp32, bf16 bit patterns as uint16, or fp16: the fp64 sum rounded to fp32 and then to binary16)."""
    if users.dtype == np.float16:
        wide = users_add_noise(users.astype(np.float32), sigma, seed, stream)
        with np.errstate(over="ignore"):
            return f16_round(wide).astype(np.float16)
    users, dt = _table(users)
    out = np.empty_like(users)
    rc = _load().oracle_users_add_noise(_ptr(users), dt, ctypes.c_int64(users.shape[0]), int(users.shape[1]),
                                        ctypes.c_double(sigma), ctypes.c_uint64(seed), ctypes.c_uint64(stream),
                                        _ptr(out))
    if rc != 0:
        raise ValueError(f"oracle_users_add_noise failed rc={rc}")
    return out


def f16_round(a: np.ndarray) -> np.ndarray:
    """fp32 -> binary16 (nearest even) -> fp32: the rounding act_round = 3 applies to hidden activations."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.float32)
    _load().oracle_f16_round(_ptr(a), ctypes.c_int64(a.size), _ptr(out))
    return out


def e4m3_encode(a: np.ndarray, scale: float = 1.0) -> np.ndarray:
    """The e4m3 codes (uint8) of scale * a, nearest even, magnitudes above 448 clamped (and counted:
    raises if any was)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.uint8)
    n = _load().oracle_e4m3_encode(_ptr(a), ctypes.c_int64(a.size), ctypes.c_double(scale), _ptr(out))
    if n:
        raise ValueError(f"{n} values exceed the e4m3 range at scale {scale}")
    return out


def e4m3_quantize(a: np.ndarray, scale: float = 1.0) -> np.ndarray:
    """e4m3(scale * a) / scale as fp32: the values an 8-bit table or weight matrix really holds."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.float32)
    n = _load().oracle_e4m3_quantize(_ptr(a), ctypes.c_int64(a.size), ctypes.c_double(scale), _ptr(out))
    if n:
        raise ValueError(f"{n} values exceed the e4m3 range at scale {scale}")
    return out
