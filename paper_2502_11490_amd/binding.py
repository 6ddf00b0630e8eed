"""ctypes marshalling for include/gmpgr_ann.h.  PyTorch is used for device memory and the
current HIP stream only."""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

ANN_OK, ANN_EINVAL, ANN_ENOMEM, ANN_EDEVICE, ANN_ENOTIMPL, ANN_EWORKSPACE = 0, -1, -2, -3, -4, -5
ANN_F32, ANN_BF16, ANN_F8, ANN_F16 = 0, 1, 2, 3
ANN_VALIDATE, ANN_MLP_GENERIC = 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
# GMPGR_ANN_LIB names another build of the same library (measurement builds with other tuning constants)
_LIB_PATH = os.environ.get("GMPGR_ANN_LIB") or os.path.join(_HERE, "libgmpgr_ann.so")
_lib = None

EXPORTS = [
    "ann_graph_load", "ann_graph_free", "ann_mlp_load", "ann_mlp_free", "ann_mlp_uses_mfma",
    "ann_search_workspace_bytes", "ann_search", "ann_search_ragged", "ann_search_layers_workspace_bytes",
    "ann_search_layers", "ann_search_walkers_workspace_bytes", "ann_search_walkers",
    "ann_search_stream_workspace_bytes", "ann_search_stream", "ann_stream_open", "ann_stream_submit", "ann_stream_step",
    "ann_stream_drain", "ann_stream_close", "ann_score_pairs", "ann_score_pairs_noalloc", "ann_graph_set_locality", "ann_search_visited_set_is_bitmap", "ann_brute_force", "ann_brute_force_workspace_bytes", "ann_rerank", "ann_rerank_workspace_bytes", "ann_users_add_noise", "ann_quantize_e4m3",
    "ann_search_stats", "ann_set_progress_timeout", "ann_profile_enable", "ann_profile_read", "ann_profile_copy", "ann_last_error",
]


class AnnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ann error {code}: {msg}")
        self.code = code


class Stats(ctypes.Structure):
    _fields_ = [("pairs_scored", ctypes.c_int64), ("nodes_expanded", ctypes.c_int64),
                ("max_query_iters", ctypes.c_int64), ("visited_overflow", ctypes.c_int64),
                ("queries", ctypes.c_int64), ("adjacency_bytes", ctypes.c_int64),
                ("embedding_bytes", ctypes.c_int64), ("pair_list_bytes", ctypes.c_int64)]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libgmpgr_ann.so (built by paper_2502_11490_amd/build.py).  Raises if it is missing:
    there is no other implementation to fall back to."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} not found: build it with `python -m paper_2502_11490_amd.build` "
            "(or __graft_entry__.build()); the library has no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, u32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_size_t
    lib.ann_graph_load.argtypes = [vp, vp, i64, i32, i32, i32, u32, vp, ctypes.POINTER(vp)]
    lib.ann_graph_load.restype = ctypes.c_int
    lib.ann_graph_free.argtypes = [vp]
    lib.ann_graph_free.restype = None
    lib.ann_mlp_load.argtypes = [i32, ctypes.POINTER(i32), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                 ctypes.POINTER(ctypes.c_float), i32, i32, u32, vp, ctypes.POINTER(vp)]
    lib.ann_mlp_load.restype = ctypes.c_int
    lib.ann_mlp_free.argtypes = [vp]
    lib.ann_mlp_free.restype = None
    lib.ann_mlp_uses_mfma.argtypes = [vp]
    lib.ann_mlp_uses_mfma.restype = ctypes.c_int
    lib.ann_search_workspace_bytes.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32]
    lib.ann_search_workspace_bytes.restype = sz
    lib.ann_search.argtypes = [vp, vp, vp, i32, vp, i32, i32, i32, i32, i32, vp, sz, vp, vp, vp]
    lib.ann_search.restype = ctypes.c_int
    lib.ann_search_ragged.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp, vp, i32, i32, i32, i32, vp, sz, vp, vp, vp]
    lib.ann_search_ragged.restype = ctypes.c_int
    pi32 = ctypes.POINTER(i32)
    lib.ann_search_layers_workspace_bytes.argtypes = [ctypes.POINTER(vp), i32, vp, i32, i32, pi32, pi32, pi32, i32]
    lib.ann_search_layers_workspace_bytes.restype = sz
    lib.ann_search_layers.argtypes = [ctypes.POINTER(vp), i32, vp, vp, i32, vp, i32, pi32, pi32, pi32, i32, vp, sz,
                                      vp, vp, vp]
    lib.ann_search_layers.restype = ctypes.c_int
    lib.ann_search_walkers_workspace_bytes.argtypes = [vp, vp, i32, i32, i32, i32]
    lib.ann_search_walkers_workspace_bytes.restype = sz
    lib.ann_search_walkers.argtypes = [vp, vp, vp, i32, vp, i32, i32, i32, vp, sz, vp, vp, vp]
    lib.ann_search_walkers.restype = ctypes.c_int
    lib.ann_search_stream_workspace_bytes.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32]
    lib.ann_search_stream_workspace_bytes.restype = sz
    lib.ann_search_stream.argtypes = [vp, vp, vp, i32, vp, i32, i32, i32, i32, i32, i32, vp, sz, vp, vp, vp]
    lib.ann_search_stream.restype = ctypes.c_int
    lib.ann_stream_open.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp, ctypes.POINTER(vp)]
    lib.ann_stream_open.restype = ctypes.c_int
    lib.ann_stream_submit.argtypes = [vp, i32]
    lib.ann_stream_step.argtypes = [vp, i32]
    lib.ann_stream_drain.argtypes = [vp]
    lib.ann_stream_close.argtypes = [vp]
    for name in ("ann_stream_submit", "ann_stream_step", "ann_stream_drain", "ann_stream_close"):
        getattr(lib, name).restype = ctypes.c_int
    lib.ann_score_pairs.argtypes = [vp, vp, vp, i32, i64, vp, vp, vp, i32, vp]
    lib.ann_score_pairs.restype = ctypes.c_int
    lib.ann_score_pairs_noalloc.argtypes = [vp, vp, vp, i32, i64, vp, vp, vp, vp]
    lib.ann_score_pairs_noalloc.restype = ctypes.c_int
    lib.ann_search_visited_set_is_bitmap.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32]
    lib.ann_search_visited_set_is_bitmap.restype = ctypes.c_int
    lib.ann_graph_set_locality.argtypes = [vp, vp, vp]
    lib.ann_graph_set_locality.restype = ctypes.c_int
    lib.ann_brute_force.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, ctypes.c_size_t, vp]
    lib.ann_brute_force.restype = ctypes.c_int
    lib.ann_brute_force_workspace_bytes.argtypes = [vp, vp, i32, i32]
    lib.ann_brute_force_workspace_bytes.restype = ctypes.c_size_t
    lib.ann_rerank_workspace_bytes.argtypes = [vp, vp, i32, i32, i32]
    lib.ann_rerank_workspace_bytes.restype = ctypes.c_size_t
    lib.ann_rerank.argtypes = [vp, vp, vp, i32, vp, i32, i32, vp, vp, vp, ctypes.c_size_t, vp]
    lib.ann_rerank.restype = ctypes.c_int
    lib.ann_users_add_noise.argtypes = [vp, vp, i32, i32, i32, ctypes.c_double, ctypes.c_uint64, ctypes.c_uint64, vp]
    lib.ann_users_add_noise.restype = ctypes.c_int
    lib.ann_quantize_e4m3.argtypes = [vp, i32, i64, ctypes.c_float, vp, vp]
    lib.ann_quantize_e4m3.restype = ctypes.c_int
    lib.ann_search_stats.argtypes = [vp, ctypes.POINTER(Stats), vp]
    lib.ann_search_stats.restype = ctypes.c_int
    lib.ann_set_progress_timeout.argtypes = [ctypes.c_double]
    lib.ann_set_progress_timeout.restype = ctypes.c_int
    lib.ann_profile_enable.argtypes = [ctypes.c_int]
    lib.ann_profile_enable.restype = ctypes.c_int
    lib.ann_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.ann_profile_read.restype = ctypes.c_int
    lib.ann_profile_copy.argtypes = [vp, vp, sz, vp]
    lib.ann_profile_copy.restype = ctypes.c_int
    lib.ann_last_error.argtypes = []
    lib.ann_last_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def ann_last_error() -> str:
    return load_library().ann_last_error().decode()


def _check(rc: int):
    if rc != ANN_OK:
        raise AnnError(rc, ann_last_error())


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return ANN_F32
    if t.dtype == torch.bfloat16:
        return ANN_BF16
    if t.dtype == torch.float8_e4m3fn:
        return ANN_F8
    if t.dtype == torch.float16:
        return ANN_F16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev_ptr(t: Optional[torch.Tensor], name: str, dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _queries_ptr(queries: torch.Tensor, m, Q: Optional[int] = None) -> Optional[int]:
    """User vectors must be [Q][d_user] in the metric's element type (bf16 for the 8-bit metric, whose user half
    stays 16-bit): the library takes a bare pointer and could not tell.  With Q given, the row count is checked
    too (the kernels read Q rows)."""
    want = {ANN_F32: torch.float32, ANN_BF16: torch.bfloat16, ANN_F16: torch.float16, ANN_F8: torch.bfloat16}[m.dtype]
    if queries.dim() != 2 or queries.shape[1] != m.d_user:
        raise ValueError(f"queries must be [Q][{m.d_user}], got {tuple(queries.shape)}")
    if Q is not None and queries.shape[0] != Q:
        raise ValueError(f"queries has {queries.shape[0]} rows, entries has {Q}")
    return _dev_ptr(queries, "queries", want)


def _entries_shape(entries: torch.Tensor):
    if entries.dim() != 2:
        raise ValueError(f"entries must be [Q][E], got {tuple(entries.shape)}")
    return int(entries.shape[0]), int(entries.shape[1])


def _check_out(out_ids, out_scores, Q: int, k: int) -> None:
    """Caller-supplied result arrays must be exactly [Q][k]: the library writes Q * k elements into each."""
    for name, t in (("out_ids", out_ids), ("out_scores", out_scores)):
        if t is None or tuple(t.shape) != (Q, k):
            raise ValueError(f"{name} must be [{Q}][{k}], got {None if t is None else tuple(t.shape)}")


def _per_query_ptr(t: torch.Tensor, name: str, Q: int) -> Optional[int]:
    if t is None or t.numel() != Q:
        raise ValueError(f"{name} must hold one int32 per query ({Q}), got {None if t is None else t.numel()}")
    return _dev_ptr(t, name, torch.int32)


class Graph:
    """Owns the C handle and keeps the borrowed tensors alive."""

    def __init__(self, handle, adj, emb):
        self.handle, self.adj, self.emb = handle, adj, emb

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ann_graph_free(self.handle)
            self.handle = None


class Mlp:
    def __init__(self, handle, dims, d_user, dtype):
        self.handle, self.dims, self.d_user, self.dtype = handle, list(dims), d_user, dtype

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ann_mlp_free(self.handle)
            self.handle = None


def ann_graph_load(adj: torch.Tensor, emb: torch.Tensor, flags: int = 0, stream=None) -> Graph:
    lib = load_library()
    if adj.dim() != 2 or emb.dim() != 2 or adj.shape[0] != emb.shape[0]:
        raise ValueError("adj must be [N,R] and emb [N,d]")
    h = ctypes.c_void_p()
    rc = lib.ann_graph_load(_dev_ptr(adj, "adj", torch.int32), _dev_ptr(emb, "emb"), adj.shape[0], adj.shape[1],
                            emb.shape[1], _dtype_code(emb), flags, _stream_ptr(stream), ctypes.byref(h))
    _check(rc)
    return Graph(h, adj, emb)


def ann_graph_set_locality(g: Graph, rank: Optional[torch.Tensor], stream=None) -> None:
    """Addresses the visited bitmap of searches on `g` by rank [N] (int32 permutation of the ids, device; None
    removes it).  Results do not change; the tensor is kept alive with the graph."""
    if rank is not None and (rank.dim() != 1 or rank.shape[0] != g.adj.shape[0]):
        raise ValueError(f"rank must be [{g.adj.shape[0]}], got {tuple(rank.shape)}")
    _check(load_library().ann_graph_set_locality(g.handle, _dev_ptr(rank, "rank", torch.int32), _stream_ptr(stream)))
    g.rank = rank


def ann_search_visited_set_is_bitmap(g: Graph, m: Mlp, Q: int, E: int, W: int, L: int, k: int, max_iters: int = 0) -> bool:
    rc = load_library().ann_search_visited_set_is_bitmap(g.handle, m.handle, Q, E, W, L, k, max_iters)
    if rc < 0:
        _check(rc)
    return rc == 1


def _host_bytes(t) -> np.ndarray:
    """Host copy of a weight tensor as a contiguous numpy array (bf16 as raw uint16)."""
    if isinstance(t, torch.Tensor):
        t = t.detach().to("cpu").contiguous()
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).numpy().view(np.uint16).copy()
        return t.numpy().copy()
    return np.ascontiguousarray(t)


def ann_mlp_load(W: Sequence, b: Sequence, head_w, d_user: int, dtype: int, flags: int = 0, stream=None) -> Mlp:
    """W[l]: [out,in] torch tensors (fp32, bf16 or fp16, matching dtype) or numpy arrays (bf16 as uint16 bits);
    b[l]: [out] fp32; head_w: [J] fp32."""
    lib = load_library()
    n = len(W)
    Wh = [_host_bytes(w) for w in W]
    # the 8-bit metric takes bf16 weights and quantises them
    want = {ANN_F32: np.float32, ANN_F16: np.float16}.get(dtype, np.uint16)
    for w in Wh:
        if w.dtype != want:
            raise TypeError(f"weights must be {np.dtype(want).name if want != np.uint16 else 'bf16'}")
    bh = [np.ascontiguousarray(_host_bytes(x), dtype=np.float32) for x in b]
    hw = np.ascontiguousarray(_host_bytes(head_w), dtype=np.float32)
    dims = [Wh[0].shape[1]] + [w.shape[0] for w in Wh]
    for l in range(n):
        if Wh[l].shape != (dims[l + 1], dims[l]) or bh[l].shape != (dims[l + 1],):
            raise ValueError("layer shapes do not chain")
    if hw.shape != (dims[-1],):
        raise ValueError("head_w must have one weight per head")
    dims_c = (ctypes.c_int32 * (n + 1))(*dims)
    W_c = (ctypes.c_void_p * n)(*[w.ctypes.data for w in Wh])
    b_c = (ctypes.c_void_p * n)(*[x.ctypes.data for x in bh])
    h = ctypes.c_void_p()
    rc = lib.ann_mlp_load(n, dims_c, W_c, b_c, hw.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), d_user, dtype,
                          flags, _stream_ptr(stream), ctypes.byref(h))
    _check(rc)
    return Mlp(h, dims, d_user, dtype)


def ann_mlp_uses_mfma(m: Mlp) -> bool:
    return bool(load_library().ann_mlp_uses_mfma(m.handle))


def ann_search_workspace_bytes(g: Graph, m: Mlp, Q: int, E: int, W_max: int, L_max: int, k: int,
                               max_iters_max: int) -> int:
    n = load_library().ann_search_workspace_bytes(g.handle, m.handle, Q, E, W_max, L_max, k, max_iters_max)
    if n == 0:
        raise AnnError(ANN_EINVAL, ann_last_error())
    return int(n)


def _alloc_out(Q, k, device):
    return (torch.empty((Q, k), dtype=torch.int32, device=device),
            torch.empty((Q, k), dtype=torch.float32, device=device))


def ann_search(g: Graph, m: Mlp, queries: torch.Tensor, entries: torch.Tensor, W: int, L: int, k: int,
               max_iters: int = 0, workspace: Optional[torch.Tensor] = None, out_ids=None, out_scores=None,
               stream=None):
    """Returns (ids [Q,k] int32, scores [Q,k] fp32) on the device.  `workspace` is a uint8 device tensor of at
    least ann_search_workspace_bytes(...) bytes; one is allocated when omitted."""
    lib = load_library()
    Q, E = _entries_shape(entries)
    if workspace is None:
        workspace = torch.empty(ann_search_workspace_bytes(g, m, Q, E, W, L, k, max_iters), dtype=torch.uint8,
                                device=queries.device)
    if out_ids is None:
        out_ids, out_scores = _alloc_out(Q, k, queries.device)
    _check_out(out_ids, out_scores, Q, k)
    rc = lib.ann_search(g.handle, m.handle, _queries_ptr(queries, m, Q), Q, _dev_ptr(entries, "entries", torch.int32),
                        E, W, L, k, max_iters, _dev_ptr(workspace, "workspace", torch.uint8), workspace.numel(),
                        _dev_ptr(out_ids, "out_ids", torch.int32), _dev_ptr(out_scores, "out_scores", torch.float32),
                        _stream_ptr(stream))
    _check(rc)
    return out_ids, out_scores


def ann_search_ragged(g: Graph, m: Mlp, queries, entries, W_q, L_q, iters_q, W_max: int, L_max: int, k: int,
                      max_iters_max: int, workspace: Optional[torch.Tensor] = None, out_ids=None, out_scores=None,
                      stream=None):
    lib = load_library()
    Q, E = _entries_shape(entries)
    if workspace is None:
        workspace = torch.empty(ann_search_workspace_bytes(g, m, Q, E, W_max, L_max, k, max_iters_max),
                                dtype=torch.uint8, device=queries.device)
    if out_ids is None:
        out_ids, out_scores = _alloc_out(Q, k, queries.device)
    _check_out(out_ids, out_scores, Q, k)
    for name, t in (("W_q", W_q), ("L_q", L_q), ("iters_q", iters_q)):  # sizes first: they need no device
        if t is None or t.numel() != Q:
            raise ValueError(f"{name} must hold one int32 per query ({Q}), got {None if t is None else t.numel()}")
    rc = lib.ann_search_ragged(g.handle, m.handle, _queries_ptr(queries, m, Q), Q,
                               _dev_ptr(entries, "entries", torch.int32), E, _per_query_ptr(W_q, "W_q", Q),
                               _per_query_ptr(L_q, "L_q", Q), _per_query_ptr(iters_q, "iters_q", Q), W_max,
                               L_max, k, max_iters_max, _dev_ptr(workspace, "workspace", torch.uint8),
                               workspace.numel(), _dev_ptr(out_ids, "out_ids", torch.int32),
                               _dev_ptr(out_scores, "out_scores", torch.float32), _stream_ptr(stream))
    _check(rc)
    return out_ids, out_scores


def ann_search_walkers_workspace_bytes(g: Graph, m: Mlp, Q: int, E: int, T: int, k: int) -> int:
    nbytes = load_library().ann_search_walkers_workspace_bytes(g.handle, m.handle, Q, E, T, k)
    if nbytes == 0:
        raise AnnError(-1, ann_last_error())
    return nbytes


def ann_search_walkers(g: Graph, m: Mlp, queries: torch.Tensor, entries: torch.Tensor, T: int, k: int,
                       workspace: Optional[torch.Tensor] = None, out_ids=None, out_scores=None, stream=None):
    """One walker per seed, T greedy hops each, one shared result list.  Returns (ids [Q,k], scores [Q,k])."""
    lib = load_library()
    Q, E = _entries_shape(entries)
    if workspace is None:
        workspace = torch.empty(ann_search_walkers_workspace_bytes(g, m, Q, E, T, k), dtype=torch.uint8,
                                device=queries.device)
    if out_ids is None:
        out_ids, out_scores = _alloc_out(Q, k, queries.device)
    _check_out(out_ids, out_scores, Q, k)
    rc = lib.ann_search_walkers(g.handle, m.handle, _queries_ptr(queries, m, Q), Q,
                                _dev_ptr(entries, "entries", torch.int32), E, T, k,
                                _dev_ptr(workspace, "workspace", torch.uint8), workspace.numel(),
                                _dev_ptr(out_ids, "out_ids", torch.int32),
                                _dev_ptr(out_scores, "out_scores", torch.float32), _stream_ptr(stream))
    _check(rc)
    return out_ids, out_scores


def ann_search_stream_workspace_bytes(g: Graph, m: Mlp, Q_total: int, slots: int, E: int, W: int, L: int, k: int,
                                      max_iters: int = 0) -> int:
    nbytes = load_library().ann_search_stream_workspace_bytes(g.handle, m.handle, Q_total, slots, E, W, L, k, max_iters)
    if nbytes == 0:
        raise AnnError(-1, ann_last_error())
    return nbytes


def ann_search_stream(g: Graph, m: Mlp, queries: torch.Tensor, entries: torch.Tensor, slots: int, W: int, L: int,
                      k: int, max_iters: int = 0, workspace: Optional[torch.Tensor] = None, out_ids=None,
                      out_scores=None, stream=None):
    """All queries, `slots` of them in flight at a time; a finished query's slot goes to the next one.
    Returns (ids [Q_total,k], scores [Q_total,k])."""
    lib = load_library()
    Q, E = _entries_shape(entries)
    if workspace is None:
        workspace = torch.empty(ann_search_stream_workspace_bytes(g, m, Q, slots, E, W, L, k, max_iters),
                                dtype=torch.uint8, device=queries.device)
    if out_ids is None:
        out_ids, out_scores = _alloc_out(Q, k, queries.device)
    _check_out(out_ids, out_scores, Q, k)
    rc = lib.ann_search_stream(g.handle, m.handle, _queries_ptr(queries, m, Q), Q,
                               _dev_ptr(entries, "entries", torch.int32), E, slots, W, L, k, max_iters,
                               _dev_ptr(workspace, "workspace", torch.uint8), workspace.numel(),
                               _dev_ptr(out_ids, "out_ids", torch.int32),
                               _dev_ptr(out_scores, "out_scores", torch.float32), _stream_ptr(stream))
    _check(rc)
    return out_ids, out_scores


class Stream:
    """An open stream (ann_stream_open): queries are written into rows of `queries` / `entries` and submitted
    while earlier ones are being searched; results land in the same rows of `out_ids` / `out_scores`.  The
    object keeps the caller's arrays and the workspace alive."""

    def __init__(self, g: Graph, m: Mlp, queries: torch.Tensor, entries: torch.Tensor, slots: int, W: int, L: int,
                 k: int, max_iters: int = 0, workspace: Optional[torch.Tensor] = None, out_ids=None, out_scores=None,
                 stream=None):
        lib = load_library()
        cap, E = _entries_shape(entries)
        if workspace is None:
            workspace = torch.empty(ann_search_stream_workspace_bytes(g, m, cap, slots, E, W, L, k, max_iters),
                                    dtype=torch.uint8, device=queries.device)
        if out_ids is None:
            out_ids, out_scores = _alloc_out(cap, k, queries.device)
        _check_out(out_ids, out_scores, cap, k)
        self.g, self.m, self.queries, self.entries, self.workspace = g, m, queries, entries, workspace
        self.out_ids, self.out_scores, self.capacity = out_ids, out_scores, cap
        self.handle = ctypes.c_void_p()
        _check(lib.ann_stream_open(g.handle, m.handle, cap, slots, E, W, L, k, max_iters, _queries_ptr(queries, m, cap),
                                   _dev_ptr(entries, "entries", torch.int32), _dev_ptr(out_ids, "out_ids", torch.int32),
                                   _dev_ptr(out_scores, "out_scores", torch.float32),
                                   _dev_ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream_ptr(stream),
                                   ctypes.byref(self.handle)))

    def submit(self, n: int) -> None:
        _check(load_library().ann_stream_submit(self.handle, n))

    def step(self, rounds: int) -> None:
        _check(load_library().ann_stream_step(self.handle, rounds))

    def drain(self) -> None:
        _check(load_library().ann_stream_drain(self.handle))

    def close(self) -> None:
        if getattr(self, "handle", None):
            _check(load_library().ann_stream_close(self.handle))
            self.handle = None

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ann_stream_close(self.handle)
            self.handle = None


def ann_stream_open(g: Graph, m: Mlp, queries, entries, slots: int, W: int, L: int, k: int, max_iters: int = 0,
                    **kw) -> Stream:
    return Stream(g, m, queries, entries, slots, W, L, k, max_iters, **kw)


def _layer_args(graphs: Sequence[Graph], W_l, L_l, K_l):
    n = len(graphs)
    if not (len(W_l) == len(L_l) == len(K_l) == n):
        raise ValueError("W_l, L_l, K_l need one entry per layer")
    handles = (ctypes.c_void_p * n)(*[g.handle for g in graphs])
    arr = lambda v: (ctypes.c_int32 * n)(*[int(x) for x in v])
    return n, handles, arr(W_l), arr(L_l), arr(K_l)


def ann_search_layers_workspace_bytes(graphs: Sequence[Graph], m: Mlp, Q: int, E: int, W_l, L_l, K_l,
                                      max_iters: int = 0) -> int:
    n, handles, W, L, K = _layer_args(graphs, W_l, L_l, K_l)
    nbytes = load_library().ann_search_layers_workspace_bytes(handles, n, m.handle, Q, E, W, L, K, max_iters)
    if nbytes == 0:
        raise AnnError(-1, ann_last_error())
    return nbytes


def ann_search_layers(graphs: Sequence[Graph], m: Mlp, queries: torch.Tensor, entries: torch.Tensor, W_l, L_l, K_l,
                      max_iters: int = 0, workspace: Optional[torch.Tensor] = None, out_ids=None, out_scores=None,
                      stream=None):
    """Layer-by-layer search, coarsest graph first; K_l[-1] results per query.  Returns (ids, scores)."""
    lib = load_library()
    Q, E = _entries_shape(entries)
    n, handles, W, L, K = _layer_args(graphs, W_l, L_l, K_l)
    if workspace is None:
        workspace = torch.empty(ann_search_layers_workspace_bytes(graphs, m, Q, E, W_l, L_l, K_l, max_iters),
                                dtype=torch.uint8, device=queries.device)
    if out_ids is None:
        out_ids, out_scores = _alloc_out(Q, int(K_l[-1]), queries.device)
    _check_out(out_ids, out_scores, Q, int(K_l[-1]))
    rc = lib.ann_search_layers(handles, n, m.handle, _queries_ptr(queries, m, Q), Q,
                               _dev_ptr(entries, "entries", torch.int32), E, W, L, K, max_iters,
                               _dev_ptr(workspace, "workspace", torch.uint8), workspace.numel(),
                               _dev_ptr(out_ids, "out_ids", torch.int32),
                               _dev_ptr(out_scores, "out_scores", torch.float32), _stream_ptr(stream))
    _check(rc)
    return out_ids, out_scores


def ann_score_pairs(g: Graph, m: Mlp, queries: torch.Tensor, q_idx: torch.Tensor, item: torch.Tensor,
                    out: Optional[torch.Tensor] = None, tile_rows: int = 0, stream=None) -> torch.Tensor:
    lib = load_library()
    M = q_idx.numel()
    if item.numel() != M:
        raise ValueError(f"q_idx names {M} pairs, item {item.numel()}")
    if out is None:
        out = torch.empty(M, dtype=torch.float32, device=queries.device)
    if out.numel() != M:
        raise ValueError(f"out must hold {M} scores, got {out.numel()}")
    rc = lib.ann_score_pairs(g.handle, m.handle, _queries_ptr(queries, m), queries.shape[0], M,
                             _dev_ptr(q_idx, "q_idx", torch.int32), _dev_ptr(item, "item", torch.int32),
                             _dev_ptr(out, "out", torch.float32), tile_rows, _stream_ptr(stream))
    _check(rc)
    return out


def ann_score_pairs_noalloc(g: Graph, m: Mlp, queries: torch.Tensor, q_idx: torch.Tensor, item: torch.Tensor,
                            out: torch.Tensor, stream=None) -> torch.Tensor:
    """ann_score_pairs without any allocation: `out` ([M] fp32) is the caller's, the library's scratch is a
    fixed array on the device.  Only enqueues; synchronise the stream before reading `out`."""
    lib = load_library()
    M = q_idx.numel()
    if item.numel() != M or out.numel() != M:
        raise ValueError(f"q_idx names {M} pairs, item {item.numel()}, out {out.numel()}")
    rc = lib.ann_score_pairs_noalloc(g.handle, m.handle, _queries_ptr(queries, m), queries.shape[0], M,
                                     _dev_ptr(q_idx, "q_idx", torch.int32), _dev_ptr(item, "item", torch.int32),
                                     _dev_ptr(out, "out", torch.float32), _stream_ptr(stream))
    _check(rc)
    return out


def _workspace_args(workspace: Optional[torch.Tensor]):
    if workspace is None:
        return None, 0
    return _dev_ptr(workspace, "workspace", torch.uint8), workspace.numel()


def ann_brute_force_workspace_bytes(g: Graph, m: Mlp, Q: int, k: int) -> int:
    n = load_library().ann_brute_force_workspace_bytes(g.handle, m.handle, Q, k)
    if n == 0:
        raise AnnError(ANN_EINVAL, ann_last_error())
    return int(n)


def ann_rerank_workspace_bytes(g: Graph, m: Mlp, Q: int, n: int, k: int) -> int:
    b = load_library().ann_rerank_workspace_bytes(g.handle, m.handle, Q, n, k)
    if b == 0:
        raise AnnError(ANN_EINVAL, ann_last_error())
    return int(b)


def ann_brute_force(g: Graph, m: Mlp, queries: torch.Tensor, k: int, out_ids: Optional[torch.Tensor] = None,
                    out_scores: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """Exhaustive search: the k most relevant items of the whole table per query (ids [Q][k] int32, relevances
    [Q][k] fp32; relevance descending, ties by ascending id).  With a `workspace` (uint8 device tensor of
    ann_brute_force_workspace_bytes) the call only enqueues; without one it allocates and synchronises."""
    lib = load_library()
    Q = queries.shape[0]
    if out_ids is None:
        out_ids = torch.empty(Q, k, dtype=torch.int32, device=queries.device)
    if out_scores is None:
        out_scores = torch.empty(Q, k, dtype=torch.float32, device=queries.device)
    _check_out(out_ids, out_scores, Q, k)
    ws, ws_bytes = _workspace_args(workspace)
    rc = lib.ann_brute_force(g.handle, m.handle, _queries_ptr(queries, m), Q, k,
                             _dev_ptr(out_ids, "out_ids", torch.int32),
                             _dev_ptr(out_scores, "out_scores", torch.float32), ws, ws_bytes, _stream_ptr(stream))
    _check(rc)
    return out_ids, out_scores


def ann_rerank(g: Graph, m: Mlp, queries: torch.Tensor, cand: torch.Tensor, k: int,
               out_ids: Optional[torch.Tensor] = None, out_scores: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None, stream=None):
    """The k most relevant of each query's candidates cand [Q][n] (int32; ids outside the table are skipped)
    under this metric: ids [Q][k] int32, relevances [Q][k] fp32.  `workspace` as for ann_brute_force
    (ann_rerank_workspace_bytes)."""
    lib = load_library()
    Q = queries.shape[0]
    if cand.dim() != 2 or cand.shape[0] != Q:
        raise ValueError(f"cand must be [{Q}][n], got {tuple(cand.shape)}")
    if out_ids is None:
        out_ids = torch.empty(Q, k, dtype=torch.int32, device=queries.device)
    if out_scores is None:
        out_scores = torch.empty(Q, k, dtype=torch.float32, device=queries.device)
    _check_out(out_ids, out_scores, Q, k)
    ws, ws_bytes = _workspace_args(workspace)
    rc = lib.ann_rerank(g.handle, m.handle, _queries_ptr(queries, m), Q, _dev_ptr(cand, "cand", torch.int32),
                        cand.shape[1], k, _dev_ptr(out_ids, "out_ids", torch.int32),
                        _dev_ptr(out_scores, "out_scores", torch.float32), ws, ws_bytes, _stream_ptr(stream))
    _check(rc)
    return out_ids, out_scores


def ann_users_add_noise(users: torch.Tensor, sigma: float, seed: int, draw: int = 0,
                        out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """users + sigma * N(0, I) (Eq. 5), same dtype and shape; `out` may be `users`."""
    if users.dim() != 2:
        raise ValueError("users must be [Q][d]")
    if out is None:
        out = torch.empty_like(users)
    if out.shape != users.shape or out.dtype != users.dtype:
        raise ValueError("out must have the shape and dtype of users")
    Q, d = users.shape
    _check(load_library().ann_users_add_noise(_dev_ptr(users, "users") if Q else None, _dev_ptr(out, "out") if Q else None,
                                              Q, d, _dtype_code(users), float(sigma), int(seed), int(draw),
                                              _stream_ptr(stream)))
    return out


def ann_quantize_e4m3(src: torch.Tensor, scale: float = 1.0, out: Optional[torch.Tensor] = None,
                      stream=None) -> torch.Tensor:
    """e4m3(scale * src) as a torch.float8_e4m3fn tensor of the same shape (src: fp32 or bf16, on the device)."""
    if out is None:
        out = torch.empty(src.shape, dtype=torch.float8_e4m3fn, device=src.device)
    if out.shape != src.shape or out.dtype != torch.float8_e4m3fn:
        raise ValueError("out must be float8_e4m3fn with the shape of src")
    code = _dtype_code(src)
    if code == ANN_F8:
        raise TypeError("src must be fp32 or bf16")
    n = src.numel()
    _check(load_library().ann_quantize_e4m3(_dev_ptr(src, "src") if n else None, code, n, float(scale),
                                            _dev_ptr(out, "out") if n else None, _stream_ptr(stream)))
    return out


def ann_search_stats(workspace: torch.Tensor, stream=None) -> Stats:
    st = Stats()
    _check(load_library().ann_search_stats(_dev_ptr(workspace, "workspace", torch.uint8), ctypes.byref(st),
                                           _stream_ptr(stream)))
    return st


def ann_set_progress_timeout(seconds: float) -> None:
    _check(load_library().ann_set_progress_timeout(float(seconds)))


STAGES = ("score", "round", "pack")


def ann_profile_enable(on: bool) -> None:
    _check(load_library().ann_profile_enable(1 if on else 0))


def ann_profile_read() -> dict:
    """{stage: (milliseconds, launches)} since the last read."""
    ms = (ctypes.c_double * len(STAGES))()
    n = (ctypes.c_int64 * len(STAGES))()
    _check(load_library().ann_profile_read(ms, n))
    return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(STAGES)}


def ann_profile_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """Reference copy of known size for hardware traffic counters (dst, src: same-size device tensors)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("dst and src must have the same size")
    _check(load_library().ann_profile_copy(_dev_ptr(dst, "dst"), _dev_ptr(src, "src"), nbytes, _stream_ptr(stream)))
