"""Helpers shared by the GPU parity tests: move a seeded workload to the device, open the
library handles, and build the oracle's view of the same arrays."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2502_11490_amd as ann
from workloads import to_host


def open_handles(wl, flags_mlp: int = 0, validate: bool = True):
    """wl: dict from workloads.make_workload (tensors on any device).  Returns (graph, mlp, dev dict)."""
    dev = {}
    for key in ("emb", "adj", "users", "entries", "W_q", "L_q", "cap_q"):
        if key in wl:
            dev[key] = wl[key].to("cuda").contiguous()
    dtype = {torch.bfloat16: ann.ANN_BF16, torch.float16: ann.ANN_F16}.get(wl["emb"].dtype, ann.ANN_F32)
    g = ann.ann_graph_load(dev["adj"], dev["emb"], ann.ANN_VALIDATE if validate else 0)
    d_user = wl["users"].shape[1]
    m = ann.ann_mlp_load(wl["W"], wl["b"], wl["head_w"], d_user, dtype, flags_mlp)
    return g, m, dev


def oracle_mlp(wl_host) -> oracle.Mlp:
    return oracle.Mlp(wl_host["W"], wl_host["b"], wl_host["head_w"])


def host_view(wl):
    return to_host(wl)


def same_list_fraction(a: np.ndarray, b: np.ndarray) -> float:
    return float(np.mean(np.all(a == b, axis=1)))
