"""Pins the exhaustive ranking that the benchmark and the full-size GPU tests use as recall ground truth.

`bench.torch_ground_truth` is a plain fp32 torch evaluation of the relevance (Sec. 3.1, Eq. 5-8) over every
item, in chunks, with the user half of the first layer applied once per query.  It runs where the workload
lives (the GPU in the benchmark); here it runs on CPU tensors and is compared with the oracle's brute force
(fp64, plain loops), which is itself pinned by the tests of the oracle.  Recall@k (Sec. 5.1.3) only uses the
set of the first k ids, but the order is checked too.
"""
import os
import sys

import numpy as np
import torch

import oracle
from workloads import PRESETS, make_workload, scaled, to_host

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from bench import recall_at, torch_ground_truth  # noqa: E402


def _check(cfg, k, chunk, bias_scale=0.0):
    wl = make_workload(cfg, device="cpu", with_graph=False)
    if bias_scale:
        g = torch.Generator().manual_seed(11)
        wl["b"] = [bias_scale * torch.randn(b.shape, generator=g) for b in wl["b"]]
    q_sel = list(range(cfg.Q))
    truth = torch_ground_truth(wl, q_sel, k, chunk=chunk).numpy()
    h = to_host(wl)
    mlp = oracle.Mlp(h["W"], h["b"], h["head_w"])
    bf = oracle.brute_force(h["emb"], h["users"], mlp, k + 8, n_threads=8)
    ids, sc = bf["ids"], bf["scores"].astype(np.float64)
    n_swapped = 0
    for q in range(cfg.Q):
        want = ids[q, :k]
        got = truth[q]
        assert len(set(got.tolist())) == k and got.min() >= 0 and got.max() < cfg.N
        if np.array_equal(got, want):
            continue
        # fp32 against fp64: two items may change places only where their exact relevances are a rounding apart
        exact = oracle.score_pairs(h["emb"], h["users"], mlp, np.full(k, q, np.int32), got.astype(np.int32))
        assert np.all(np.abs(exact - sc[q, :k]) <= 2e-6), (q, np.abs(exact - sc[q, :k]).max())
        # and an id outside the exact first k must tie with the k-th relevance to that precision
        extra = set(got.tolist()) - set(want.tolist())
        assert len(extra) <= 2
        n_swapped += 1
    # recall of the exact ranking against this ground truth is 1 up to such swaps at the k-th place
    r = recall_at(torch.from_numpy(ids[:, :k].astype(np.int64)), torch.from_numpy(truth), k)
    assert r >= 1.0 - 2.0 / k
    return n_swapped


def test_ground_truth_equals_oracle_brute_force_fp32_items():
    cfg = scaled(PRESETS["C1"], 6000, Q=12)
    _check(cfg, 50, chunk=2048, bias_scale=0.3)   # several chunks and a ragged last one, non-zero biases


def test_ground_truth_equals_oracle_brute_force_bf16_items():
    # the headline shape (two hidden layers, four heads) on a small item table; chunk larger than the table
    cfg = scaled(PRESETS["C3"], 20000, n_clusters=32, Q=8)
    _check(cfg, 100, chunk=1 << 20)
    _check(cfg, 100, chunk=4096)


def test_ground_truth_is_ordered_by_relevance_then_id_on_ties():
    """All-equal relevance (zero weights): any k ids are a correct ground truth for recall; the function must
    still return k distinct valid ids."""
    cfg = scaled(PRESETS["C1"], 500, Q=3)
    wl = make_workload(cfg, device="cpu", with_graph=False)
    wl["W"] = [torch.zeros_like(w) for w in wl["W"]]
    truth = torch_ground_truth(wl, [0, 1, 2], 10, chunk=128)
    for row in truth.tolist():
        assert len(set(row)) == 10 and min(row) >= 0 and max(row) < cfg.N
