#!/usr/bin/env python3
"""Recall@100 of the CPU oracle's search as the list grows (test infrastructure, CPU only).

Answers, with the oracle alone, whether the search of Sec. 3.2 / Algorithm 1 reaches recall@100 >= 0.95
(Sec. 5.1.3) on the synthetic stand-in for the paper's data at any list length: the 10 M-item workload is
generated on the CPU with the same recipe the GPU runs use (other random streams, so other numbers of the
same distribution), the exhaustive ranking of a few queries comes from the plain-torch reference that the
tests pin to oracle.brute_force, and oracle.search runs at L = 128 ... 16384.

    python oracle/recall_curve.py [n_queries=32] [out.json]

Needs about 12 GB of memory and, on 8 cores, 25 minutes (the exhaustive ranking is half of it).
"""
from __future__ import annotations

import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    import torch

    import oracle
    from bench import torch_ground_truth
    from workloads import PRESETS, make_workload, to_host

    n_q = int(sys.argv[1]) if len(sys.argv) > 1 else 32
    out_path = sys.argv[2] if len(sys.argv) > 2 else ""
    threads = os.cpu_count() or 1
    torch.set_num_threads(threads)
    cfg = PRESETS["C3"]
    t = time.time()
    wl = make_workload(cfg, device="cpu")
    print(f"workload {cfg.name} on the CPU in {time.time() - t:.0f} s", flush=True)
    t = time.time()
    truth = torch_ground_truth(wl, list(range(n_q)), 100, chunk=1 << 18).numpy()
    print(f"exhaustive ranking of {n_q} queries in {time.time() - t:.0f} s", flush=True)
    h = to_host(wl)
    mlp = oracle.Mlp(h["W"], h["b"], h["head_w"])
    users, entries = h["users"][:n_q], h["entries"][:n_q]
    rows = []
    for W, L in [(8, 128), (8, 1024), (8, 2048), (8, 4096), (32, 4096), (32, 8192), (32, 16384)]:
        t = time.time()
        r = oracle.search(h["emb"], h["adj"], users, mlp, entries, W, L, cfg.k, 0, n_threads=threads, trace=True)
        rows.append({"W": W, "L": L, "recall_at_100": round(oracle.recall_at(r["ids"], truth, 100), 4),
                     "pairs_per_query": float(r["n_scored"].mean()), "rounds_avg": float(r["n_iters"].mean()),
                     "rounds_max": int(r["n_iters"].max()), "oracle_s": round(time.time() - t, 1)})
        print(rows[-1], flush=True)
    if out_path:
        with open(out_path, "w") as f:
            json.dump({"workload": cfg.name, "queries": n_q, "rows": rows}, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
