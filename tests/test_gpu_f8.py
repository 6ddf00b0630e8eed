"""Parity of the 8-bit (e4m3) metric with the oracle, through the C ABI: the quantiser bit for bit, the
relevance against the oracle run at the kernel's precision and against the unquantised metric (the
error the 8 bits cost), and the search on top of it."""
import os
import sys
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
from workloads import PRESETS, make_workload, random_mlp, scaled, to_host

pytestmark = pytest.mark.gpu

# Budget of the 8-bit metric against the exact (unquantised, fp64) oracle: mean and largest |relevance error|
# over random pairs, and recall@k lost against the exact oracle's search at equal L.
F8_MEAN_BUDGET, F8_MAX_BUDGET, F8_RECALL_BUDGET = 1e-2, 6e-2, 0.05

ann = pytest.importorskip("paper_2502_11490_amd")
sys.path.insert(0, os.path.dirname(__file__))
from gpu_util import oracle_mlp, same_list_fraction  # noqa: E402


def _codes(t):
    return t.view(torch.uint8).cpu().numpy()


def _decode_table():
    tab = np.zeros(256, np.float32)
    for c in range(256):
        s = -1.0 if c & 0x80 else 1.0
        e, m = (c >> 3) & 15, c & 7
        tab[c] = np.nan if (e == 15 and m == 7) else s * (m / 8 * 2.0 ** -6 if e == 0 else 2.0 ** (e - 7) * (1 + m / 8))
    return tab


@pytest.mark.parametrize("scale", [1.0, 4.0, 0.125])
def test_quantiser_matches_oracle_bit_for_bit(scale):
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(50001) * s for s in (1e-3, 1e-2, 0.1, 1.0, 10.0)]).astype(np.float32)
    x = x[np.abs(x * scale) <= 448]
    got = _codes(ann.ann_quantize_e4m3(torch.from_numpy(x).cuda(), scale))
    assert np.array_equal(got, oracle.e4m3_encode(x, scale))
    xb = torch.from_numpy(x).to(torch.bfloat16)
    got = _codes(ann.ann_quantize_e4m3(xb.cuda(), scale))
    assert np.array_equal(got, oracle.e4m3_encode(xb.float().numpy(), scale))


def test_quantiser_clamps_and_handles_empty_and_bad_arguments():
    x = torch.tensor([500.0, -1000.0, 448.0, 0.0, -0.0], device="cuda")
    assert _codes(ann.ann_quantize_e4m3(x)).tolist() == [0x7E, 0xFE, 0x7E, 0x00, 0x80]
    assert ann.ann_quantize_e4m3(torch.empty(0, 4, device="cuda")).shape == (0, 4)
    for bad in (0.0, -1.0, float("inf")):
        with pytest.raises(ann.AnnError):
            ann.ann_quantize_e4m3(x, bad)


def _f8_problem(N=6000, Q=45, seed=13, bias_scale=0.2, preset="C2"):
    """A C2-shaped (64-wide items, 128 -> 256 -> 128 -> J) or C3-shaped (128-wide, 256 -> 512 -> 256 -> J) workload
    in the 8-bit metric: the device handles and the oracle's view of the same numbers (quantised tables and
    weights as ordinary fp32 values)."""
    cfg = scaled(PRESETS[preset], N, n_clusters=12, Q=Q)
    wl = make_workload(cfg)
    wl["W"], wl["b"] = random_mlp(cfg.dims, seed, cfg.dtype, bias_scale=bias_scale)
    emb8 = ann.ann_quantize_e4m3(wl["emb"].cuda())
    g = ann.ann_graph_load(wl["adj"].cuda().contiguous(), emb8, ann.ANN_VALIDATE)
    users = wl["users"].cuda().contiguous()
    m = ann.ann_mlp_load(wl["W"], wl["b"], wl["head_w"], cfg.d, ann.ANN_F8)
    assert ann.ann_mlp_uses_mfma(m)
    h = to_host(wl)
    W = [oracle.widen_bf16(w) for w in h["W"]]
    Wq = [np.concatenate([W[0][:, :cfg.d], oracle.e4m3_quantize(W[0][:, cfg.d:], 4.0)], axis=1),
          oracle.e4m3_quantize(W[1], 4.0), oracle.e4m3_quantize(W[2], 4.0)]
    view = {"emb": _decode_table()[_codes(emb8)], "users": oracle.widen_bf16(h["users"]), "adj": h["adj"],
            "entries": h["entries"], "mlp_q": oracle.Mlp(Wq, h["b"], h["head_w"]),
            "emb_exact": oracle.widen_bf16(h["emb"]), "mlp_exact": oracle.Mlp(W, h["b"], h["head_w"])}
    assert np.array_equal(_codes(emb8), oracle.e4m3_encode(view["emb_exact"]))
    return cfg, g, m, users, wl["entries"].cuda().contiguous(), view


@pytest.mark.parametrize("preset", ["C2", "C3"])
def test_relevance_f8(preset):
    cfg, g, m, users, _, v = _f8_problem(preset=preset)
    rng = np.random.default_rng(3)
    M = 2 * 1024 + 77   # several batches and a ragged tail
    q = np.sort(rng.integers(0, cfg.Q, M)).astype(np.int32)
    it = rng.integers(0, cfg.N, M).astype(np.int32)
    got = ann.ann_score_pairs(g, m, users, torch.from_numpy(q).cuda(), torch.from_numpy(it).cuda()).cpu().numpy()
    assert np.all(np.isfinite(got))
    kern = oracle.score_pairs(v["emb"], v["users"], v["mlp_q"], q, it, act_round=2, n_threads=8)
    err = np.abs(got - kern)
    # Same quantised operands on both sides; what differs is the order of the fp32 sums, which now and then
    # moves an activation across an e4m3 rounding boundary: one step of one unit of the last hidden layer is at
    # most 1/8 of its value, times a head weight row (< 0.5), the sigmoid's slope (1/4) and a head weight.
    assert np.max(err) <= 1e-2, f"max {np.max(err)}"
    assert np.median(err) <= 1e-4, f"median {np.median(err)}"
    exact = oracle.score_pairs(v["emb_exact"], v["users"], v["mlp_exact"], q, it, n_threads=8)
    cost = np.abs(got - exact)
    print(f"{preset} 8-bit metric against the unquantised one: mean |error| {cost.mean():.4f}, max {cost.max():.4f}; "
          f"against the oracle at the kernel's precision: median {np.median(err):.2e}, max {err.max():.2e}")
    # The budget of the 8-bit metric against the relevance the paper defines (the exact oracle): three mantissa
    # bits are a relative rounding error of up to 1/16 per operand; over items, two weight matrices and two
    # hidden layers that is a mean error of the relevance below 1e-2 and a largest one below 6e-2.  The 16-bit
    # bar (1e-2 for every pair) is NOT met by this format, and the tests of the 16-bit modes do not use it.
    assert cost.mean() <= F8_MEAN_BUDGET and cost.max() <= F8_MAX_BUDGET, (cost.mean(), cost.max())


def test_relevance_f8_out_of_range_pairs_are_nan():
    cfg, g, m, users, _, _ = _f8_problem(N=2000, Q=8)
    q = torch.tensor([0, 8, 1, -1, 2], dtype=torch.int32).cuda()
    it = torch.tensor([5, 5, 2000, 3, 7], dtype=torch.int32).cuda()
    got = ann.ann_score_pairs(g, m, users, q, it).cpu().numpy()
    assert np.isnan(got[1]) and np.isnan(got[2]) and np.isnan(got[3])
    assert np.isfinite(got[0]) and np.isfinite(got[4])


@pytest.mark.parametrize("preset", ["C2", "C3"])
def test_search_f8_recall_matches_oracle(preset):
    cfg, g, m, users, entries, v = _f8_problem(N=20000, Q=48, bias_scale=0.0, preset=preset)
    k = 50
    ids, sc = ann.ann_search(g, m, users, entries, cfg.W, cfg.L, k, 0)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    for q in range(cfg.Q):
        r = ids[q][ids[q] >= 0]
        assert len(set(r.tolist())) == len(r)
        assert np.all(sc[q][: len(r) - 1] >= sc[q][1: len(r)])
    kern = oracle.search(v["emb"], v["adj"], v["users"], v["mlp_q"], v["entries"], cfg.W, cfg.L, k, 0, act_round=2,
                         n_threads=8)
    exact = oracle.search(v["emb_exact"], v["adj"], v["users"], v["mlp_exact"], v["entries"], cfg.W, cfg.L, k, 0,
                          n_threads=8)
    bf = oracle.brute_force(v["emb_exact"], v["users"][:16], v["mlp_exact"], k, n_threads=8)
    r_gpu = oracle.recall_at(ids[:16], bf["ids"], k)
    r_kern = oracle.recall_at(kern["ids"][:16], bf["ids"], k)
    r_exact = oracle.recall_at(exact["ids"][:16], bf["ids"], k)
    print(f"{preset} 8-bit search: recall@{k} against the exact metric's ranking: gpu {r_gpu:.4f}, oracle at the kernel's "
          f"precision {r_kern:.4f}, oracle with the unquantised metric {r_exact:.4f}; identical lists vs the "
          f"kernel-precision oracle {same_list_fraction(ids, kern['ids']):.3f}")
    assert abs(r_gpu - r_kern) <= 0.01 + 1e-9
    assert r_exact - r_gpu <= F8_RECALL_BUDGET, (r_exact, r_gpu)   # what the format may cost in recall
    valid = ids.ravel() >= 0
    qq = np.repeat(np.arange(cfg.Q), k).astype(np.int32)[valid]
    ref = oracle.score_pairs(v["emb"], v["users"], v["mlp_q"], qq, ids.ravel()[valid], act_round=2, n_threads=8)
    assert np.max(np.abs(sc.ravel()[valid] - ref)) <= 1e-2


def test_f8_metric_argument_errors():
    cfg = scaled(PRESETS["C4"], 2000, n_clusters=4, Q=4)
    wl = make_workload(cfg)
    with pytest.raises(ann.AnnError) as e:     # another shape
        ann.ann_mlp_load(wl["W"], wl["b"], wl["head_w"], cfg.d, ann.ANN_F8)
    assert e.value.code == -4   # ANN_ENOTIMPL
    cfg2 = scaled(PRESETS["C2"], 2000, n_clusters=4, Q=4)
    wl2 = make_workload(cfg2)
    big = [w.clone() for w in wl2["W"]]
    big[1][3, 5] = 200.0                       # 4 * 200 > 448
    with pytest.raises(ann.AnnError) as e:
        ann.ann_mlp_load(big, wl2["b"], wl2["head_w"], cfg2.d, ann.ANN_F8)
    assert e.value.code == -1   # ANN_EINVAL
    m8 = ann.ann_mlp_load(wl2["W"], wl2["b"], wl2["head_w"], cfg2.d, ann.ANN_F8)
    g16 = ann.ann_graph_load(wl2["adj"].cuda().contiguous(), wl2["emb"].cuda().contiguous())
    with pytest.raises(ann.AnnError):          # 8-bit metric on a bf16 table
        ann.ann_search(g16, m8, wl2["users"].cuda(), wl2["entries"].cuda(), cfg2.W, cfg2.L, 10, 0)
