"""Parity of the on-device serendipity noise (Eq. 5) with the oracle's draw, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_11490_amd as ann

pytestmark = pytest.mark.gpu


def _ulps_f32(a, b):
    ia, ib = a.view(np.int32).astype(np.int64), b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, -(ia & 0x7fffffff), ia)
    ib = np.where(ib < 0, -(ib & 0x7fffffff), ib)
    return np.abs(ia - ib)


@pytest.mark.parametrize("Q,d", [(1, 1), (3, 5), (257, 64), (4096, 128)])
@pytest.mark.parametrize("sigma,seed,draw", [(1.0, 2025, 0), (0.3, (7 << 40) + 11, (3 << 33) + 1)])
def test_noise_fp32_matches_oracle(Q, d, sigma, seed, draw):
    rng = np.random.default_rng(Q * 1000 + d)
    u = rng.standard_normal((Q, d)).astype(np.float32)
    got = ann.ann_users_add_noise(torch.from_numpy(u).cuda(), sigma, seed, draw).cpu().numpy()
    want = oracle.users_add_noise(u, sigma, seed, draw)
    # both sides sum in fp64 and round once; the libraries' fp64 log / sin / cos may differ in their last
    # bit, which can move a sum across an fp32 rounding boundary: at most a few elements, by one ulp
    ulps = _ulps_f32(got, want)
    assert ulps.max() <= 1
    assert (ulps != 0).sum() <= max(2, got.size // 100000)


def test_noise_bf16_matches_oracle():
    rng = np.random.default_rng(3)
    u = torch.from_numpy(rng.standard_normal((4096, 128)).astype(np.float32)).to(torch.bfloat16)
    bits = u.view(torch.int16).numpy().view(np.uint16)
    got = ann.ann_users_add_noise(u.cuda(), 1.0, 5, 9).cpu().view(torch.int16).numpy().view(np.uint16)
    want = oracle.users_add_noise(bits, 1.0, 5, 9)
    assert (got != want).sum() <= 2
    assert np.abs(got.astype(np.int32) - want.astype(np.int32)).max() <= 1


def test_noise_f16_matches_oracle():
    rng = np.random.default_rng(4)
    u = torch.from_numpy(rng.standard_normal((4096, 128)).astype(np.float32)).to(torch.float16)
    got = ann.ann_users_add_noise(u.cuda(), 1.0, 5, 9).cpu().numpy()
    want = oracle.users_add_noise(u.numpy(), 1.0, 5, 9)
    assert got.dtype == np.float16 and want.dtype == np.float16
    gb, wb = got.view(np.uint16).astype(np.int32), want.view(np.uint16).astype(np.int32)
    assert (gb != wb).sum() <= 2 and np.abs(gb - wb).max() <= 1


def test_noise_in_place_zero_sigma_empty_and_errors():
    u = torch.randn(33, 7, device="cuda")
    keep = u.clone()
    assert torch.equal(ann.ann_users_add_noise(u, 0.0, 1), keep)
    fresh = ann.ann_users_add_noise(u, 1.0, 1, 2)
    ann.ann_users_add_noise(u, 1.0, 1, 2, out=u)
    assert torch.equal(u, fresh) and not torch.equal(u, keep)
    e = torch.empty(0, 7, device="cuda")
    assert ann.ann_users_add_noise(e, 1.0, 1).shape == (0, 7)
    for bad in (-1.0, float("nan"), float("inf")):
        with pytest.raises(ann.AnnError):
            ann.ann_users_add_noise(keep, bad, 1)
    with pytest.raises(TypeError):
        ann.ann_users_add_noise(keep.double(), 1.0, 1)


def test_search_on_noisy_users_matches_oracle_on_the_oracles_noisy_users():
    import os
    import sys
    sys.path.insert(0, os.path.dirname(__file__))
    from gpu_util import open_handles, oracle_mlp, same_list_fraction
    from workloads import PRESETS, make_workload, scaled, to_host
    cfg = scaled(PRESETS["C1"], 4000, n_clusters=8, Q=32)
    wl = make_workload(cfg, seed=9)
    g, m, dev = open_handles(wl)
    h = to_host(wl)
    noisy = ann.ann_users_add_noise(dev["users"], 1.0, 77, 1)
    noisy_ref = oracle.users_add_noise(h["users"], 1.0, 77, 1)
    assert _ulps_f32(noisy.cpu().numpy(), noisy_ref).max() <= 1
    assert np.abs(noisy_ref - h["users"]).std() > 0.5   # the vectors really moved
    ids, sc = ann.ann_search(g, m, noisy, dev["entries"], cfg.W, cfg.L, cfg.k, 0)
    ref = oracle.search(h["emb"], h["adj"], noisy_ref, oracle_mlp(h), h["entries"], cfg.W, cfg.L, cfg.k, 0, n_threads=8)
    plain = oracle.search(h["emb"], h["adj"], h["users"], oracle_mlp(h), h["entries"], cfg.W, cfg.L, cfg.k, 0, n_threads=8)
    assert same_list_fraction(ids.cpu().numpy(), ref["ids"]) >= 0.99
    assert same_list_fraction(ref["ids"], plain["ids"]) < 0.5   # and the results moved with them
