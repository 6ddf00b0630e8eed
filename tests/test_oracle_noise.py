"""Pins of the oracle's serendipity-noise draw (Eq. 5): the generator against its published known-answer
vectors, the normal transform against the distribution it must produce, the array function against
its defining properties and an independent bf16 rounding."""
import json
import os

import numpy as np
import pytest
import torch
from scipy import stats

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    kat = json.load(open(os.path.join(GOLD, "philox4x32_10_kat.json")))
    for v in kat["vectors"]:
        got = oracle.philox4x32_10([int(x, 16) for x in v["ctr"]], [int(x, 16) for x in v["key"]])
        assert [f"{x:08x}" for x in got] == v["out"]


def _draws(n, seed=12345, stream=7):
    z = oracle.users_add_noise(np.zeros((n // 4, 4), np.float32), 1.0, seed, stream)
    return z.astype(np.float64)


def test_draws_are_standard_normal():
    z = _draws(400_000).ravel()
    assert abs(z.mean()) < 4 / np.sqrt(z.size)
    assert abs(z.var() - 1.0) < 4 * np.sqrt(2.0 / z.size)
    assert abs(stats.skew(z)) < 0.02 and abs(stats.kurtosis(z)) < 0.04
    assert stats.kstest(z, "norm").pvalue > 1e-3
    # both tails are there, and about as heavy as they should be
    assert abs((z > 3).mean() - stats.norm.sf(3)) < 3e-4 and abs((z < -3).mean() - stats.norm.sf(3)) < 3e-4


def test_the_two_words_of_a_pair_are_a_box_muller_pair():
    z = _draws(200_000)
    for a in (0, 2):
        x, y = z[:, a], z[:, a + 1]
        assert abs(np.corrcoef(x, y)[0, 1]) < 0.01
        # radius^2 is exponential with mean 2, the angle is uniform on the circle
        assert stats.kstest(x * x + y * y, "expon", args=(0, 2)).pvalue > 1e-3
        assert stats.kstest((np.arctan2(y, x) + np.pi) / (2 * np.pi), "uniform").pvalue > 1e-3
    # words of different pairs, and neighbouring blocks, are unrelated
    assert abs(np.corrcoef(z[:, 0], z[:, 2])[0, 1]) < 0.01
    assert abs(np.corrcoef(z[:-1, 3], z[1:, 0])[0, 1]) < 0.01


def test_element_numbering_seed_and_stream():
    # element e = q * d + c: the draw does not depend on how the array is shaped or how long it is
    a = oracle.users_add_noise(np.zeros((6, 10), np.float32), 1.0, 99, 3).ravel()
    b = oracle.users_add_noise(np.zeros((15, 4), np.float32), 1.0, 99, 3).ravel()
    c = oracle.users_add_noise(np.zeros((3, 10), np.float32), 1.0, 99, 3).ravel()
    assert np.array_equal(a, b) and np.array_equal(a[:30], c)
    for e in (0, 1, 2, 3, 4, 37, 59):
        assert np.float32(oracle.noise_element(99, 3, e)) == a[e]
    assert not np.array_equal(a, oracle.users_add_noise(np.zeros((6, 10), np.float32), 1.0, 100, 3).ravel())
    assert not np.array_equal(a, oracle.users_add_noise(np.zeros((6, 10), np.float32), 1.0, 99, 4).ravel())
    # the high halves of seed, stream and block index are used
    assert oracle.noise_element(1, 0, 5) != oracle.noise_element(1 + (1 << 32), 0, 5)
    assert oracle.noise_element(1, 0, 5) != oracle.noise_element(1, 1 << 32, 5)
    assert oracle.noise_element(1, 0, 5) != oracle.noise_element(1, 0, 5 + (1 << 34))


def test_noise_is_added_and_scaled():
    rng = np.random.default_rng(5)
    u = rng.standard_normal((50, 16)).astype(np.float32)
    assert np.array_equal(oracle.users_add_noise(u, 0.0, 1, 0), u)
    z = np.array([oracle.noise_element(8, 2, e) for e in range(u.size)]).reshape(u.shape)
    for sigma in (1.0, 0.25, 3.0):
        got = oracle.users_add_noise(u, sigma, 8, 2)
        assert np.array_equal(got, (u.astype(np.float64) + sigma * z).astype(np.float32))


def test_bf16_output_is_the_rounded_sum():
    rng = np.random.default_rng(6)
    u32 = rng.standard_normal((40, 24)).astype(np.float32)
    ub = torch.from_numpy(u32).to(torch.bfloat16)
    bits = ub.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.users_add_noise(bits, 0.0, 1, 0), bits)
    z = np.array([oracle.noise_element(21, 0, e) for e in range(u32.size)]).reshape(u32.shape)
    want = torch.from_numpy(ub.to(torch.float64).numpy() + 0.5 * z).to(torch.float32).to(torch.bfloat16)
    got = oracle.users_add_noise(bits, 0.5, 21, 0)
    assert np.array_equal(got, want.view(torch.int16).numpy().view(np.uint16))


def test_fp16_arrays_get_the_fp32_result_rounded_to_binary16():
    rng = np.random.default_rng(11)
    u = rng.standard_normal((50, 12)).astype(np.float16)
    out = oracle.users_add_noise(u, 0.7, 3, 2)
    wide = oracle.users_add_noise(u.astype(np.float32), 0.7, 3, 2)
    assert out.dtype == np.float16 and np.array_equal(out, wide.astype(np.float16))   # numpy's conversion
    assert np.array_equal(oracle.users_add_noise(u, 0.0, 3, 2), u)
