"""Pins for the oracle's relevance metric (Sec. 3.1 (1), Eq. 5-8).

The oracle is checked against things that are not itself: hand-worked values
(tests/golden/mlp_hand_cases.json), closed forms, a library MLP forward pass
(scikit-learn) with a library sigmoid (scipy), and exactness of the bf16 path.
"""
import json
import os

import numpy as np
import pytest
from scipy.special import expit
from sklearn.neural_network import MLPRegressor

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _score_one(user, item, W, b, head_w, **kw):
    emb = np.asarray([item], dtype=np.float32)
    users = np.asarray([user], dtype=np.float32)
    mlp = oracle.Mlp([np.asarray(w, dtype=np.float32) for w in W],
                     [np.asarray(x, dtype=np.float32) for x in b],
                     np.asarray(head_w, dtype=np.float32))
    return float(oracle.score_pairs(emb, users, mlp, np.array([0]), np.array([0]), **kw)[0])


@pytest.mark.parametrize("case", json.load(open(os.path.join(GOLD, "mlp_hand_cases.json")))["cases"],
                         ids=lambda c: c["name"])
def test_hand_worked_values(case):
    got = _score_one(case["user"], case["item"], case["W"], case["b"], case["head_w"])
    assert got == pytest.approx(case["expected"], rel=0, abs=1e-7)


def test_all_zero_parameters_give_half_the_weight_sum():
    # Eq. 8 with every logit 0: sum_j w_j / 2, exactly representable here
    rng = np.random.default_rng(0)
    dims = [12, 9, 7, 4]
    W = [np.zeros((dims[i + 1], dims[i]), np.float32) for i in range(3)]
    b = [np.zeros(dims[i + 1], np.float32) for i in range(3)]
    hw = np.array([0.5, 0.25, 0.125, 0.0625], np.float32)
    mlp = oracle.Mlp(W, b, hw)
    emb = rng.standard_normal((50, 6)).astype(np.float32)
    users = rng.standard_normal((5, 6)).astype(np.float32)
    q = rng.integers(0, 5, 200)
    it = rng.integers(0, 50, 200)
    s = oracle.score_pairs(emb, users, mlp, q, it)
    assert np.all(s == np.float32(0.46875))


def test_single_head_bias_only():
    # zero last-layer weights, bias beta, one head of weight 1: sigmoid(beta)
    for beta in (-3.0, -0.5, 0.0, 1.25, 6.0):
        W = [np.ones((4, 6), np.float32), np.zeros((1, 4), np.float32)]
        b = [np.zeros(4, np.float32), np.array([beta], np.float32)]
        got = _score_one([1, 2, 3], [4, 5, 6], W, b, [1.0])
        assert got == pytest.approx(float(expit(np.float64(beta))), abs=6e-8)


def _library_scores(emb, users, W, b, head_w, q, it):
    """scikit-learn's MLP forward (ReLU hidden, identity output) + scipy's logistic."""
    reg = MLPRegressor(hidden_layer_sizes=tuple(w.shape[0] for w in W[:-1]), activation="relu")
    reg.coefs_ = [np.asarray(w, np.float64).T.copy() for w in W]
    reg.intercepts_ = [np.asarray(x, np.float64) for x in b]
    reg.n_layers_ = len(W) + 1
    reg.n_outputs_ = W[-1].shape[0]
    reg.out_activation_ = "identity"
    reg.n_features_in_ = W[0].shape[1]
    X = np.concatenate([users[q], emb[it]], axis=1).astype(np.float64)
    Z = reg.predict(X).reshape(len(q), -1)
    return expit(Z) @ np.asarray(head_w, np.float64)


@pytest.mark.parametrize("dims,seed", [([64, 64, 3], 1), ([128, 256, 128, 3], 2), ([24, 40, 16, 8, 4], 3),
                                       ([10, 5], 4)])
def test_matches_library_mlp_forward(dims, seed):
    rng = np.random.default_rng(seed)
    d = dims[0] // 2
    W = [(rng.standard_normal((dims[i + 1], dims[i])) * np.sqrt(2.0 / dims[i])).astype(np.float32)
         for i in range(len(dims) - 1)]
    b = [(0.3 * rng.standard_normal(dims[i + 1])).astype(np.float32) for i in range(len(dims) - 1)]
    hw = rng.random(dims[-1]).astype(np.float32)
    emb = rng.standard_normal((300, d)).astype(np.float32)
    users = rng.standard_normal((20, d)).astype(np.float32)
    q = rng.integers(0, 20, 1500)
    it = rng.integers(0, 300, 1500)
    got = oracle.score_pairs(emb, users, oracle.Mlp(W, b, hw), q, it, n_threads=4)
    if len(dims) == 2:  # no hidden layer: sklearn needs one, use the direct expression
        X = np.concatenate([users[q], emb[it]], axis=1).astype(np.float64)
        want = expit(X @ W[0].astype(np.float64).T + b[0]) @ hw.astype(np.float64)
    else:
        want = _library_scores(emb, users, W, b, hw, q, it)
    np.testing.assert_allclose(got, want.astype(np.float32), rtol=2e-7, atol=0)


def test_unequal_user_and_item_widths():
    rng = np.random.default_rng(5)
    du, d = 3, 7
    W = [rng.standard_normal((6, du + d)).astype(np.float32), rng.standard_normal((2, 6)).astype(np.float32)]
    b = [rng.standard_normal(6).astype(np.float32), rng.standard_normal(2).astype(np.float32)]
    hw = np.array([0.7, 0.3], np.float32)
    emb = rng.standard_normal((40, d)).astype(np.float32)
    users = rng.standard_normal((4, du)).astype(np.float32)
    q = rng.integers(0, 4, 100)
    it = rng.integers(0, 40, 100)
    got = oracle.score_pairs(emb, users, oracle.Mlp(W, b, hw), q, it)
    want = _library_scores(emb, users, W, b, hw, q, it)
    np.testing.assert_allclose(got, want.astype(np.float32), rtol=2e-7)


def _to_bf16_bits(x):
    import torch

    return torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_bf16_tables_equal_their_widened_values():
    # bf16 inputs are used exactly as stored: same result as passing the widened fp32 values
    rng = np.random.default_rng(6)
    dims = [32, 48, 3]
    W = [(rng.standard_normal((dims[i + 1], dims[i])) * 0.2).astype(np.float32) for i in range(2)]
    b = [np.zeros(dims[i + 1], np.float32) for i in range(2)]
    hw = np.array([0.5, 0.3, 0.2], np.float32)
    emb_bits = _to_bf16_bits(rng.standard_normal((100, 16)))
    usr_bits = _to_bf16_bits(rng.standard_normal((8, 16)))
    W_bits = [_to_bf16_bits(w) for w in W]
    q = rng.integers(0, 8, 300)
    it = rng.integers(0, 100, 300)
    a = oracle.score_pairs(emb_bits, usr_bits, oracle.Mlp(W_bits, b, hw), q, it)
    Wf = [oracle.widen_bf16(w) for w in W_bits]
    c = oracle.score_pairs(oracle.widen_bf16(emb_bits), oracle.widen_bf16(usr_bits), oracle.Mlp(Wf, b, hw), q, it)
    assert np.array_equal(a, c)
    # and widening is the IEEE definition: known bit patterns
    assert oracle.widen_bf16(np.array([0x3F80, 0xC000, 0x3DCD, 0x0000], np.uint16)).tolist() == \
        [1.0, -2.0, 0.10009765625, 0.0]


def test_activation_rounding_option_rounds_to_nearest_even_bf16():
    # hidden unit = user value passed through an identity weight; head logit = that unit.
    # bf16 keeps 8 significant bits: 1+3/256 is a tie between 1+2/256 and 1+4/256 -> even -> 1+4/256;
    # 1+1/256 is a tie between 1 and 1+2/256 -> even -> 1; 1+1/512 rounds down to 1.
    W = [np.array([[1.0, 0.0]], np.float32), np.array([[1.0]], np.float32)]
    b = [np.zeros(1, np.float32), np.zeros(1, np.float32)]
    for x, rounded in ((1 + 3 / 256, 1 + 4 / 256), (1 + 1 / 256, 1.0), (1 + 1 / 512, 1.0), (-0.75, 0.0),
                       (1.5, 1.5)):
        exact = _score_one([x], [0.0], W, b, [1.0])
        kern = _score_one([x], [0.0], W, b, [1.0], act_round=1)
        assert exact == pytest.approx(float(expit(max(x, 0.0))), abs=6e-8)
        assert kern == pytest.approx(float(expit(rounded)), abs=6e-8)


def test_rejects_out_of_range_pairs_and_bad_dims():
    emb = np.zeros((4, 2), np.float32)
    users = np.zeros((2, 2), np.float32)
    mlp = oracle.Mlp([np.zeros((1, 4), np.float32)], [np.zeros(1, np.float32)], np.ones(1, np.float32))
    with pytest.raises(ValueError):
        oracle.score_pairs(emb, users, mlp, np.array([0]), np.array([4]))
    with pytest.raises(ValueError):
        oracle.score_pairs(emb, users, mlp, np.array([2]), np.array([0]))
    bad = oracle.Mlp([np.zeros((1, 5), np.float32)], [np.zeros(1, np.float32)], np.ones(1, np.float32))
    with pytest.raises(ValueError):
        oracle.score_pairs(emb, users, bad, np.array([0]), np.array([0]))


# ----------------------------------------------------------------------------- the 8-bit (e4m3) metric
def _e4m3_value(code):
    """An e4m3 code's value from the format's definition (sign, 4 exponent bits with bias 7, 3 mantissa
    bits, no infinities, exponent 15 / mantissa 7 is NaN)."""
    s = -1.0 if code & 0x80 else 1.0
    e, m = (code >> 3) & 15, code & 7
    if e == 15 and m == 7:
        return float("nan")
    return s * (m / 8 * 2.0 ** -6 if e == 0 else 2.0 ** (e - 7) * (1 + m / 8))


def test_e4m3_codes_round_trip_and_known_values():
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8)
    values = np.array([_e4m3_value(int(c)) for c in codes], np.float32)
    assert np.array_equal(oracle.e4m3_encode(values), codes)
    assert np.array_equal(oracle.e4m3_quantize(values), values)
    # 1 -> 0x38, -2 -> 0xC0, largest 448 -> 0x7E, smallest subnormal 2^-9 -> 0x01
    assert oracle.e4m3_encode(np.array([1.0, -2.0, 448.0, 2.0 ** -9], np.float32)).tolist() == [0x38, 0xC0, 0x7E, 0x01]
    # ties go to the even mantissa: between 1 (m=0) and 1.125 (m=1) -> 1; between 1.125 and 1.25 (m=2) -> 1.25;
    # between the subnormals 1/512 and 2/512 -> 2/512; half of the smallest subnormal -> 0
    assert oracle.e4m3_quantize(np.array([1.0625, 1.1875, 3 / 1024, 1 / 1024], np.float32)).tolist() == \
        [1.0, 1.25, 2 / 512, 0.0]
    # the scale is applied before and taken out after
    assert oracle.e4m3_quantize(np.array([0.3], np.float32), 4.0).tolist() == [1.25 / 4]
    with pytest.raises(ValueError):
        oracle.e4m3_encode(np.array([500.0], np.float32))
    with pytest.raises(ValueError):
        oracle.e4m3_quantize(np.array([120.0], np.float32), 4.0)


def test_e4m3_rounding_equals_a_library_conversion():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000) * s for s in (1e-3, 1e-2, 0.1, 1, 10, 100)]).astype(np.float32)
    x = x[np.abs(x) <= 448]
    t = torch.from_numpy(x).to(torch.float8_e4m3fn)
    assert np.array_equal(oracle.e4m3_encode(x), t.view(torch.uint8).numpy())
    assert np.array_equal(oracle.e4m3_quantize(x), t.to(torch.float32).numpy())


def test_activation_rounding_option_rounds_to_e4m3_at_the_layers_scale():
    # one hidden layer (scale 4): the unit passes x through; the logit is the quantised unit.
    W = [np.array([[1.0, 0.0]], np.float32), np.array([[1.0]], np.float32)]
    b = [np.zeros(1, np.float32), np.zeros(1, np.float32)]
    # 4x = 1.0625 is a tie -> 1 -> 0.25;  4x = 1.2 -> 1.25 -> 0.3125;  relu first;  clamp at 448 / 4 = 112
    for x, rounded in ((1.0625 / 4, 0.25), (0.3, 0.3125), (-3.0, 0.0), (200.0, 112.0), (1 / 4096, 0.0)):
        assert _score_one([x], [0.0], W, b, [1.0], act_round=2) == pytest.approx(float(expit(rounded)), abs=6e-8)
    # two hidden layers: the second one is quantised at scale 16 (0.3 * 16 = 4.8 -> 5 -> 0.3125; 20 -> 448 / 16)
    W2 = [np.array([[1.0, 0.0]], np.float32), np.array([[1.0]], np.float32), np.array([[1.0]], np.float32)]
    b2 = [np.zeros(1, np.float32)] * 3
    assert _score_one([0.3125], [0.0], W2, b2, [1.0], act_round=2) == pytest.approx(float(expit(0.3125)), abs=6e-8)
    b2s = [np.zeros(1, np.float32), np.array([0.0195], np.float32), np.zeros(1, np.float32)]
    # 0.3125 + 0.0195 = 0.332 -> x16 = 5.312 -> 5.5 -> 0.34375
    assert _score_one([0.3125], [0.0], W2, b2s, [1.0], act_round=2) == pytest.approx(float(expit(0.34375)), abs=6e-8)
    assert _score_one([40.0], [0.0], W2, b2, [1.0], act_round=2) == pytest.approx(float(expit(28.0)), abs=6e-8)


# ----------------------------------------------------------------------------- the fp16 metric
def test_f16_rounding_equals_a_library_conversion_and_known_values():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(100000) * s for s in (1e-7, 1e-5, 1e-3, 0.1, 1, 10, 1000, 30000)])
    x = x.astype(np.float32)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).astype(np.float32)     # numpy's conversion: IEEE nearest even
    got = oracle.f16_round(x)
    assert np.array_equal(got, want)
    assert np.isinf(got).any() and (got == 0).any()        # the sample reaches both ends of the range
    # by hand: 11 significant bits -> spacing 2^-10 at 1: the tie 1 + 2^-11 goes to the even 1, 1 + 3 * 2^-11 to
    # 1 + 2^-9 ... (even mantissa 2); largest value 65504, 65520 is the tie that goes to infinity;
    # smallest subnormal 2^-24, half of it goes to zero
    hand = np.array([1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 65504.0, 65519.0, 65520.0, -65520.0, 2.0 ** -24, 2.0 ** -25,
                     3 * 2.0 ** -25, -0.0], np.float32)
    out = oracle.f16_round(hand)
    assert out.tolist() == [1.0, 1 + 2.0 ** -9, 65504.0, 65504.0, np.inf, -np.inf, 2.0 ** -24, 0.0, 2.0 ** -23, 0.0]
    assert np.signbit(out[-1])


def test_activation_rounding_option_rounds_to_f16():
    W = [np.array([[1.0, 0.0]], np.float32), np.array([[1.0]], np.float32)]
    b = [np.zeros(1, np.float32), np.zeros(1, np.float32)]
    for x, rounded in ((1 + 2.0 ** -11, 1.0), (1 + 3 * 2.0 ** -11, 1 + 2.0 ** -9), (-3.0, 0.0), (0.1, 0.0999755859375)):
        assert _score_one([x], [0.0], W, b, [1.0], act_round=3) == pytest.approx(float(expit(rounded)), abs=6e-8)
    # without the option the activation is not rounded
    assert _score_one([0.1], [0.0], W, b, [1.0]) == pytest.approx(float(expit(np.float32(0.1))), abs=6e-8)
