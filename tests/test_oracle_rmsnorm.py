"""Pins of the oracle's RMS normalisation (the producer of the activations that
the paper's Section 3 quantizes token-wise): the textbook definition evaluated
in another precision by another library, closed forms, and invariants."""
import numpy as np
import pytest
import torch

import oracle
from paper_2307_09782_amd import inputs

CFG = inputs.CONFIGS


def _bf16(x):
    return inputs.f32_to_bf16_bits(np.asarray(x, np.float32))


def _f32(bits):
    return inputs.bf16_bits_to_f32(bits)


def _gain(K, seed=3):
    rng = np.random.default_rng(seed)
    return _bf16(1.0 + 0.1 * rng.standard_normal(K))


@pytest.mark.parametrize("name,M", [("tiny", 16), ("llama7b_qkv", 33), ("llama70b_ffn_decode", 4)])
def test_matches_float64_definition_within_one_bf16_step(name, M):
    cfg = CFG[name]
    X = inputs.make_x(cfg, M)
    g = _gain(cfg.K)
    eps = 1e-5
    Y = _f32(oracle.rmsnorm_bf16(X, g, eps)).astype(np.float64)
    x = torch.from_numpy(_f32(X).astype(np.float64))
    gg = torch.from_numpy(_f32(g).astype(np.float64))
    ref = (x * torch.rsqrt((x * x).mean(dim=1, keepdim=True) + eps) * gg).numpy()
    # a bf16 rounding of a value within a few binary32 ulps of ref: equal to bf16(ref) or its neighbour
    want = _f32(_bf16(ref.astype(np.float32))).astype(np.float64)
    step = np.abs(want) * 2.0 ** -7 + 1e-38
    assert np.all(np.abs(Y - want) <= step)
    assert (Y == want).mean() > 0.995
    # a dropped gain, a missing eps or mean-vs-sum would be far outside
    assert np.abs(Y - ref).max() <= np.abs(ref).max() * 2.0 ** -8


def test_constant_row_closed_form():
    # x = c everywhere: y = sign(c) * g / sqrt(1 + eps / c^2)
    K, eps = 256, 0.25
    for c in (2.0, -0.5, 8.0):
        X = _bf16(np.full((1, K), c))
        g = _gain(K)
        Y = _f32(oracle.rmsnorm_bf16(X, g, eps))[0]
        want = np.sign(c) * _f32(g).astype(np.float64) / np.sqrt(1.0 + eps / (c * c))
        assert np.all(np.abs(Y - want) <= np.abs(want) * 2.0 ** -8)
    # with c^2 >> eps and unit gain the output is exactly +-1 only if eps rounds away: here it does not
    Y1 = _f32(oracle.rmsnorm_bf16(_bf16(np.full((1, K), 1.0)), _bf16(np.ones(K)), 1.0))[0]
    assert np.all(Y1 == _f32(_bf16(np.float32(1.0) / np.sqrt(np.float32(2.0)))))


def test_power_of_two_input_scaling_cancels_when_eps_is_negligible():
    cfg = CFG["tiny"]
    X = inputs.make_x(cfg, 8)
    g = _gain(cfg.K)
    eps = 1e-30
    Y0 = oracle.rmsnorm_bf16(X, g, eps)
    X4 = _bf16(_f32(X) * 16.0)  # exact in bf16
    assert np.array_equal(oracle.rmsnorm_bf16(X4, g, eps), Y0)


def test_zero_row_unit_gain_and_sign():
    K = 128
    X = _bf16(np.zeros((2, K)))
    X[1, 5] = _bf16(np.array([-3.0]))[0]
    Y = _f32(oracle.rmsnorm_bf16(X, _bf16(np.ones(K)), 1e-6))
    assert np.all(Y[0] == 0)
    # one nonzero of K: x / sqrt(x^2 / K) = -sqrt(K)
    assert Y[1, 5] == _f32(_bf16(np.float32(-np.sqrt(K)))) and np.count_nonzero(Y[1]) == 1
    # the output's mean square is 1 for unit gain (up to bf16 rounding)
    Z = _f32(oracle.rmsnorm_bf16(inputs.make_x(CFG["tiny"], 4), _bf16(np.ones(256)), 1e-6)).astype(np.float64)
    assert np.all(np.abs((Z * Z).mean(axis=1) - 1.0) < 2.0 ** -7)  # bf16 rounding of the few dominant entries


def test_rejects_nonpositive_eps():
    with pytest.raises(ValueError):
        oracle.rmsnorm_bf16(_bf16(np.ones((1, 128))), _bf16(np.ones(128)), 0.0)


# ------------------------------------------------------------------ layer normalisation
def _bias(K, seed=4):
    rng = np.random.default_rng(seed)
    return _bf16(0.05 * rng.standard_normal(K))


@pytest.mark.parametrize("name,M", [("tiny", 16), ("opt1p3b_fc1", 33), ("llama70b_ffn_decode", 4)])
def test_layernorm_matches_float64_library_routine_within_one_bf16_step(name, M):
    cfg = CFG[name]
    X = inputs.make_x(cfg, M)
    X = _bf16(_f32(X) + 0.75)  # a non-zero mean, so that a dropped mean would show
    g, b = _gain(cfg.K), _bias(cfg.K)
    eps = 1e-5
    Y = _f32(oracle.layernorm_bf16(X, g, b, eps)).astype(np.float64)
    x = torch.from_numpy(_f32(X).astype(np.float64))
    ref = torch.nn.functional.layer_norm(x, (cfg.K,), torch.from_numpy(_f32(g).astype(np.float64)),
                                         torch.from_numpy(_f32(b).astype(np.float64)), eps).numpy()
    want = _f32(_bf16(ref.astype(np.float32))).astype(np.float64)
    step = np.abs(want) * 2.0 ** -7 + 2.0 ** -10   # near zero the gain*x and bias terms cancel: absolute slack
    assert np.all(np.abs(Y - want) <= step)
    assert (Y == want).mean() > 0.99
    assert np.abs(Y - ref).max() <= np.abs(ref).max() * 2.0 ** -8


def test_layernorm_closed_forms():
    K, eps = 256, 0.25
    g, b = _gain(K), _bias(K)
    # constant row: x - mean = 0 exactly, so y = b
    Y = oracle.layernorm_bf16(_bf16(np.full((1, K), 3.0)), g, b, eps)
    assert np.array_equal(Y[0], b)
    # +c, -c alternating: mean 0, variance c^2: y = +-g / sqrt(1 + eps / c^2) + b
    for c in (2.0, 0.5):
        x = np.where(np.arange(K) % 2 == 0, c, -c).astype(np.float32)[None, :]
        Y = _f32(oracle.layernorm_bf16(_bf16(x), g, b, eps))[0].astype(np.float64)
        want = np.sign(x[0]) * _f32(g).astype(np.float64) / np.sqrt(1.0 + eps / (c * c)) + _f32(b)
        assert np.all(np.abs(Y - want) <= np.abs(want) * 2.0 ** -8 + 2.0 ** -12)
    # zero gain leaves the bias, zero bias and unit gain give zero mean and unit variance
    assert np.array_equal(oracle.layernorm_bf16(inputs.make_x(CFG["tiny"], 2), _bf16(np.zeros(K)), b, eps)[0], b)
    Z = _f32(oracle.layernorm_bf16(inputs.make_x(CFG["tiny"], 4), _bf16(np.ones(K)), _bf16(np.zeros(K)), 1e-6)).astype(np.float64)
    assert np.all(np.abs(Z.mean(axis=1)) < 2e-3) and np.all(np.abs((Z * Z).mean(axis=1) - 1.0) < 2.0 ** -7)


def test_layernorm_power_of_two_scaling_cancels_when_eps_is_negligible():
    cfg = CFG["tiny"]
    X = inputs.make_x(cfg, 8)
    g, b = _gain(cfg.K), _bias(cfg.K)
    Y0 = oracle.layernorm_bf16(X, g, b, 1e-30)
    assert np.array_equal(oracle.layernorm_bf16(_bf16(_f32(X) * 8.0), g, b, 1e-30), Y0)
