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


# ------------------------------------------------------------------ the fixed binary32 operation order
# The codes that follow a normalisation have one right answer only because its arithmetic is a fixed sequence
# of IEEE operations.  These pins retrace that sequence with another library's binary32 operations (PyTorch CPU
# tensors: every torch op below rounds once to binary32) and ask for the same bits; each also shows that the
# neighbouring order of operations does NOT give the same bits, so a swap inside the oracle would fail here.
def _t32(bits):
    return torch.from_numpy(_f32(bits).copy())


def _seq_sum64(v):
    """Left-to-right binary64 sum of every row (numpy's cumulative sum adds in index order)."""
    return np.cumsum(v, axis=1)[:, -1]


def _bf16_bits_of(t):
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


# The two orders differ in the last binary32 bit for about half the elements, which moves the bfloat16 result of
# about one element in 2^17: the large case (2M elements) is there so that the other order is seen to differ.
@pytest.mark.parametrize("name,M", [("tiny", 16), ("llama7b_qkv", 512), ("llama13b_ffn_lorc", 5), ("llama70b_ffn_decode", 4)])
def test_rmsnorm_operation_order_retraced_in_binary32(name, M):
    cfg = CFG[name]
    X = inputs.make_x(cfg, M)
    g = _gain(cfg.K)
    eps = 1e-5
    x64 = _f32(X).astype(np.float64)
    ss = _seq_sum64(x64 * x64)                                        # squares of bf16 values are exact in binary64
    ms = torch.from_numpy((ss / float(cfg.K)).astype(np.float32))     # ms = fl32(ss / K)
    rstd = 1.0 / torch.sqrt(ms + torch.tensor(eps, dtype=torch.float32))
    assert rstd.dtype == torch.float32
    x, gg = _t32(X), _t32(g)
    want = _bf16_bits_of((x * rstd[:, None]) * gg[None, :])           # (x * rstd) * g
    got = oracle.rmsnorm_bf16(X, g, eps)
    assert np.array_equal(got, want)
    other = _bf16_bits_of(x * (rstd[:, None] * gg[None, :]))          # x * (rstd * g): another rounding
    if cfg.K * M >= 1 << 21:
        assert not np.array_equal(other, want)


@pytest.mark.parametrize("name,M", [("tiny", 16), ("opt1p3b_fc1", 9), ("llama7b_qkv", 512), ("llama70b_ffn_decode", 4)])
def test_layernorm_operation_order_retraced_in_binary32(name, M):
    cfg = CFG[name]
    X = _bf16(_f32(inputs.make_x(cfg, M)) + 0.75)
    g, b = _gain(cfg.K), _bias(cfg.K)
    eps = 1e-5
    x64 = _f32(X).astype(np.float64)
    s1, s2 = _seq_sum64(x64), _seq_sum64(x64 * x64)
    mean = s1 / float(cfg.K)
    var = np.maximum(s2 / float(cfg.K) - mean * mean, 0.0)
    mu = torch.from_numpy(mean.astype(np.float32))
    v = torch.from_numpy(var.astype(np.float32))
    rstd = 1.0 / torch.sqrt(v + torch.tensor(eps, dtype=torch.float32))
    x, gg, bb = _t32(X), _t32(g), _t32(b)
    d = x - mu[:, None]
    want = _bf16_bits_of(((d * rstd[:, None]) * gg[None, :]) + bb[None, :])
    got = oracle.layernorm_bf16(X, g, b, eps)
    assert np.array_equal(got, want)
    other = _bf16_bits_of((d * (rstd[:, None] * gg[None, :])) + bb[None, :])
    fused = _bf16_bits_of(torch.addcmul(bb[None, :].expand_as(d).to(torch.float64), (d * rstd[:, None]).to(torch.float64),
                                        gg[None, :].to(torch.float64).expand_as(d)).to(torch.float32))  # one rounding for a*g+b
    if cfg.K * M >= 1 << 21:
        assert not np.array_equal(other, want) and not np.array_equal(fused, want)
