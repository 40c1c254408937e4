"""Pins of the oracle's token-wise activation quantizer (Section 3, Appendix A)
and of its group-wise FP4 weight quantizer with power-of-two scales (Section 3,
methods M1 and M2).  CPU only."""
import math
import os
from fractions import Fraction

import numpy as np
import torch

import oracle
from paper_2307_09782_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
E2M1_VALUES = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def _golden(name):
    return [l.split("#")[0].split() for l in open(os.path.join(GOLDEN, name)) if l.split("#")[0].split()]


def _bf16(a):
    return inputs.f32_to_bf16_bits(np.asarray(a, np.float32))


def _e4m3_values():
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()


# ------------------------------------------------------------ act quantizer
def test_quantizer_hand_row():
    """amax = 448 makes the scale 1, so codes are the hand-derived E4M3 codes."""
    rows = [(float(v), int(c, 16)) for v, c, *_ in _golden("e4m3_hand_cases.txt") if abs(float(v)) <= 448]
    x = np.array([[v for v, _ in rows]], np.float32)
    assert np.array_equal(inputs.bf16_bits_to_f32(_bf16(x)), x)  # all are bfloat16 numbers
    Xq, sx = oracle.quantize_act(_bf16(x))
    assert sx[0] == 1.0
    assert list(Xq[0]) == [c for _, c in rows]


def test_quantizer_roundtrips_scaled_e4m3_grid():
    """A row made of every E4M3 value times 2^j is reproduced exactly."""
    vals = _e4m3_values()
    codes = np.array([c for c in range(256) if not math.isnan(vals[c])], np.uint8)
    for j in (-20, -3, 0, 5, 40):
        x = (vals[codes] * 2.0 ** j).astype(np.float32)[None, :]
        Xq, sx = oracle.quantize_act(_bf16(x))
        assert sx[0] == np.float32(2.0 ** j)
        assert np.array_equal(Xq[0], codes)


def test_quantizer_power_of_two_row_scaling_changes_only_sx():
    cfg = inputs.CONFIGS["tiny"]
    X = inputs.make_x(cfg, 16)
    Xq0, sx0 = oracle.quantize_act(X)
    for j in (-7, 3, 11):
        Xs = _bf16(inputs.bf16_bits_to_f32(X) * np.float32(2.0 ** j))
        Xq, sx = oracle.quantize_act(Xs)
        assert np.array_equal(Xq, Xq0)
        assert np.array_equal(sx, sx0 * np.float32(2.0 ** j))


def test_quantizer_matches_torch_ops_and_error_bound():
    """Library special case: the same binary32 sequence with PyTorch CPU ops and
    PyTorch's float8 conversion; plus the half-ulp reconstruction bound."""
    cfg = inputs.CONFIGS["tiny"]
    X = inputs.make_x(cfg, 16)
    Xq, sx = oracle.quantize_act(X)
    xf = torch.from_numpy(inputs.bf16_bits_to_f32(X))
    amax = xf.abs().amax(dim=1)
    assert np.array_equal(sx, (amax / torch.full_like(amax, 448.0)).numpy())
    # tensor / tensor is a true binary32 division (scalar / tensor multiplies by a reciprocal)
    y = xf * (torch.full_like(amax, 448.0) / amax)[:, None]
    ref = y.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(Xq, ref)
    assert Xq.max() <= 0xFE and not np.any((Xq & 0x7F) == 0x7F)
    # every row uses the top code for its largest element
    assert np.all((Xq & 0x7F).max(axis=1) == 0x7E)
    dec = _e4m3_values()[Xq]
    ya = np.abs(y.numpy().astype(np.float64))
    ulp = np.where(ya < 2.0 ** -6, 2.0 ** -9, 2.0 ** (np.floor(np.log2(np.maximum(ya, 1e-30))) - 3))
    assert np.all(np.abs(dec - y.numpy()) <= ulp / 2 + 1e-12)


def test_quantizer_zero_and_tiny_rows():
    x = np.zeros((3, 64), np.float32)
    x[1, 5] = -0.0
    x[2, :] = 2.0 ** -100
    x[2, 7] = -(2.0 ** -100)
    Xq, sx = oracle.quantize_act(_bf16(x))
    assert np.all(sx == 1.0)
    assert Xq[0].max() == 0 and Xq[1, 5] == 0x80 and Xq[2, 7] == 0x80 and Xq[2, 0] == 0


# ------------------------------------------------------------ weight packer
def _column_with_absmax(a, G, sign=1.0):
    col = np.linspace(-0.9, 0.9, G).astype(np.float32) * np.float32(a)
    col[3] = sign * a
    return col


def test_m1_hand_exponents():
    G = 32
    rows = [r for r in _golden("pow2_scale_hand_cases.txt") if r[0] == "M1"]
    W = np.stack([_column_with_absmax(float(a), G, -1.0 if i % 2 else 1.0) for i, (_, a, _n) in enumerate(rows)], axis=1)
    codes, exps, c, clipped = oracle.pack_weight(_bf16(W), G, 1)
    assert [int(e) - 127 for e in exps[0]] == [int(n) for _, _, n in rows]
    assert np.all(c == 1.0) and clipped == 0


def test_m2_hand_shifts():
    G = 32
    rows = [r for r in _golden("pow2_scale_hand_cases.txt") if r[0] == "M2"]
    # one column: group 0 carries absmax_max, the following groups the listed absmax_i
    amax_max = float(rows[0][1])
    groups = [_column_with_absmax(amax_max, G)] + [_column_with_absmax(float(a), G) for _, _, a, _k in rows]
    W = np.concatenate(groups)[:, None]
    codes, exps, c, clipped = oracle.pack_weight(_bf16(W), G, 2)
    assert c[0] == np.float32(amax_max) / np.float32(6)
    assert int(exps[0, 0]) == 127
    assert [127 - int(e) for e in exps[1:, 0]] == [int(k) for *_, k in rows]


def _dequant(codes, exps, c, G):
    val = np.array(E2M1_VALUES + [-v for v in E2M1_VALUES])[codes]
    scale = c[None, :].astype(np.float64) * 2.0 ** (np.repeat(exps.astype(np.int64), G, axis=0) - 127)
    return val * scale, scale


def test_m1_invariants_random():
    cfg = inputs.CONFIGS["tiny"]
    W = inputs.make_w(cfg)
    G = cfg.G
    codes, exps, c, clipped = oracle.pack_weight(W, G, 1)
    assert clipped == 0 and codes.max() <= 15
    w = inputs.bf16_bits_to_f32(W).astype(np.float64)
    amax = np.abs(w).reshape(-1, G, w.shape[1]).max(axis=1)
    S_hat = 2.0 ** (exps.astype(np.int64) - 127)
    S = amax / 6
    assert np.all(S <= S_hat) and np.all(S_hat < 2 * S)  # S <= 2^ceil(log2 S) < 2S
    # the group's absmax element lands on magnitude 3, 4 or 6 (amax / S^ in (3, 6])
    top = (codes & 7).reshape(-1, G, w.shape[1]).max(axis=1)
    assert np.all(top >= 5)
    # nearest-value property in exact arithmetic on a sample of elements
    wq, scale = _dequant(codes, exps, c, G)
    rng = np.random.default_rng(0)
    for k, n in zip(rng.integers(0, w.shape[0], 300), rng.integers(0, w.shape[1], 300)):
        y = Fraction(float(w[k, n])) / Fraction(float(scale[k, n]))
        d = [abs(abs(y) - Fraction(v)) for v in E2M1_VALUES]
        assert d[codes[k, n] & 7] == min(d)
    assert np.all(np.abs(wq - w) <= scale)  # largest gap on the grid is 2 -> half gap = 1


def test_m2_invariants_random():
    cfg = inputs.CONFIGS["tiny"]
    G = 32
    w = inputs.bf16_bits_to_f32(inputs.make_w(cfg)).copy()
    w[64:96, :] *= 0.25  # make group maxima differ clearly
    w[128:160, ::2] *= 3.0
    W = _bf16(w)
    w = inputs.bf16_bits_to_f32(W).astype(np.float64)
    codes, exps, c, clipped = oracle.pack_weight(W, G, 2)
    amax = np.abs(w).reshape(-1, G, w.shape[1]).max(axis=1)
    S = amax / 6
    assert np.array_equal(c, (amax.max(axis=0).astype(np.float32) / np.float32(6)))
    k = 127 - exps.astype(np.int64)
    assert np.all(k >= 0) and np.all(k[amax.argmax(axis=0), np.arange(w.shape[1])] == 0)
    S_hat = c[None, :].astype(np.float64) * 2.0 ** (-k)
    # S_i / 2 < S^_i <= S_i up to the one rounding of c to binary32
    assert np.all(S_hat <= S * (1 + 2.0 ** -23)) and np.all(S_hat > S / 2 * (1 - 2.0 ** -23))
    # with ceil the scale is rounded DOWN, so group maxima may saturate
    y = np.abs(w) / np.repeat(S_hat, G, axis=0)
    # (the oracle decides "> 6" on its binary32 quotient; allow for that one rounding here)
    assert int((y > 6 * (1 + 1e-6)).sum()) <= clipped <= int((y > 6 * (1 - 1e-6)).sum())
    assert clipped > 0
    assert np.all((codes & 7)[y > 6.0001] == 7)


def test_m2_equals_unconstrained_when_all_groups_share_absmax():
    G = 32
    w = np.random.default_rng(1).uniform(-0.05, 0.05, (128, 8)).astype(np.float32)
    w[3::32, :] = 0.0625
    W = _bf16(w)
    codes, exps, c, clipped = oracle.pack_weight(W, G, 2)
    assert np.all(exps == 127) and np.all(c == np.float32(0.0625) / np.float32(6))
    # codes are then the plain real-scale quantization of w / (amax/6)
    y = inputs.bf16_bits_to_f32(W) / c[None, :]
    want = np.array([[oracle.e2m1_encode(float(v)) for v in row] for row in y], np.uint8)
    assert np.array_equal(codes, want)


def test_zero_groups():
    G = 32
    w = np.zeros((64, 2), np.float32)
    w[40, 1] = 0.5
    c1, e1, s1, _ = oracle.pack_weight(_bf16(w), G, 1)
    assert e1[0, 0] == 127 and e1[1, 0] == 127 and e1[0, 1] == 127 and np.all(c1[:, 0] == 0)
    c2, e2, s2, _ = oracle.pack_weight(_bf16(w), G, 2)
    assert s2[0] == 1.0 and np.all(e2[:, 0] == 127 - 15) and e2[0, 1] == 127 - 15 and e2[1, 1] == 127
    assert c2[40, 1] == 7
