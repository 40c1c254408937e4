"""Pins for the oracle's other producers of quantized activations: residual add, ReLU (Section 3,
"Distribution of Activations"), gated SiLU.  None of the expected values below comes from the oracle
or the HIP path: they are closed forms, exact rational arithmetic, and independent library routines."""
from fractions import Fraction

import numpy as np
import torch

import oracle
from paper_2307_09782_amd import inputs


def _bits(vals):
    """Exactly representable values -> bf16 bits (asserts exactness)."""
    a = np.asarray(vals, np.float32)
    b = (a.view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal((b.astype(np.uint32) << 16).view(np.float32), a), "not a bfloat16 value"
    return b


def _vals(bits):
    return (np.asarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32)


def _round_fraction(x, sig_bits, emin):
    """Exact rational -> nearest binary floating-point value with `sig_bits` significant bits (ties to
    even, gradual underflow below 2^emin), as a Fraction."""
    if x == 0:
        return Fraction(0)
    s, a = (-1 if x < 0 else 1), abs(x)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    e = max(e, emin)
    ulp = Fraction(2) ** (e - sig_bits + 1)
    q, r = divmod(a, ulp)
    if r * 2 > ulp or (r * 2 == ulp and q % 2 == 1):
        q += 1
    return s * q * ulp


def _to_bf16_via_f32(x):
    """fl32 first, then bfloat16 (both round-to-nearest-even), in exact arithmetic."""
    return _round_fraction(_round_fraction(x, 24, -126), 8, -126)


# ---------------------------------------------------------------- residual add
def test_add_worked_examples_of_rounding():
    cases = [  # x, r, expected
        (1.0, 2.0 ** -8, 1.0),                        # tie between 1 and 1 + 2^-7: even
        (1.0 + 2.0 ** -7, 2.0 ** -8, 1.0 + 2.0 ** -6),  # tie, odd neighbour below: rounds up to even
        (256.0, 1.0, 256.0),                          # 257 is a tie between 256 and 258
        (258.0, 1.0, 260.0),                          # 259 is a tie between 258 and 260: even is 260
        (1.0, 2.0 ** -9, 1.0), (1.0, 3 * 2.0 ** -9, 1.0 + 2.0 ** -7),
        (3.0, -3.0, 0.0), (0.5, 0.0, 0.5), (-0.0, 0.0, 0.0), (1.5, 2.25, 3.75),
        (2.0 ** 100, 2.0 ** -100, 2.0 ** 100),
    ]
    X = _bits([[c[0] for c in cases]])
    R = _bits([[c[1] for c in cases]])
    H = oracle.add_bf16(X, R)
    assert np.array_equal(_vals(H)[0], np.array([c[2] for c in cases], np.float32))
    assert H[0, 6] == 0 and H[0, 8] == 0  # x + (-x) and -0 + 0 are +0


def test_add_equals_exact_rational_sum_rounded_and_a_tensor_library():
    rng = np.random.default_rng(11)
    x = (rng.standard_normal((4, 512)) * np.exp2(rng.integers(-12, 12, (4, 512)))).astype(np.float32)
    r = (rng.standard_normal((4, 512)) * np.exp2(rng.integers(-12, 12, (4, 512)))).astype(np.float32)
    X, R = inputs.f32_to_bf16_bits(x), inputs.f32_to_bf16_bits(r)
    H = oracle.add_bf16(X, R)
    xv, rv, hv = _vals(X), _vals(R), _vals(H)
    for i in range(0, 512, 7):
        exact = Fraction(float(xv[0, i])) + Fraction(float(rv[0, i]))
        assert Fraction(float(hv[0, i])) == _to_bf16_via_f32(exact)
    t = (torch.from_numpy(xv) + torch.from_numpy(rv)).to(torch.bfloat16).float().numpy()
    assert np.array_equal(hv, t)
    assert np.array_equal(oracle.add_bf16(R, X), H)  # commutative


# ---------------------------------------------------------------- ReLU
def test_relu_voids_negatives_and_passes_positives_unmodified():
    X = _bits([[1.5, -1.5, 0.0, -0.0, 2.0 ** -130, -(2.0 ** -130), 448.0, -(2.0 ** 127), 2.0 ** 127]])
    Y = oracle.relu_bf16(X)
    assert Y[0].tolist() == [X[0, 0], 0, 0, 0, X[0, 4], 0, X[0, 6], 0, X[0, 8]]
    Xr = inputs.make_x(inputs.CONFIGS["tiny"], 8)
    Yr = oracle.relu_bf16(Xr)
    assert np.array_equal(_vals(Yr), np.maximum(_vals(Xr), np.float32(0)))
    assert not np.any(Yr & 0x8000)  # no negative zero comes out
    assert np.array_equal(oracle.relu_bf16(Yr), Yr)  # idempotent


# ---------------------------------------------------------------- gated SiLU
def _exp_fraction(x, terms=120):
    s, t = Fraction(1), Fraction(1)
    for n in range(1, terms):
        t = t * x / n
        s += t
    return s


def test_swiglu_equals_exact_rational_evaluation_on_a_grid():
    gs = [0.5, -0.5, 1.0, -1.0, 2.0, -3.0, 0.0078125, 4.5, -6.0, 0.3125]
    us = [1.0, -1.5, 0.0078125, 3.0, -0.4375]
    G = _bits([[g for g in gs for _ in us]])
    U = _bits([[u for _ in gs for u in us]])
    Y = _vals(oracle.swiglu_bf16(G, U))[0]
    i = 0
    for g in gs:
        e = _exp_fraction(-Fraction(g))
        for u in us:
            exact = Fraction(g) / (1 + e) * Fraction(u)
            assert Fraction(float(Y[i])) == _to_bf16_via_f32(exact), (g, u)
            i += 1


def test_swiglu_closed_forms_and_limits():
    G = _bits([[0.0, 0.0, 64.0, 64.0, -200.0, 1.0, -1.0]])
    U = _bits([[3.0, -3.0, 1.5, -0.5, 2.0, 0.0, 1.0]])
    Yb = oracle.swiglu_bf16(G, U)
    Y = _vals(Yb)[0]
    assert Y[0] == 0 and Y[1] == 0          # silu(0) = 0
    assert Y[2] == 96.0 and Y[3] == -32.0   # silu(g) = g once exp(-g) is below half an ulp of 1
    assert Y[4] == 0                        # -200 / (1 + e^200) underflows
    assert Y[5] == 0
    # silu(1) - silu(-1) = 1:  silu(-1) = -1/(1+e) = -0.2689..., nearest bfloat16 is -0.26953125
    assert Y[6] == np.float32(-0.26953125)


def test_swiglu_agrees_with_the_tanh_form_from_another_library_routine():
    rng = np.random.default_rng(5)
    g = (3.0 * rng.standard_normal((16, 1024))).astype(np.float32)
    u = rng.standard_normal((16, 1024)).astype(np.float32)
    G, U = inputs.f32_to_bf16_bits(g), inputs.f32_to_bf16_bits(u)
    Y = oracle.swiglu_bf16(G, U)
    gv, uv = _vals(G).astype(np.float64), _vals(U).astype(np.float64)
    ref = (0.5 * gv * (1.0 + np.tanh(0.5 * gv)) * uv).astype(np.float32)  # silu(g) = g (1 + tanh(g/2)) / 2
    ref_bits = inputs.f32_to_bf16_bits(ref)
    diff = np.abs(Y.astype(np.int32) - ref_bits.astype(np.int32))
    assert diff.max() <= 1 and np.count_nonzero(diff) <= 4  # only a value within 1e-15 of a rounding boundary may differ
    t = (torch.nn.functional.silu(torch.from_numpy(gv)) * torch.from_numpy(uv)).float().to(torch.bfloat16).float().numpy()
    assert np.count_nonzero(t != _vals(Y)) <= 4
    # the gate is not symmetric: a sign error in the exponent would swap these
    assert _vals(oracle.swiglu_bf16(_bits([[2.0]]), _bits([[1.0]])))[0, 0] > 1.7
    assert abs(_vals(oracle.swiglu_bf16(_bits([[-2.0]]), _bits([[1.0]])))[0, 0]) < 0.25
