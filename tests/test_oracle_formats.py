"""Pins of the oracle's number formats and encoders against what the paper and
the mathematics fix (Section 2: ExMy formats; Section 3: FP4->FP8 by exponent
shift).  CPU only.  Independent references used here: PyTorch's float8 dtypes
(bit-cast decode and its own round-to-nearest-even conversion), hand-derived
fixtures under tests/golden/, and exact rational arithmetic."""
import math
import os
from fractions import Fraction

import numpy as np
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
E2M1_VALUES = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]  # fixed by the benchmark spec


def _golden(name):
    rows = []
    for line in open(os.path.join(GOLDEN, name)):
        line = line.split("#")[0].split()
        if line:
            rows.append(line)
    return rows


def _torch_decode(dtype):
    return torch.arange(256, dtype=torch.uint8).view(dtype).to(torch.float64).numpy()


# ---------------------------------------------------------------- E4M3 decode
def test_e4m3_decode_all_codes_match_torch_bitcast():
    ref = _torch_decode(torch.float8_e4m3fn)
    for c in range(256):
        v = oracle.e4m3_decode(c)
        if c in (0x7F, 0xFF):
            assert math.isnan(v) and math.isnan(ref[c])
        else:
            assert v == ref[c], (c, v, ref[c])


def test_e4m3_structure():
    vals = [oracle.e4m3_decode(c) for c in range(256)]
    finite = [v for v in vals if not math.isnan(v)]
    assert len(finite) == 254
    assert max(finite) == 448.0 == vals[0x7E] and min(finite) == -448.0
    assert vals[0x01] == 2.0 ** -9 and vals[0x08] == 2.0 ** -6
    pos = vals[0:0x7F]
    assert all(b > a for a, b in zip(pos, pos[1:]))  # strictly increasing
    assert all(vals[c | 0x80] == -vals[c] for c in range(0x7F))
    assert math.copysign(1.0, vals[0x80]) == -1.0 and vals[0x80] == 0.0


def test_e5m2_decode_all_codes_match_torch_bitcast():
    ref = _torch_decode(torch.float8_e5m2)
    for c in range(256):
        v = oracle.e5m2_decode(c)
        assert (math.isnan(v) and math.isnan(ref[c])) or v == ref[c], (c, v, ref[c])


# ---------------------------------------------------------------- E2M1 decode
def test_e2m1_value_set():
    for c in range(8):
        assert oracle.e2m1_decode(c) == E2M1_VALUES[c]
        assert oracle.e2m1_decode(c | 8) == -E2M1_VALUES[c]
    assert math.copysign(1.0, oracle.e2m1_decode(8)) == -1.0


# ---------------------------------------------------------------- E4M3 encode
def test_e4m3_encode_hand_cases():
    for val, code, *_ in _golden("e4m3_hand_cases.txt"):
        assert oracle.e4m3_encode(float(val)) == int(code, 16), (val, code)


def test_e4m3_encode_midpoints_and_neighbours():
    pos = [oracle.e4m3_decode(c) for c in range(0x7F)]
    for c in range(0x7E):
        lo, hi = pos[c], pos[c + 1]
        mid = np.float32((lo + hi) / 2)
        assert float(mid) == (lo + hi) / 2  # midpoints are binary32 numbers
        even = c if c % 2 == 0 else c + 1
        assert oracle.e4m3_encode(mid) == even
        assert oracle.e4m3_encode(np.nextafter(mid, np.float32(0))) == c
        assert oracle.e4m3_encode(np.nextafter(mid, np.float32(1e9))) == c + 1
        assert oracle.e4m3_encode(-mid) == even | 0x80
    for c in range(0x7F):  # representable values are fixed points
        assert oracle.e4m3_encode(pos[c]) == c


def test_e4m3_encode_saturation_and_sign():
    for y in (448.0, 449.0, 463.9, 464.0, 480.0, 1e6, 3e38):
        assert oracle.e4m3_encode(y) == 0x7E
        assert oracle.e4m3_encode(-y) == 0xFE
    assert oracle.e4m3_encode(-0.0) == 0x80
    assert oracle.e4m3_encode(-1e-30) == 0x80
    assert oracle.e4m3_encode(1e-30) == 0x00


def test_e4m3_encode_all_bf16_inputs_match_torch_conversion():
    """Library special case: PyTorch's own float32 -> float8_e4m3fn conversion
    (round to nearest even) on every bfloat16 input below the overflow boundary."""
    bits = np.arange(65536, dtype=np.uint32)
    vals = (bits << 16).view(np.float32)
    ok = np.isfinite(vals) & (np.abs(vals) < 464.0)
    ref = torch.from_numpy(vals[ok].copy()).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode(v) for v in vals[ok]], np.uint8)
    assert np.array_equal(got, ref)


def test_e4m3_encode_random_f32_match_torch_conversion():
    rng = np.random.default_rng(7)
    vals = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(100),
        (rng.standard_normal(20000) * 0.05).astype(np.float32),
        np.exp(rng.uniform(-12, 6.1, 20000)).astype(np.float32),
    ])
    vals = vals[np.abs(vals) < 464.0]
    ref = torch.from_numpy(vals).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode(v) for v in vals], np.uint8)
    assert np.array_equal(got, ref)


# ---------------------------------------------------------------- E2M1 encode
def test_e2m1_encode_hand_cases():
    for val, code, *_ in _golden("e2m1_hand_cases.txt"):
        assert oracle.e2m1_encode(float(val)) == int(code, 16), (val, code)


def test_e2m1_encode_is_nearest_on_all_bf16_in_range():
    """Brute force: for every bfloat16 y in [-8, 8] the chosen value is a nearest
    one (exact rational distance); on an exact tie the even code is chosen."""
    bits = np.arange(65536, dtype=np.uint32)
    vals = (bits << 16).view(np.float32)
    vals = vals[np.isfinite(vals) & (np.abs(vals) <= 8.0)]
    grid = [Fraction(v) for v in E2M1_VALUES]
    for y in vals:
        code = oracle.e2m1_encode(float(y))
        assert (code >> 3) == (1 if math.copysign(1.0, float(y)) < 0 else 0)
        a = abs(Fraction(float(y)))
        d = [abs(g - a) for g in grid]
        best = min(d)
        winners = [i for i, di in enumerate(d) if di == best]
        want = winners[0] if len(winners) == 1 else [i for i in winners if i % 2 == 0][0]
        assert (code & 7) == want, (float(y), code)


# ---------------------------------------------------------------- shift cast
def test_fp4_to_fp8_shift_is_exact_power_of_two_scaling():
    """For every E2M1 code and every exponent in the container's range, the FP8
    code obtained by integer exponent-field addition decodes (with PyTorch's
    decode) to exactly value * 2^n; outside the range the function refuses."""
    dec = {"e4m3": _torch_decode(torch.float8_e4m3fn), "e5m2": _torch_decode(torch.float8_e5m2)}
    rng_ok = {"e4m3": range(-5, 7), "e5m2": range(-13, 14)}
    for cont in ("e4m3", "e5m2"):
        for n in range(-40, 41):
            results = [oracle.fp4_to_fp8_shift(c, n, cont) for c in range(16)]
            nonzero = [results[c] for c in range(16) if c & 7]
            if n in rng_ok[cont]:
                assert all(r is not None for r in results), (cont, n)
                for c in range(16):
                    want = oracle.e2m1_decode(c) * 2.0 ** n
                    got = dec[cont][results[c]]
                    assert got == want and math.copysign(1, got) == math.copysign(1, want)
            else:
                assert any(r is None for r in nonzero), (cont, n)
            # zero never needs the exponent and always passes
            assert results[0] == 0x00 and results[8] == 0x80
