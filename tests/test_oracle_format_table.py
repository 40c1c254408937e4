"""Pins of the value-table quantizer behind the format ablation (oracle.quantize_to_format): it must agree with the
separately pinned scalar encoders for E2M1 and E4M3, with another library's conversion for E5M2, and with
hand-derived cases for E3M0; and the committed table must be what the script prints."""
import io
import os
from contextlib import redirect_stdout

import numpy as np
import torch

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _points(tab):
    mids = (tab[:-1] + tab[1:]) / 2
    pts = np.concatenate([tab, mids, mids * (1 + 1e-9), mids * (1 - 1e-9), [tab[-1] * 1.5, tab[-1] * 100, 1e-12]])
    return np.concatenate([pts, -pts, [0.0, -0.0]])


def test_agrees_with_the_scalar_encoders():
    rng = np.random.default_rng(0)
    y = np.concatenate([_points(oracle.format_values("e2m1")), rng.standard_normal(2000) * 3])
    want = np.array([oracle.e2m1_decode(oracle.e2m1_encode(float(v))) for v in y])
    assert np.array_equal(oracle.quantize_to_format(y, "e2m1"), want)
    y = np.concatenate([_points(oracle.format_values("e4m3")), rng.standard_normal(4000) * 100]).astype(np.float32)
    want = np.array([oracle.e4m3_decode(oracle.e4m3_encode(float(v))) for v in y])
    assert np.array_equal(oracle.quantize_to_format(y.astype(np.float64), "e4m3"), want)


def test_e5m2_agrees_with_another_librarys_conversion():
    rng = np.random.default_rng(1)
    tab = oracle.format_values("e5m2")
    assert tab[-1] == 57344.0 and tab[1] == 2.0 ** -16 and len(tab) == 0x7C
    y = np.concatenate([_points(tab)[: -2 * 3 - 2], rng.standard_normal(4000) * 1000]).astype(np.float32)
    y = y[np.abs(y) <= 57344.0]                      # torch does not saturate; in range it rounds to nearest even
    want = torch.from_numpy(y).to(torch.float8_e5m2).float().numpy().astype(np.float64)
    assert np.array_equal(oracle.quantize_to_format(y.astype(np.float64), "e5m2"), want)
    assert oracle.quantize_to_format(np.array([1e9, -1e9]), "e5m2").tolist() == [57344.0, -57344.0]


def test_e3m0_hand_cases():
    tab = oracle.format_values("e3m0")
    assert tab.tolist() == [0.0, 0.25, 0.5, 1.0, 2.0, 4.0, 8.0, 16.0]
    # midpoints go to the even magnitude code: 0.125 -> 0 (code 0), 0.375 -> 0.5 (code 2), 0.75 -> 0.5, 1.5 -> 2 (code 4),
    # 3 -> 2, 6 -> 8 (code 6), 12 -> 8; beyond 16 saturates; the sign is kept
    y = np.array([0.125, 0.375, 0.75, 1.5, 3.0, 6.0, 12.0, 20.0, -1.4, -1.6, 0.3, 0.1])
    want = [0.0, 0.5, 0.5, 2.0, 2.0, 8.0, 8.0, 16.0, -1.0, -2.0, 0.25, 0.0]
    assert oracle.quantize_to_format(y, "e3m0").tolist() == want


def test_committed_table_is_what_the_script_prints():
    from oracle import format_table
    buf = io.StringIO()
    with redirect_stdout(buf):
        format_table.main()
    assert buf.getvalue() == open(os.path.join(ROOT, "oracle", "format_table.txt")).read()
