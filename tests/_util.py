"""Shared helpers of the GPU parity tests: numpy bit patterns <-> torch tensors
and the tolerance check.  No arithmetic of the method lives here."""
import numpy as np
import torch


def bf16_tensor(bits, device="cuda"):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)


def f16_tensor(bits, device="cuda"):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.float16).to(device)


def u8_tensor(a, device="cuda"):
    return torch.from_numpy(np.ascontiguousarray(a, np.uint8)).to(device)


def f32_tensor(a, device="cuda"):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(device)


def bits_equal_f32(a, b):
    return np.array_equal(np.ascontiguousarray(a, np.float32).view(np.uint32),
                          np.ascontiguousarray(b, np.float32).view(np.uint32))


# tolerance of the benchmark spec for GEMM outputs
REL_FRO = 1e-5
ELEM = 2.0 ** -18


def check_gemm(got, want, sabs, what=""):
    """got, want float arrays; sabs = sum of absolute terms per output (float64)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    err = np.abs(got - want)
    fro = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    ratio = (err / np.maximum(sabs, 1e-300)).max() if err.size else 0.0
    assert fro <= REL_FRO, f"{what}: relative Frobenius error {fro:.3e} > {REL_FRO}"
    assert ratio <= ELEM, f"{what}: max |err| / sum|a w| = {ratio:.3e} > 2^-18 = {ELEM:.3e}"
    return fro, ratio
