"""zqfp_w4a8_gemm_lorc_static (the GEMM entry point that allocates nothing: partial results go through an array
inside the library's device image) against zqfp_w4a8_gemm_lorc with a caller's workspace, through the C ABI: the
same kernels, so the same bits; and against the oracle to the GEMM tolerance.  Two calls in a row share the
array, the second with a smaller input; then shapes that never touch it, and the refusal beyond its size."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2307_09782_amd import inputs, zqfp
from _util import bf16_tensor, check_gemm, f16_tensor, f32_tensor

pytestmark = pytest.mark.gpu


def _case(M, K, N, G, mode, r, seed):
    cfg = inputs.Config("static", K, N, (M,), G, mode, 0.01, 0, 20.0, r, seed)
    X, W = inputs.make_x(cfg, M), inputs.make_w(cfg)
    packed = zqfp.pack_weight_fp4(bf16_tensor(W), G, mode)
    T = V = None
    if r:
        U, Vb = inputs.make_uv(cfg, rank=r)
        Xq, sx, T = zqfp.quantize_act_fp8(bf16_tensor(X), f16_tensor(U))
        V = f16_tensor(Vb)
    else:
        Xq, sx = zqfp.quantize_act_fp8(bf16_tensor(X))
    return dict(M=M, K=K, N=N, G=G, mode=mode, r=r, X=X, W=W, packed=packed, Xq=Xq, sx=sx, T=T, V=V,
                U=U if r else None, Vb=Vb if r else None)


def _both(c, out_dtype=torch.float32):
    """(static entry point, workspace entry point) on the same inputs; outputs pre-filled with a sentinel."""
    ya = torch.full((c["M"], c["N"]), 7.0, dtype=out_dtype, device="cuda")
    yb = torch.full((c["M"], c["N"]), 9.0, dtype=out_dtype, device="cuda")
    zqfp.w4a8_gemm_lorc_static(c["Xq"], c["sx"], c["packed"], c["N"], c["G"], ya, c["T"], c["V"])
    if c["r"]:
        zqfp.w4a8_gemm_lorc(c["Xq"], c["sx"], c["packed"], c["N"], c["G"], c["T"], c["V"], out=yb)
    else:
        zqfp.w4a8_gemm(c["Xq"], c["sx"], c["packed"], c["N"], c["G"], out=yb)
    torch.cuda.synchronize()
    return ya.float().cpu().numpy(), yb.float().cpu().numpy()


def _oracle_check(c, Y, what):
    Xq_o, sx_o = oracle.quantize_act(c["X"])
    codes, exps, cs, _ = oracle.pack_weight(c["W"], c["G"], c["mode"])
    T_o = None
    if c["r"]:  # the GPU's own T went into the product: use it on the oracle side as well
        T_o = c["T"].cpu().numpy()
    Y_o, Sabs = oracle.gemm(Xq_o, sx_o, codes, exps, cs, c["G"], T=T_o, V=c["Vb"])
    check_gemm(Y, Y_o, Sabs, what)


def test_two_calls_in_a_row_share_the_array_second_one_smaller():
    print("static entry point: decode form in 4 chunks (M=16 K=28672 N=4096), then one tile split 4 ways (M=64 K=4096 N=128)",
          flush=True)
    big = _case(16, 28672, 4096, 128, 1, 8, 11)        # 224 k-tiles: 4 chunks of 56, 4 * 16 * 4096 floats of partials
    small = _case(64, 4096, 128, 128, 1, 8, 12)        # one 64 x 128 tile, K split 4 ways: 4 * 64 * 128 floats
    assert zqfp.gemm_workspace_bytes(16, 28672, 4096) > zqfp.gemm_workspace_bytes(64, 4096, 128) > 0
    a1, b1 = _both(big)
    a2, b2 = _both(small)
    assert np.array_equal(a1, b1) and np.array_equal(a2, b2)
    _oracle_check(big, a1, "static, chunked decode form")
    _oracle_check(small, a2, "static, K-split tile")
    # and the other way round, bfloat16 out, then the first shape again: stale partials of a larger call are never read
    a3, b3 = _both(small, torch.bfloat16)
    a4, b4 = _both(big)
    assert np.array_equal(a3, b3) and np.array_equal(a4, b4) and np.array_equal(a4, a1)


@pytest.mark.parametrize("M,K,N,G,mode,r", [(16, 256, 256, 128, 1, 0), (200, 1280, 400, 256, 2, 0), (33, 11008, 256, 128, 2, 0),
                                         (100, 3072, 136, 128, 1, 3)])
def test_static_equals_workspace_form(M, K, N, G, mode, r):
    print(f"static entry point: M={M} K={K} N={N} G={G} mode={mode} r={r}", flush=True)
    c = _case(M, K, N, G, mode, r, 13)
    a, b = _both(c)
    assert np.array_equal(a, b)
    _oracle_check(c, a, f"static M{M} K{K} N{N}")


def test_refuses_partials_beyond_the_array_without_touching_a_pointer():
    lib = zqfp.lib()
    M, K, N = 16, 128 * 4000, 16384          # 63 chunks x 16 x 16384 floats = 66 MB of partials
    assert lib.zqfp_gemm_workspace_bytes(M, K, N) > zqfp.STATIC_SCRATCH_BYTES
    rc = lib.zqfp_w4a8_gemm_lorc_static(None, None, M, K, None, N, 128 * 16, None, None, 0, None, N, 0, 0, None)
    assert rc == -6 and b"built-in scratch array" in lib.zqfp_last_hip_error()
    # at the limit the size check passes and the NULL pointers are what is refused
    assert lib.zqfp_w4a8_gemm_lorc_static(None, None, 64, 4096, None, 128, 128, None, None, 0, None, 128, 0, 0, None) == -1
