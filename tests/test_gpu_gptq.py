"""GPTQ on the E2M1 grid (Section 3, Appendix A) on the GPU against the oracle.  With an identity Hessian the
result has one right answer (the plain packer's blob, bit for bit).  With feedback the kernel works in binary32
and the oracle in float64, so a code can differ where an updated weight sits within rounding error of a grid
midpoint, and each such difference perturbs the channels behind it: the tests compare the share of identical
codes, the objective tr((W - Q)^T H (W - Q)) that the algorithm reduces, and the validity of the result."""
import numpy as np
import pytest
import torch

import oracle
from paper_2307_09782_amd import inputs, zqfp
from _util import bf16_tensor

pytestmark = pytest.mark.gpu


def _w(K, N, seed):
    cfg = inputs.Config("g", K, N, (1,), 128, 1, 0.0, 4, 20.0, 0, seed)
    return inputs.make_w(cfg)


def _hessian(K, seed):
    """Covariance of strongly correlated input channels, its samples, and the upper Cholesky factor of its inverse."""
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((K, 4 * K)) + 2.0 * rng.standard_normal((1, 4 * K))
    H = A @ A.T / (4 * K) + 0.01 * np.eye(K)
    return H, A, np.ascontiguousarray(np.linalg.cholesky(np.linalg.inv(H)).T)


def _unpacked(packed, K, N, G):
    codes, exps, c = zqfp.unpack_codes(packed, K, N, G)
    torch.cuda.synchronize()
    return codes.cpu().numpy(), exps.cpu().numpy(), c.cpu().numpy()


@pytest.mark.parametrize("K,N,G,mode", [(256, 256, 128, 1), (256, 256, 32, 1), (512, 200, 64, 2), (512, 96, 256, 2),
                                        (768, 40, 256, 1), (128, 17, 128, 2)])
def test_identity_hessian_gives_the_plain_packers_blob_bit_for_bit(K, N, G, mode):
    W = _w(K, N, K + N)
    Wd = bf16_tensor(W)
    eye = torch.eye(K, dtype=torch.float32, device="cuda")
    got = zqfp.gptq_pack_weight_fp4(Wd, eye, G, mode)
    want = zqfp.pack_weight_fp4(Wd, G, mode)
    torch.cuda.synchronize()
    # header, then every section the GEMM reads (the alignment gaps between sections are nobody's)
    g, w = got.cpu().numpy(), want.cpu().numpy()
    assert np.array_equal(g[:88], w[:88])
    off_codes, off_exps, off_cs, total = (int(v) for v in w[56:88].view(np.uint64))
    Np = (N + 15) // 16 * 16
    assert np.array_equal(g[off_codes:off_codes + Np * K // 2], w[off_codes:off_codes + Np * K // 2])
    ngq = int(w[48:52].view(np.int32)[0])
    assert np.array_equal(g[off_exps:off_exps + Np // 16 * ngq * 64], w[off_exps:off_exps + Np // 16 * ngq * 64])
    assert np.array_equal(g[off_cs:off_cs + 4 * Np], w[off_cs:off_cs + 4 * Np])
    for a, b in zip(_unpacked(got, K, N, G), _unpacked(want, K, N, G)):
        assert np.array_equal(a, b)
    # and against the oracle itself: its plain packer, and its GPTQ under the same identity Hessian
    codes_o, exps_o, c_o, _ = oracle.pack_weight(W, G, mode)
    for a, b in zip(_unpacked(got, K, N, G), (codes_o, exps_o, c_o)):
        assert np.array_equal(a, b)
    codes_g, exps_g, c_g, _ = oracle.gptq_fp4(W, np.eye(K), G, mode)
    for a, b in zip(_unpacked(got, K, N, G), (codes_g, exps_g, c_g)):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("K,N,G,mode", [(256, 64, 128, 1), (512, 200, 64, 2), (512, 96, 256, 1), (1024, 130, 128, 2)])
def test_error_feedback_against_the_oracle(K, N, G, mode):
    W = _w(K, N, 3 * K + N)
    H, _, U = _hessian(K, K)
    packed = zqfp.gptq_pack_weight_fp4(bf16_tensor(W), torch.from_numpy(U.astype(np.float32)).cuda(), G, mode)
    codes, exps, c = _unpacked(packed, K, N, G)
    codes_o, exps_o, c_o, Q_o = oracle.gptq_fp4(W, U, G, mode)
    Wf = inputs.bf16_bits_to_f32(W).astype(np.float64)
    Q = oracle.dequant_weight(codes, exps, c, G)
    obj = np.trace((Wf - Q).T @ H @ (Wf - Q))
    obj_o = np.trace((Wf - Q_o).T @ H @ (Wf - Q_o))
    cp, ep, ccp, _ = oracle.pack_weight(W, G, mode)
    Qr = oracle.dequant_weight(cp, ep, ccp, G)
    obj_rtn = np.trace((Wf - Qr).T @ H @ (Wf - Qr))
    same = np.mean(codes == codes_o)
    print(f"identical codes {same:.4f}, exponents {np.mean(exps == exps_o):.4f}; objective {obj:.5e} oracle {obj_o:.5e} "
          f"round-to-nearest {obj_rtn:.5e}")
    assert np.array_equal(c, c_o)                       # column scales come from the original W: one right answer
    assert same >= 0.995 and np.mean(exps == exps_o) >= 0.995
    assert abs(obj - obj_o) <= 0.02 * obj_o
    assert obj < 0.8 * obj_rtn
    assert codes.max() <= 15 and exps.min() >= 1 and exps.max() <= 254
    # the first input channel of every output channel sees no feedback: identical to the oracle's
    assert np.array_equal(codes[0], codes_o[0]) and np.array_equal(exps[0], exps_o[0])


def test_blob_from_gptq_serves_the_gemm_and_lowers_the_layer_output_error():
    K, N, G, M = 512, 256, 128, 64
    W = _w(K, N, 5)
    H, A, U = _hessian(K, 9)
    X = inputs.f32_to_bf16_bits(A[:, :M].T.astype(np.float32))  # tokens drawn from the distribution H describes
    Wd, Xd = bf16_tensor(W), bf16_tensor(X)
    Xq, sx = zqfp.quantize_act_fp8(Xd)
    ref = inputs.bf16_bits_to_f32(X).astype(np.float64) @ inputs.bf16_bits_to_f32(W).astype(np.float64)
    errs = []
    for packed in (zqfp.gptq_pack_weight_fp4(Wd, torch.from_numpy(U.astype(np.float32)).cuda(), G, 1),
                   zqfp.pack_weight_fp4(Wd, G, 1)):
        Y = zqfp.w4a8_gemm(Xq, sx, packed, N, G).double().cpu().numpy()
        errs.append(np.linalg.norm(Y - ref))
    print(f"layer output error: GPTQ {errs[0]:.4f}, round-to-nearest {errs[1]:.4f}")
    assert errs[0] < 0.9 * errs[1]


def test_argument_checks():
    W = bf16_tensor(_w(256, 64, 1))
    eye = torch.eye(256, dtype=torch.float32, device="cuda")
    with pytest.raises(zqfp.ZqfpError):
        zqfp.gptq_pack_weight_fp4(W, eye, 96, 1)       # group size outside the supported set
    with pytest.raises(zqfp.ZqfpError):
        zqfp.gptq_pack_weight_fp4(W, eye[:128, :128].contiguous(), 128, 1)
    assert zqfp.lib().zqfp_gptq_workspace_bytes(256, 64, 96) == 0
