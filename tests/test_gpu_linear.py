"""zqfp_w4a8_linear: the whole layer from bfloat16 activations in one call.  For at most 16 tokens, K <= 4096 and
no LoRC the decode GEMM quantizes the tokens in its own prologue (one kernel): Y must equal the two-call sequence
bit for bit, the codes and scales it can write out must be the oracle's, and Y meets the GEMM tolerance against
the oracle.  Beyond those limits the call is the two-call sequence itself."""
import numpy as np
import pytest
import torch

import oracle
from paper_2307_09782_amd import inputs, zqfp
from _util import bf16_tensor, bits_equal_f32, check_gemm, f16_tensor

pytestmark = pytest.mark.gpu


def _np(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def _case(M, K, N, G, mode, seed=3, outliers=0.01):
    cfg = inputs.Config("lin", K, N, (M,), G, mode, outliers, 0, 20.0, 0, seed)
    return cfg, inputs.make_x(cfg, M), inputs.make_w(cfg)


@pytest.mark.parametrize("M,K,N,G,mode", [
    (16, 256, 256, 128, 1),      # the tiny configuration: one k-tile per wave, 6 of 8 waves idle
    (1, 256, 48, 64, 1),
    (5, 512, 1664, 128, 2),      # strips in pairs, column scales
    (9, 1024, 272, 128, 1),      # one k-tile per wave, ragged N
    (16, 2560, 176, 128, 1),     # 20 k-tiles: three per wave, the last four waves one fewer
    (7, 3072, 200, 256, 2),      # three per wave, groups of 256
    (16, 4096, 320, 128, 1),     # four per wave
    (3, 3968, 96, 32, 2),        # 31 k-tiles: the last wave one fewer; groups of 32
])
def test_fused_decode_equals_two_calls_and_oracle(M, K, N, G, mode):
    print(f"fused linear M={M} K={K} N={N} G={G} mode={mode}", flush=True)
    assert zqfp.linear_is_fused(M, K)
    cfg, X, W = _case(M, K, N, G, mode)
    Xd = bf16_tensor(X)
    packed = zqfp.pack_weight_fp4(bf16_tensor(W), G, mode)
    for accum in (zqfp.ACCUM_EXACT, zqfp.ACCUM_FAST):
        Y, Xq, sx = zqfp.w4a8_linear(Xd, packed, N, G, accum=accum, want_codes=True)
        Xq2, sx2 = zqfp.quantize_act_fp8(Xd)
        Y2 = zqfp.w4a8_gemm(Xq2, sx2, packed, N, G, accum=accum)
        assert np.array_equal(_np(Y).view(np.uint32), _np(Y2).view(np.uint32))
        Xq_o, sx_o = oracle.quantize_act(X)
        assert np.array_equal(_np(Xq), Xq_o) and bits_equal_f32(_np(sx), sx_o)
    # without the optional outputs, bfloat16 out
    Yb = zqfp.w4a8_linear(Xd, packed, N, G, out_dtype=torch.bfloat16)
    Yb2 = zqfp.w4a8_gemm(Xq2, sx2, packed, N, G, out_dtype=torch.bfloat16)
    assert torch.equal(Yb, Yb2)
    codes, exps, c, _ = oracle.pack_weight(W, G, mode)
    Y_o, Sabs = oracle.gemm(Xq_o, sx_o, codes, exps, c, G)
    check_gemm(_np(zqfp.w4a8_linear(Xd, packed, N, G)), Y_o, Sabs, f"fused M{M} K{K} N{N}")


def test_fused_decode_zero_tiny_and_strided_rows():
    M, K, N, G = 8, 1024, 128, 128
    cfg, X, W = _case(M, K, N, G, 1)
    x = inputs.bf16_bits_to_f32(X).copy()
    x[1] = 0.0
    x[2] = -0.0
    x[3] *= 2.0 ** -110        # below the 2^-96 threshold: scale 1, signed-zero codes
    x[4, 5] = 3.0e38           # a huge element
    x[5, :] = 0.0
    x[5, 77] = -1.0            # one-hot row
    X = inputs.f32_to_bf16_bits(x)
    wide = torch.zeros((M, K + 64), dtype=torch.bfloat16, device="cuda")
    wide[:, :K] = bf16_tensor(X)
    Xs = wide[:, :K]           # row stride K + 64
    packed = zqfp.pack_weight_fp4(bf16_tensor(W), G, 1)
    Y, Xq, sx = zqfp.w4a8_linear(Xs, packed, N, G, want_codes=True)
    Xq_o, sx_o = oracle.quantize_act(X)
    assert np.array_equal(_np(Xq), Xq_o) and bits_equal_f32(_np(sx), sx_o)
    codes, exps, c, _ = oracle.pack_weight(W, G, 1)
    Y_o, Sabs = oracle.gemm(Xq_o, sx_o, codes, exps, c, G)
    check_gemm(_np(Y), Y_o, Sabs + 1e-300, "fused, edge rows")
    assert np.all(_np(Y)[1] == 0) and np.all(_np(Y)[2] == 0) and np.all(_np(Y)[3] == 0)


@pytest.mark.parametrize("name,M", [("llama7b_qkv", 16), ("llama7b_qkv", 1), ("llama7b_ffn_up", 16), ("llama7b_attn_out", 4)])
def test_fused_decode_full_size(name, M):
    print(f"fused linear {name} M={M}", flush=True)
    cfg = inputs.CONFIGS[name]
    X, W = inputs.make_x(cfg, M), inputs.make_w(cfg)
    Xd = bf16_tensor(X)
    packed = zqfp.pack_weight_fp4(bf16_tensor(W), cfg.G, cfg.mode)
    Y, Xq, sx = zqfp.w4a8_linear(Xd, packed, cfg.N, cfg.G, want_codes=True)
    Xq2, sx2 = zqfp.quantize_act_fp8(Xd)
    Y2 = zqfp.w4a8_gemm(Xq2, sx2, packed, cfg.N, cfg.G)
    assert np.array_equal(_np(Y).view(np.uint32), _np(Y2).view(np.uint32))
    Xq_o, sx_o = oracle.quantize_act(X)
    assert np.array_equal(_np(Xq), Xq_o) and bits_equal_f32(_np(sx), sx_o)


@pytest.mark.parametrize("M,K,N,r", [(16, 8192, 256, 0), (40, 512, 200, 0), (8, 1024, 272, 8), (64, 2048, 200, 8)])
def test_beyond_the_fused_limits_the_call_is_the_two_call_sequence(M, K, N, r):
    cfg = inputs.Config("lin", K, N, (M,), 128, 1, 0.01, 0, 20.0, r, 5)
    X, W = inputs.make_x(cfg, M), inputs.make_w(cfg)
    Xd = bf16_tensor(X)
    packed = zqfp.pack_weight_fp4(bf16_tensor(W), 128, 1)
    assert not zqfp.linear_is_fused(M, K, r)
    if r:
        U, V = inputs.make_uv(cfg, rank=r)
        Ud, Vd = f16_tensor(U), f16_tensor(V)
        Y = zqfp.w4a8_linear(Xd, packed, N, 128, Ud, Vd)
        Xq, sx, T = zqfp.quantize_act_fp8(Xd, Ud)
        Y2 = zqfp.w4a8_gemm_lorc(Xq, sx, packed, N, 128, T, Vd)
    else:
        Y = zqfp.w4a8_linear(Xd, packed, N, 128)
        Xq, sx = zqfp.quantize_act_fp8(Xd)
        Y2 = zqfp.w4a8_gemm(Xq, sx, packed, N, 128)
    assert torch.equal(Y, Y2)


def test_fused_step_in_a_graph_replays_to_the_eager_bits():
    cfg = inputs.CONFIGS["llama7b_attn_out"]
    M = 16
    Xd = bf16_tensor(inputs.make_x(cfg, M))
    packed = zqfp.pack_weight_fp4(bf16_tensor(inputs.make_w(cfg)), cfg.G, cfg.mode)
    Y = torch.empty((M, cfg.N), device="cuda")
    eager = zqfp.w4a8_linear(Xd, packed, cfg.N, cfg.G).clone()
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        zqfp.w4a8_linear(Xd, packed, cfg.N, cfg.G, out=Y)
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        zqfp.w4a8_linear(Xd, packed, cfg.N, cfg.G, out=Y)
    for _ in range(3):
        Y.fill_(5.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, eager)
