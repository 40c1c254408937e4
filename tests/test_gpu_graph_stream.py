"""The whole step (activation quantizer with the LoRC left factor, GEMM with the LoRC epilogue, K-split and
chunked-K reductions through a caller's workspace) on a side stream and inside a HIP graph: every call
enqueues kernels only, so a captured step replays to the bits of the eager step."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2307_09782_amd import inputs, zqfp
from _util import bf16_tensor, f16_tensor

pytestmark = pytest.mark.gpu
CFG = inputs.CONFIGS


def _case(name, M, K=None, N=None, rank=None):
    cfg = CFG[name]
    cfg = dataclasses.replace(cfg, K=K or cfg.K, N=N or cfg.N, rank=cfg.rank if rank is None else rank, seed=M)
    X = bf16_tensor(inputs.make_x(cfg, M))
    packed = zqfp.pack_weight_fp4(bf16_tensor(inputs.make_w(cfg)), cfg.G, cfg.mode)
    U = V = None
    if cfg.rank:
        Ub, Vb = inputs.make_uv(cfg)
        U, V = f16_tensor(Ub), f16_tensor(Vb)
    ws_bytes = zqfp.gemm_workspace_bytes(M, cfg.K, cfg.N)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    Y = torch.empty((M, cfg.N), dtype=torch.float32, device="cuda")

    def step(x):
        if cfg.rank:
            Xq, sx, T = zqfp.quantize_act_fp8(x, U)
            zqfp.w4a8_gemm_lorc(Xq, sx, packed, cfg.N, cfg.G, T, V, out=Y, workspace=ws)
        else:
            Xq, sx = zqfp.quantize_act_fp8(x)
            zqfp.w4a8_gemm(Xq, sx, packed, cfg.N, cfg.G, out=Y, workspace=ws)

    return X, Y, step, ws_bytes


CASES = [("llama70b_ffn_decode", 16, None, 2048, None),   # decode form with LoRC
         ("llama7b_qkv", 300, None, 1024, 0),              # tiled form
         ("llama7b_qkv", 64, 11008, 512, 8),               # tiled form with a K-split through the workspace
         ("llama7b_qkv", 12, 28672, 8192, 0)]              # decode form, K in chunks through the workspace


@pytest.mark.parametrize("name,M,K,N,rank", CASES)
def test_step_on_a_side_stream_matches_the_default_stream(name, M, K, N, rank):
    X, Y, step, _ = _case(name, M, K, N, rank)
    step(X)
    torch.cuda.synchronize()
    want = Y.clone()
    Y.zero_()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(X)
    side.synchronize()
    assert torch.equal(Y, want)


@pytest.mark.parametrize("name,M,K,N,rank", CASES)
def test_captured_step_replays_to_the_bits_of_the_eager_step(name, M, K, N, rank):
    X, Y, step, ws_bytes = _case(name, M, K, N, rank)
    if name == "llama7b_qkv" and M in (64, 12):
        assert ws_bytes > 0  # these cases are here for the workspace paths
    X2 = torch.flip(X, dims=[0]).contiguous()
    wants = []
    for x in (X, X2):
        step(x)
        torch.cuda.synchronize()
        wants.append(Y.clone())
    assert not torch.equal(wants[0], wants[1])
    xin = X.clone()
    step(xin)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(xin)
    # replays with the program's own eager work and synchronisations in between, alternating inputs
    for i in range(4):
        src, want = ((X, wants[0]), (X2, wants[1]))[i % 2]
        xin.copy_(src)
        Y.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, want), f"replay {i}"
        step(src)  # eager launch between replays
        torch.cuda.synchronize()
        assert torch.equal(Y, want)
