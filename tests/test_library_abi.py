"""CPU-side checks of the C-ABI library: it loads, exports every symbol the
header declares, and its argument checks reject bad calls before touching the
GPU.  No compute call is made here."""
import ctypes
import os
import re

import pytest

from paper_2307_09782_amd import zqfp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    syms = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        syms |= set(re.findall(r"\b(zqfp_\w+)\s*\(", text))
    return sorted(syms)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(zqfp.LIB_PATH):
        from paper_2307_09782_amd.build import build_lib
        build_lib()
    return zqfp.lib()


def test_header_declares_the_four_calls_of_the_boundary():
    syms = _declared_symbols()
    for name in ("zqfp_quantize_act_fp8", "zqfp_pack_weight_fp4", "zqfp_w4a8_gemm", "zqfp_w4a8_gemm_lorc"):
        assert name in syms


def test_library_exports_every_declared_symbol(lib):
    for name in _declared_symbols():
        assert hasattr(lib, name), name
    assert lib.zqfp_version() >= 100


def test_packed_size_and_shape_limits(lib):
    # codes K*N/2 + exponents K/G*N + column scales 4N, plus header and padding
    K, N, G = 4096, 12288, 128
    n = lib.zqfp_packed_weight_bytes(K, N, G)
    payload = K * N // 2 + (K // G) * N + 4 * N
    assert payload + 256 <= n <= payload + 256 + 3 * 256
    assert lib.zqfp_packed_weight_bytes(4096, 100, 128) > 0      # N need not be a multiple of 16
    assert lib.zqfp_packed_weight_bytes(4000, 128, 128) == 0     # K % 128
    assert lib.zqfp_packed_weight_bytes(4096, 128, 48) == 0      # G % 32
    assert lib.zqfp_packed_weight_bytes(4096, 128, 96) == 0      # K % G
    assert lib.zqfp_packed_weight_bytes(3200, 128, 320) > 0      # the paper's LLaMA-3b group size
    assert lib.zqfp_packed_weight_bytes(32768, 128, 32) == 0     # K / G > 256
    assert lib.zqfp_packed_weight_bytes(4096, 128, 256) > 0
    assert lib.zqfp_packed_weight_bytes(4096, 128, 32) > 0
    assert lib.zqfp_gemm_workspace_bytes(16, 4096, 4096) == 0


def test_argument_checks_return_error_codes_without_a_gpu(lib):
    p = ctypes.c_void_p
    buf = (ctypes.c_uint8 * 4096)()
    a = ctypes.addressof(buf)
    a16 = (a + 255) // 256 * 256
    # quantizer: K % 128, NULL pointers, alignment
    assert lib.zqfp_quantize_act_fp8(p(a16), 1, 100, 100, p(a16), p(a16), None, 0, None, None) == -2
    assert lib.zqfp_quantize_act_fp8(None, 1, 128, 128, p(a16), p(a16), None, 0, None, None) == -1
    assert lib.zqfp_quantize_act_fp8(p(a16 + 2), 1, 128, 128, p(a16), p(a16), None, 0, None, None) == -3
    assert lib.zqfp_quantize_act_fp8(p(a16), 1, 128, 128, p(a16), p(a16), None, 8, None, None) == -1
    assert lib.zqfp_quantize_act_fp8(p(a16), 0, 128, 128, p(a16), p(a16), None, 0, None, None) == 0
    # packer: mode, shape
    assert lib.zqfp_pack_weight_fp4(p(a16), 128, 16, 16, 128, 3, p(a16), None) == -4
    assert lib.zqfp_pack_weight_fp4(p(a16), 128, 16, 8, 128, 1, p(a16), None) == -2
    assert lib.zqfp_pack_weight_fp4(p(a16), 128, 16, 16, 128, 1, None, None) == -1
    assert lib.zqfp_pack_weight_fp4(p(a16), 128, 16, 16, 128, 1, p(a16 + 16), None) == -3
    # gemm: out dtype, rank, empty problem is a no-op
    assert lib.zqfp_w4a8_gemm(p(a16), p(a16), 1, 128, p(a16), 16, 128, p(a16), 16, 7, 0, None, 0, None) == -4
    assert lib.zqfp_w4a8_gemm(p(a16), p(a16), 1, 128, p(a16), 16, 128, p(a16), 16, 0, 5, None, 0, None) == -4
    assert lib.zqfp_w4a8_gemm(p(a16), p(a16), 0, 128, p(a16), 16, 128, p(a16), 16, 0, 0, None, 0, None) == 0
    assert lib.zqfp_w4a8_gemm(p(a16), p(a16), 1, 128, None, 16, 128, p(a16), 16, 0, 0, None, 0, None) == -1
    assert lib.zqfp_w4a8_gemm(p(a16), p(a16), 1, 128, p(a16), 16, 128, p(a16), 8, 0, 0, None, 0, None) == -2
    assert lib.zqfp_w4a8_gemm_lorc(p(a16), p(a16), 1, 128, p(a16), 16, 128, None, None, 8, p(a16), 16, 0, 0, None, 0, None) == -1
    assert lib.zqfp_w4a8_gemm_lorc(p(a16), p(a16), 1, 128, p(a16), 16, 128, p(a16), p(a16), 65, p(a16), 16, 0, 0, None, 0, None) == -2
    # a workspace that is given must be as large as the query says (here: one 64 x 128 tile, K split 4 ways)
    need = lib.zqfp_gemm_workspace_bytes(64, 4096, 128)
    assert need > 0
    assert lib.zqfp_w4a8_gemm(p(a16), p(a16), 64, 4096, p(a16), 128, 128, p(a16), 128, 0, 0, p(a16), need - 1, None) == -6
    assert b"workspace" in lib.zqfp_last_hip_error()
    assert lib.zqfp_w4a8_gemm(p(a16), p(a16), 16, 28672, p(a16), 8192, 128, p(a16), 8192, 0, 0, p(a16), 1 << 20, None) == -6
    # shape limits of the layout itself
    assert lib.zqfp_packed_weight_bytes(128 * 4096, 16, 128 * 16) == 0   # 4096 k-tiles: beyond the limit
    assert lib.zqfp_packed_weight_bytes(128 * 4095, 16, 128 * 21) > 0


def test_packed_weight_check_reads_a_host_copy_of_the_header(lib):
    """Header fields as the packer writes them (magic 'ZQF4', version, K, N, Np, G, Gs, mode, ngs, ngq, code width,
    four section offsets): accepted for its own (K, N, G), refused for any other and after any damage."""
    import struct
    K, N, G = 512, 200, 64
    total = lib.zqfp_packed_weight_bytes(K, N, G)
    Np = 208
    off_codes = 256
    off_exps = off_codes + Np * K // 2
    ngs = K // 64
    ngq = (ngs + 3) // 4
    off_cs = (off_exps + (Np // 16) * ngq * 64 + 255) // 256 * 256
    assert total == (off_cs + 4 * Np + 255) // 256 * 256
    hdr = struct.pack("<IIqqqiiiiiIQQQQ", 0x3446515A, 1, K, N, Np, G, 64, 2, ngs, ngq, 4, off_codes, off_exps, off_cs, total)
    hdr = hdr + bytes(256 - len(hdr))
    chk = lambda h, k, n, g: lib.zqfp_packed_weight_check(h, k, n, g)
    assert chk(hdr, K, N, G) == 0
    assert chk(hdr, K, N, 128) == -7 and chk(hdr, K, N + 1, G) == -7 and chk(hdr, 2 * K, N, G) == -7
    assert chk(hdr, K, N, 48) == -2 and chk(None, K, N, G) == -1
    assert chk(b"\0" * 256, K, N, G) == -7
    for pos in (0, 4, 8, 16, 32, 40, 52, 56, 80):
        bad = bytearray(hdr)
        bad[pos] ^= 1
        assert chk(bytes(bad), K, N, G) == -7, pos


def test_binding_refuses_sizes_the_library_must_take_on_trust():
    """The wrappers compare what the C side cannot (it never reads device memory on the host): blob size against
    (K, N, G), workspace size against the query, the output's shape, dtype and row contiguity."""
    import torch
    K, N, G, M = 4096, 128, 128, 64
    nb = zqfp.packed_weight_bytes(K, N, G)
    ok = dict(M=M, K=K, N=N, G=G, packed_numel=nb, workspace_numel=None, out_shape=(M, N), out_dtype=torch.float32,
              out_stride=(N, 1))
    zqfp.check_gemm_args(**ok)
    zqfp.check_gemm_args(**{**ok, "workspace_numel": zqfp.gemm_workspace_bytes(M, K, N)})
    zqfp.check_gemm_args(**{**ok, "out_stride": (N + 8, 1), "out_dtype": torch.bfloat16})
    for change, code in (({"packed_numel": nb - 256}, -2), ({"G": 256}, -2), ({"N": 144}, -2), ({"G": 48}, -2),
                         ({"workspace_numel": zqfp.gemm_workspace_bytes(M, K, N) - 4}, -6),
                         ({"out_dtype": torch.float16}, -4), ({"out_shape": (M, N + 1)}, -2),
                         ({"out_stride": (N, 2)}, -2), ({"out_stride": (N - 1, 1)}, -2), ({"out_is_cuda": False}, -2)):
        with pytest.raises(zqfp.ZqfpError) as e:
            zqfp.check_gemm_args(**{**ok, **change})
        assert e.value.code == code, change


def test_build_rejects_spills_in_hand_scheduled_kernels():
    """The tiled GEMM waits for its LDS reads by count; the build refuses a compile in which that
    kernel uses scratch memory (a spill could save a register whose read is still in flight)."""
    from paper_2307_09782_amd import build
    ok = ("x.hip:1:1: remark: Function Name: _ZN4zqfp11k_gemm_tileILi4EEEv [-Rpass-analysis=kernel-resource-usage]\n"
          "x.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n"
          "x.hip:1:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]\n"
          "x.hip:1:1: remark: Function Name: _ZN4zqfp13k_gemm_decodeILi8EEEv [-Rpass-analysis=kernel-resource-usage]\n"
          "x.hip:1:1: remark:     ScratchSize [bytes/lane]: 96 [-Rpass-analysis=kernel-resource-usage]\n")
    build._check_no_scratch(ok)  # other kernels may use scratch
    bad = ok.replace("ScratchSize [bytes/lane]: 0", "ScratchSize [bytes/lane]: 24")
    with pytest.raises(RuntimeError):
        build._check_no_scratch(bad)


def test_workspace_query_is_pure_host_logic():
    """zqfp_gemm_workspace_bytes plans on the host (no GPU needed): zero for every benchmark
    configuration, [slices][M][Np] floats where K is split."""
    lib = zqfp.lib()
    ws = lambda M, K, N: int(lib.zqfp_gemm_workspace_bytes(M, K, N))
    for (M, K, N) in [(16, 256, 256), (2048, 2048, 8192), (1, 4096, 12288), (16, 4096, 12288), (256, 4096, 12288),
                      (4096, 4096, 12288), (4096, 4096, 11008), (16, 5120, 13824), (2048, 5120, 13824),
                      (1, 8192, 28672), (4, 8192, 28672), (16, 8192, 28672), (64, 8192, 28672)]:
        assert ws(M, K, N) == 0, (M, K, N)
    assert ws(64, 4096, 128) == 4 * 64 * 128 * 4          # one tile, 32 k-tiles: 4 slices of 8
    assert ws(64, 11008, 4096) == 10 * 64 * 4096 * 4      # 32 tiles, 86 k-tiles: 10 slices of 9
    assert ws(100, 3072, 136) == 3 * 100 * 144 * 4        # Np = 144
    assert ws(16, 28672, 8192) == 4 * 16 * 8192 * 4       # decode form: 224 k-tiles in 4 chunks
    assert ws(8, 8192, 4096) == 0 and ws(0, 4096, 4096) == 0 and ws(64, 4100, 4096) == 0


def test_bench_refuses_more_than_one_gpu():
    """The build runs on one GPU: `bench.py --gpus 2` exits with a message before it touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
