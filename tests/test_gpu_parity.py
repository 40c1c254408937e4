"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the
same seeded inputs.  Quantized codes, token scales, exponent bytes and column
scales must be bit-exact; GEMM outputs must meet the relative-Frobenius and
the elementwise |err| <= 2^-18 * sum|a w| bounds."""
import numpy as np
import pytest
import torch

import oracle
from paper_2307_09782_amd import inputs, zqfp
from _util import ELEM, bf16_tensor, bits_equal_f32, check_gemm, f16_tensor, f32_tensor, u8_tensor

pytestmark = pytest.mark.gpu

CFG = inputs.CONFIGS


def _sync_np(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


# ------------------------------------------------------------------ quantizer
@pytest.mark.parametrize("name,M", [("tiny", 16), ("opt1p3b_fc1", 300), ("llama7b_qkv", 1), ("llama7b_qkv", 77),
                                    ("llama13b_ffn_lorc", 16), ("llama70b_ffn_decode", 64),
                                    # the wave-per-token kernel, with a ragged last workgroup
                                    ("opt1p3b_fc1", 1027), ("llama7b_qkv", 1100), ("llama70b_ffn_decode", 1025)])
def test_quantizer_codes_and_scales_bit_exact(name, M):
    cfg = CFG[name]
    X = inputs.make_x(cfg, M)
    Xq_o, sx_o = oracle.quantize_act(X)
    Xq, sx = zqfp.quantize_act_fp8(bf16_tensor(X))
    assert np.array_equal(_sync_np(Xq), Xq_o)
    assert bits_equal_f32(_sync_np(sx), sx_o)


def test_quantizer_full_size_sampled_rows():
    """Full-size launch (4096 x 4096); the oracle checks a sample of whole rows."""
    cfg = CFG["llama7b_qkv"]
    X = inputs.make_x(cfg, 4096)
    Xq, sx = zqfp.quantize_act_fp8(bf16_tensor(X))
    rows = np.random.default_rng(0).choice(4096, 96, replace=False)
    rows = np.concatenate([rows, [0, 4095]])
    Xq_o, sx_o = oracle.quantize_act(np.ascontiguousarray(X[rows]))
    assert np.array_equal(_sync_np(Xq)[rows], Xq_o)
    assert bits_equal_f32(_sync_np(sx)[rows], sx_o)


def test_quantizer_edge_rows_and_long_rows():
    """Zero rows, signed zeros, vanishing rows, exact ties, a row longer than the
    register-resident limit, and a strided input."""
    rng = np.random.default_rng(2)
    K = 128 * 80  # 10240 > 8192
    x = rng.standard_normal((6, K)).astype(np.float32)
    x[0] = 0.0
    x[1] = 0.0; x[1, 5] = -0.0
    x[2] = 2.0 ** -100; x[2, 9] = -(2.0 ** -100)
    x[3, :] = np.resize(np.array([448, 42, -42, 1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -11, -0.0, 432], np.float32), K)
    x[4, 17] = 3e38
    X = inputs.f32_to_bf16_bits(x)
    Xq_o, sx_o = oracle.quantize_act(X)
    big = torch.zeros((6, K + 64), dtype=torch.bfloat16, device="cuda")
    big[:, :K] = bf16_tensor(X)
    Xs = big[:, :K]  # row stride K + 64
    Xq = torch.empty((6, K), dtype=torch.uint8, device="cuda")
    sx = torch.empty((6,), dtype=torch.float32, device="cuda")
    rc = zqfp.lib().zqfp_quantize_act_fp8(Xs.data_ptr(), 6, K, Xs.stride(0), Xq.data_ptr(), sx.data_ptr(), None, 0, None,
                                          torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    assert np.array_equal(_sync_np(Xq), Xq_o)
    assert bits_equal_f32(_sync_np(sx), sx_o)


@pytest.mark.parametrize("name,M,r", [("tiny", 16, 8), ("llama13b_ffn_lorc", 16, 8), ("llama70b_ffn_decode", 4, 8),
                                      ("tiny", 5, 3), ("tiny", 7, 16), ("tiny", 3, 40),
                                      # many tokens: the wave-per-token kernel carries the rank-8 factor (K = 256 ... 8192);
                                      # other ranks stay with the workgroup-per-token kernel
                                      ("llama13b_ffn_lorc", 1100, 8), ("llama70b_ffn_decode", 1030, 8), ("tiny", 1025, 8),
                                      ("opt1p3b_fc1", 1024, 8), ("llama7b_qkv", 1027, 16), ("llama7b_qkv", 1500, 5)])
def test_lorc_left_factor(name, M, r):
    cfg = CFG[name]
    X = inputs.make_x(cfg, M)
    U, _ = inputs.make_uv(cfg, rank=r)
    T_o, Tabs = oracle.lorc_left(X, U)
    Xq_o, sx_o = oracle.quantize_act(X)
    Xq, sx, T = zqfp.quantize_act_fp8(bf16_tensor(X), f16_tensor(U))
    assert np.array_equal(_sync_np(Xq), Xq_o) and bits_equal_f32(_sync_np(sx), sx_o)
    err = np.abs(_sync_np(T).astype(np.float64) - T_o)
    assert (err / Tabs).max() <= 2.0 ** -18


@pytest.mark.parametrize("K,M", [(2688, 1029), (640, 1024), (5632, 1031), (6400, 1025), (640, 2100), (2688, 2056)])
def test_lorc_left_factor_many_tokens_rows_that_end_inside_a_chunk(K, M):
    """The wave-per-token kernel walks a row in chunks of 512 elements and stages all of U in LDS in the same chunks: here the
    row ends inside a chunk (K is a multiple of 128, not of 512), the token count leaves the last workgroup partly
    empty, and K picks each of the chunk counts the launcher has.  Up to 2048 tokens and 5120 elements a helper wave per
    token multiplies the second half of the row; the last two cases have more tokens than that form takes."""
    cfg = inputs.Config("q", K, 256, (M,), 128, 1, 0.01, 0, 20.0, 8, 11)
    X = inputs.make_x(cfg, M)
    U, _ = inputs.make_uv(cfg, rank=8)
    T_o, Tabs = oracle.lorc_left(X, U)
    Xq_o, sx_o = oracle.quantize_act(X)
    Xq, sx, T = zqfp.quantize_act_fp8(bf16_tensor(X), f16_tensor(U))
    assert np.array_equal(_sync_np(Xq), Xq_o) and bits_equal_f32(_sync_np(sx), sx_o)
    err = np.abs(_sync_np(T).astype(np.float64) - T_o)
    assert (err / Tabs).max() <= 2.0 ** -18


# ------------------------------------------------------------------ packer
def _pack_and_compare(W, G, mode, cols=None):
    K, N = W.shape
    packed = zqfp.pack_weight_fp4(bf16_tensor(W), G, mode)
    codes, exps, c = zqfp.unpack_codes(packed, K, N, G)
    codes, exps, c = _sync_np(codes), _sync_np(exps), _sync_np(c)
    if cols is None:
        codes_o, exps_o, c_o, _ = oracle.pack_weight(W, G, mode)
        assert np.array_equal(codes, codes_o) and np.array_equal(exps, exps_o) and bits_equal_f32(c, c_o)
    else:
        codes_o, exps_o, c_o, _ = oracle.pack_weight(np.ascontiguousarray(W[:, cols]), G, mode)
        assert np.array_equal(codes[:, cols], codes_o) and np.array_equal(exps[:, cols], exps_o)
        assert bits_equal_f32(c[cols], c_o)
    return packed


@pytest.mark.parametrize("G,mode", [(128, 1), (128, 2), (32, 1), (32, 2), (64, 1), (256, 2)])
def test_packer_tiny_bit_exact(G, mode):
    _pack_and_compare(inputs.make_w(CFG["tiny"]), G, mode)


@pytest.mark.parametrize("K,N,G,mode", [(384, 200, 384, 1), (640, 37, 320, 2), (384, 16, 96, 1), (256, 1, 128, 2)])
def test_packer_ragged_shapes_bit_exact(K, N, G, mode):
    W = inputs.make_w(CFG["tiny"], K=K, N=N)
    w = inputs.bf16_bits_to_f32(W).copy()
    w[: G, 0] = 0.0                      # a zero group
    w[3, -1] = 0.75; w[5, -1] = -0.375   # exact ties after scaling
    if N > 20:
        w[:, 20] *= 2.0 ** -120          # vanishing column
        w[:, 19] *= 2.0 ** 100
    _pack_and_compare(inputs.f32_to_bf16_bits(w), G, mode)


@pytest.mark.parametrize("name", ["opt1p3b_fc1", "llama7b_ffn_up", "llama70b_ffn_decode"])
def test_packer_full_size_sampled_columns(name):
    cfg = CFG[name]
    W = inputs.make_w(cfg)
    rng = np.random.default_rng(1)
    cols = np.sort(np.concatenate([rng.choice(cfg.N, 510, replace=False), [0, cfg.N - 1]]))
    cols = np.unique(cols)
    _pack_and_compare(W, cfg.G, cfg.mode, cols)


# ------------------------------------------------------------------ GEMM
_W_CACHE = {}


def _weights(cfg, G, mode):
    """W bits and the GPU-packed blob; the last configuration is kept so that
    the full-size cases of one layer do not regenerate and repack it."""
    key = (cfg.name, cfg.K, cfg.N, G, mode, cfg.seed)
    if key not in _W_CACHE:
        _W_CACHE.clear()
        W = inputs.make_w(cfg)
        _W_CACHE[key] = (W, zqfp.pack_weight_fp4(bf16_tensor(W), G, mode))
    return _W_CACHE[key]


def _gemm_case(M, K, N, G, mode, r=0, seed_cfg="tiny", full=True, nsamples=4096, out_dtype=torch.float32,
               x_override=None):
    cfg = CFG[seed_cfg]
    cfg = inputs.Config(cfg.name, K, N, (M,), G, mode, cfg.outlier_frac, cfg.outlier_count, cfg.outlier_gain, r, cfg.seed)
    X = inputs.make_x(cfg, M) if x_override is None else x_override
    W, packed = _weights(cfg, G, mode)
    Xq_o, sx_o = oracle.quantize_act(X)
    T = V = T_o = Vb = None
    if r:
        U, Vb = inputs.make_uv(cfg, rank=r)
        T_o, _ = oracle.lorc_left(X, U)
        Xq, sx, _T = zqfp.quantize_act_fp8(bf16_tensor(X), f16_tensor(U))
        # the GEMM check is fed the oracle's T so that it does not depend on the T check
        T, V = f32_tensor(T_o), f16_tensor(Vb)
    else:
        Xq, sx = zqfp.quantize_act_fp8(bf16_tensor(X))
    assert np.array_equal(_sync_np(Xq), Xq_o) and bits_equal_f32(_sync_np(sx), sx_o)
    if r:
        Y = zqfp.w4a8_gemm_lorc(Xq, sx, packed, N, G, T, V, out_dtype=out_dtype)
    else:
        Y = zqfp.w4a8_gemm(Xq, sx, packed, N, G, out_dtype=out_dtype)
    Y = _sync_np(Y.float())
    # oracle side: its own packing of the same W (bit-identical to the GPU's, checked by the packer tests)
    if full:
        codes_o, exps_o, c_o, _ = oracle.pack_weight(W, G, mode)
        Y_o, Sabs = oracle.gemm(Xq_o, sx_o, codes_o, exps_o, c_o, G, T=T_o, V=Vb)
        return Y, Y_o, Sabs
    rng = np.random.default_rng(5)
    ms = rng.integers(0, M, nsamples)
    ns = rng.integers(0, N, nsamples)
    ms[:4] = [0, M - 1, 0, M - 1]
    ns[:4] = [0, N - 1, N - 1, 0]
    cols = np.unique(ns)
    codes_s, exps_s, c_s, _ = oracle.pack_weight(np.ascontiguousarray(W[:, cols]), G, mode)
    ns_local = np.searchsorted(cols, ns)
    Vs = None if Vb is None else np.ascontiguousarray(Vb[:, cols])
    Y_o, Sabs = oracle.gemm_samples(Xq_o, sx_o, codes_s, exps_s, c_s, G, ms, ns_local, T=T_o, V=Vs)
    return Y[ms, ns], Y_o, Sabs


@pytest.mark.parametrize("M,K,N,G,mode,r", [
    (16, 256, 256, 128, 1, 0),      # the tiny configuration
    (16, 256, 256, 32, 2, 0),
    (1, 256, 48, 64, 1, 0),
    (5, 384, 200, 384, 1, 3),       # ragged N, one group per column, odd rank
    (33, 640, 37, 320, 2, 0),       # group size that neither divides nor is a multiple of 128
    (64, 1024, 272, 128, 1, 8),
    (77, 512, 200, 128, 2, 8),      # tiled form, ragged M and N
    (200, 1280, 400, 256, 2, 0),    # tiled form, several tiles each way
    (129, 384, 130, 32, 1, 16),
    (7, 512, 48, 128, 2, 16),       # decode form, rank too large for registers: read in place
    (16, 8192, 80, 128, 1, 8),      # decode form, 64 k-tiles (8 per wave) with LoRC
    (3, 5120, 96, 128, 2, 5),       # decode form, 40 k-tiles (5 per wave)
    (9, 2560, 176, 128, 1, 8),      # decode form, 20 k-tiles (3 per wave, the last four waves one fewer)
    (11, 5888, 112, 128, 1, 8),     # decode form, 46 k-tiles (6 per wave, the last two waves one fewer)
    (16, 7168, 64, 64, 2, 4),       # decode form, 56 k-tiles (7 per wave), groups of 64
    (17, 384, 72, 128, 1, 0),       # smallest M of the tiled form (64 x 128 tiles), N not a multiple of 16
    (64, 2048, 200, 256, 2, 8),     # 64 x 128 tiles, 16 k-steps, groups of 256, LoRC staged in LDS
    (48, 128, 64, 32, 1, 2),        # a single k-step (no load pipeline to speak of), groups of 32
    (130, 256, 300, 64, 2, 0),      # two k-steps, groups of 64
    (20, 8320, 48, 128, 1, 0),      # N < 64: streaming fallback
    (64, 4096, 128, 128, 1, 8),     # one 64 x 128 tile, long K: K split 4 ways through the workspace, LoRC in the reduce
    (100, 3072, 136, 128, 1, 3),    # 4 tiles, K split 3 ways, ragged M and N
    (33, 11008, 256, 128, 2, 0),    # a down-projection's K (86 k-tiles): uneven slices
    (16, 11008, 96, 128, 1, 8),     # M <= 16 beyond 64 k-tiles, few strips: streaming fallback with LoRC
    (3, 8320, 80, 64, 2, 0),        # the same with 65 k-tiles, groups of 64
    (9, 28672, 48, 128, 1, 0),      # the same with 224 k-tiles
    # decode form with a workgroup count that is a multiple of 8 (strips handed out in pairs per XCD):
    (16, 256, 128, 128, 1, 0),      # 8 strips on 8 workgroups: half of them start past the last strip
    (5, 512, 1664, 128, 2, 8),      # 104 strips on 104 workgroups, some start past the end
    (16, 256, 4100, 128, 1, 0),     # 257 strips on 256 workgroups: one ragged strip in the second round
    (2, 384, 6000, 128, 1, 3),      # 375 strips on 256 workgroups
])
def test_gemm_small_shapes_full_compare(M, K, N, G, mode, r):
    Y, Y_o, Sabs = _gemm_case(M, K, N, G, mode, r)
    check_gemm(Y, Y_o, Sabs, f"M{M} K{K} N{N} G{G} mode{mode} r{r}")


def _check_bf16(Y, Y_o, Sabs, what):
    """bfloat16 output against the oracle's float32 result: the stored value is the bfloat16 rounding of a
    float32 value within the GEMM tolerance of the oracle's, so it is the oracle's own rounding or the bfloat16
    neighbour of it (where the two float32 values straddle a rounding boundary), and never further from the
    oracle's float32 value than the tolerance plus half a bfloat16 step."""
    want = torch.from_numpy(np.asarray(Y_o, np.float32)).to(torch.bfloat16).float().numpy().astype(np.float64)
    Y = np.asarray(Y, np.float64)
    assert np.all(np.abs(Y - Y_o) <= ELEM * Sabs + np.abs(Y_o) * 2.0 ** -8 + 1e-300), what
    # (where the sum nearly cancels, the tolerance on the float32 value can exceed a bfloat16 step of the result)
    assert np.all(np.abs(Y - want) <= ELEM * Sabs + np.abs(want) * 2.0 ** -7 + 1e-300), what
    assert (Y == want).mean() > 0.99, what


@pytest.mark.parametrize("M,K,N,G,mode,r", [
    (40, 512, 96, 128, 1, 0),       # 64 x 128 tile
    (16, 1024, 272, 128, 1, 8),     # decode form, LoRC in registers, ragged N
    (5, 512, 1664, 128, 2, 0),      # decode form, strips in pairs, column scales
    (7, 512, 48, 128, 2, 16),       # decode form, LoRC read in place
    (16, 8192, 80, 128, 1, 8),      # decode form, upper band in LDS
    (20, 8320, 48, 128, 1, 0),      # streaming fallback
    (16, 11008, 96, 128, 1, 8),     # streaming fallback for at most 16 tokens, LoRC
    (64, 4096, 128, 128, 1, 8),     # K split through the workspace: the reduce kernel stores
    (100, 3072, 136, 128, 2, 3),    # K split 3 ways, ragged M and N
    (64, 1024, 272, 128, 1, 8),     # 64 x 128 tiles, two wave groups
    (200, 1280, 400, 256, 2, 0),    # 64 x 128 tiles, several each way
])
def test_gemm_bf16_output_small_shapes(M, K, N, G, mode, r):
    Y, Y_o, Sabs = _gemm_case(M, K, N, G, mode, r, out_dtype=torch.bfloat16)
    _check_bf16(Y, Y_o, Sabs, f"bf16 M{M} K{K} N{N} G{G} mode{mode} r{r}")


@pytest.mark.parametrize("name,M", [("llama7b_qkv", 4096), ("opt1p3b_fc1", 2048), ("llama7b_qkv", 1000),
                                    ("llama7b_qkv", 512), ("llama7b_qkv", 256), ("llama13b_ffn_lorc", 2048),
                                    ("llama70b_ffn_decode", 64), ("llama70b_ffn_decode", 16),
                                    ("llama70b_ffn_down", 16), ("llama7b_ffn_down", 64)])
def test_gemm_bf16_output_full_size_sampled(name, M):
    """Every tile shape the planner picks for the benchmark configurations (128 x 256, 256 x 256, 128 x 192,
    128 x 128 or 64 x 128, with and without a K-split), the decode form and its chunked-K variant, storing bfloat16."""
    cfg = CFG[name]
    Y, Y_o, Sabs = _gemm_case(M, cfg.K, cfg.N, cfg.G, cfg.mode, cfg.rank, seed_cfg=name, full=False,
                              out_dtype=torch.bfloat16)
    _check_bf16(Y, Y_o, Sabs, f"bf16 {name} M={M}")


def test_gemm_zero_rows_and_signed_zeros():
    cfg = CFG["tiny"]
    x = inputs.bf16_bits_to_f32(inputs.make_x(cfg, 16)).copy()
    x[3] = 0.0
    x[7] = -0.0
    Y, Y_o, Sabs = _gemm_case(16, 256, 256, 128, 1, 0, x_override=inputs.f32_to_bf16_bits(x))
    assert np.all(Y[3] == 0) and np.all(Y[7] == 0)
    check_gemm(Y, Y_o, Sabs + 1e-300)


@pytest.mark.parametrize("M,K,N", [(16, 2048, 512), (200, 2048, 512)])
def test_gemm_on_post_relu_activations(M, K, N):
    """The fc2-like input of Section 3's observation (2): half the values exactly zero, the rest one-sided, plus
    outlier channels.  Quantized through the fused ReLU entry point, multiplied in both GEMM forms."""
    cfg = inputs.Config("relu", K, N, (M,), 128, 1, 0.01, 0, 20.0, 0, 77)
    X = inputs.make_x(cfg, M)
    Xr = oracle.relu_bf16(X)
    Y, Y_o, Sabs = _gemm_case(M, K, N, 128, 1, 0, x_override=Xr)
    check_gemm(Y, Y_o, Sabs + 1e-300, f"post-ReLU M{M}")
    Xq, sx = zqfp.relu_quantize_act_fp8(bf16_tensor(X))
    Xq_o, sx_o = oracle.quantize_act(Xr)
    assert np.array_equal(_sync_np(Xq), Xq_o) and bits_equal_f32(_sync_np(sx), sx_o)
    assert (Xq_o == 0).mean() > 0.4


FULL = [
    ("opt1p3b_fc1", 2048), ("llama7b_qkv", 1000),  # M = 1000: 128 x 192 tiles with a ragged last row block
    ("llama7b_qkv", 1), ("llama7b_qkv", 16), ("llama7b_qkv", 256), ("llama7b_qkv", 4096),
    ("llama7b_ffn_up", 1), ("llama7b_ffn_up", 16), ("llama7b_ffn_up", 256), ("llama7b_ffn_up", 4096),
    ("llama13b_ffn_lorc", 16), ("llama13b_ffn_lorc", 2048),
    ("llama70b_ffn_decode", 1), ("llama70b_ffn_decode", 4), ("llama70b_ffn_decode", 16), ("llama70b_ffn_decode", 64),
    # long K, few output channels (down projections, attention output): chunked decode form, K-split tiles
    ("llama7b_ffn_down", 16), ("llama7b_ffn_down", 4096), ("llama13b_ffn_down", 16), ("llama13b_ffn_down", 2048),
    ("llama70b_ffn_down", 1), ("llama70b_ffn_down", 16), ("llama70b_ffn_down", 64),
    ("llama7b_attn_out", 16), ("llama7b_attn_out", 4096),
]


@pytest.mark.parametrize("M,K,N,G,mode,r", [(1024, 1024, 12200, 128, 2, 8), (960, 256, 12288, 64, 1, 0),
                                         (1000, 384, 12280, 128, 1, 3)])
def test_gemm_tiles_of_192_columns_sampled_outputs(M, K, N, G, mode, r):
    """Shapes the planner gives 128 x 192 tiles (a single round that 256 x 256 tiles would leave partly idle):
    ragged last row block, ragged last column tile, LoRC in the epilogue, both scale methods."""
    Y, Y_o, Sabs = _gemm_case(M, K, N, G, mode, r, full=False)
    check_gemm(Y, Y_o, Sabs, f"192-column tiles M{M} K{K} N{N}")


@pytest.mark.parametrize("name,M", FULL)
def test_gemm_full_size_sampled_outputs(name, M):
    """The benchmark configurations at full size, in the launch configuration
    the benchmark times; the oracle computes 4096 sampled outputs one by one."""
    cfg = CFG[name]
    Y, Y_o, Sabs = _gemm_case(M, cfg.K, cfg.N, cfg.G, cfg.mode, cfg.rank, seed_cfg=name, full=False)
    fro, ratio = check_gemm(Y, Y_o, Sabs, f"{name} M={M}")
    print(f"{name} M={M}: rel-Frobenius {fro:.2e}, max|err|/sum|aw| {ratio:.2e}")


# ------------------------------------------------------------------ accumulation modes
def _all_exponent_x(M, K, seed=0):
    """Rows drawn uniformly over all finite E4M3 codes (every exponent equally
    likely, row maximum 448): the widest dynamic range the format allows inside
    every run of 8 consecutive k."""
    rng = np.random.default_rng(seed)
    vals = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
    finite = np.array([c for c in range(256) if (c & 0x7F) != 0x7F])
    x = vals[rng.choice(finite, (M, K))]
    x[:, 0] = 448.0
    return inputs.f32_to_bf16_bits(x)


@pytest.mark.parametrize("M,K,N", [(16, 1024, 256), (96, 1024, 256)])
def test_exact_mode_holds_the_bound_on_widest_dynamic_range(M, K, N):
    X = _all_exponent_x(M, K)
    Y, Y_o, Sabs = _gemm_case(M, K, N, 128, 1, 0, x_override=X)
    fro, ratio = check_gemm(Y, Y_o, Sabs, "all-exponent rows, exact accumulation")
    print(f"exact: rel-Fro {fro:.2e} ratio {ratio:.2e}")


@pytest.mark.parametrize("M,K,N,seed_cfg", [(16, 256, 256, "tiny"), (16, 4096, 1024, "llama7b_qkv"),
                                            (256, 4096, 1024, "llama70b_ffn_decode")])
def test_fast_mode_meets_its_documented_bound(M, K, N, seed_cfg):
    """One-pass accumulation is OUTSIDE the parity tolerance on activations with
    outlier channels (the matrix core truncates products more than 8 binades
    below the largest of their run of 8); its documented bounds are relative
    Frobenius error <= 1e-4 and |err| <= 2^-10 * sum|a w|."""
    cfg = CFG[seed_cfg]
    cfg = inputs.Config(cfg.name, K, N, (M,), 128, 1, cfg.outlier_frac, cfg.outlier_count, cfg.outlier_gain, 0, cfg.seed)
    X = inputs.make_x(cfg, M)
    W, packed = _weights(cfg, 128, 1)
    Xq, sx = zqfp.quantize_act_fp8(bf16_tensor(X))
    Y = _sync_np(zqfp.w4a8_gemm(Xq, sx, packed, N, 128, accum=zqfp.ACCUM_FAST))
    Xq_o, sx_o = oracle.quantize_act(X)
    codes_o, exps_o, c_o, _ = oracle.pack_weight(W, 128, 1)
    Y_o, Sabs = oracle.gemm(Xq_o, sx_o, codes_o, exps_o, c_o, 128)
    err = np.abs(Y.astype(np.float64) - Y_o)
    fro = np.linalg.norm(Y - Y_o) / np.linalg.norm(Y_o)
    ratio = (err / Sabs).max()
    print(f"fast: rel-Fro {fro:.2e} ratio {ratio:.2e} (2^-18 = {2.0**-18:.2e})")
    assert fro <= 1e-4 and ratio <= 2.0 ** -10


@pytest.mark.gpu
def test_measurement_probes_run_and_report_sane_rates():
    """The two probes behind bench.py's measured ceilings: they must run, leave their inputs
    untouched and land between loose physical bounds (not a parity check: no method arithmetic)."""
    src = torch.full((1 << 28,), 7, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1024, dtype=torch.int32, device="cuda")
    ops = torch.arange(1024, dtype=torch.int32, device="cuda")
    fsink = torch.zeros(512 * 64, dtype=torch.float32, device="cuda")
    zqfp.probe_stream_read(src, sink, 1024)
    flop = zqfp.probe_mfma(ops, fsink, 10, 64)
    torch.cuda.synchronize()
    assert flop == 2.0 * 16 * 16 * 128 * 32 * 8 * 10 * 64
    assert int(src[:4096].sum().item()) == 7 * 4096 and int(ops[5].item()) == 5
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    zqfp.probe_stream_read(src, sink, 1024)
    b.record()
    torch.cuda.synchronize()
    gbs = src.numel() / (a.elapsed_time(b) * 1e-3) / 1e9
    assert 500.0 < gbs < 20000.0, gbs


def _gain_bits(K, seed=3):
    rng = np.random.default_rng(seed)
    return inputs.f32_to_bf16_bits((1.0 + 0.1 * rng.standard_normal(K)).astype(np.float32))


@pytest.mark.gpu
@pytest.mark.parametrize("name,M,eps", [("tiny", 16, 1e-5), ("opt1p3b_fc1", 300, 1e-5), ("llama7b_qkv", 77, 1e-6),
                                        ("llama13b_ffn_lorc", 16, 1e-5), ("llama70b_ffn_decode", 64, 1e-5),
                                        ("llama70b_ffn_decode", 130, 1e-2),
                                        # many tokens without LoRC: the wave-per-token kernel (K = 2048, 4096, 8192)
                                        ("opt1p3b_fc1", 1027, 1e-5), ("llama7b_qkv", 1100, 1e-5)])
def test_fused_rmsnorm_quantizer_equals_the_unfused_sequence_bit_for_bit(name, M, eps):
    """RMS normalisation fused in front of the quantizer: codes and scales are those of the oracle's
    normalisation (bf16 result) followed by the oracle's quantizer; the LoRC left factor is taken from
    the normalised rows."""
    cfg = CFG[name]
    X = inputs.make_x(cfg, M)
    X[M // 2] = 0  # an all-zero token
    g = _gain_bits(cfg.K)
    Yn = oracle.rmsnorm_bf16(X, g, eps)
    Xq_o, sx_o = oracle.quantize_act(Yn)
    gd = bf16_tensor(g.reshape(1, -1)).reshape(-1).contiguous()
    if cfg.rank:
        U, _ = inputs.make_uv(cfg)
        T_o, Tabs = oracle.lorc_left(Yn, U)
        Xq, sx, T = zqfp.rmsnorm_quantize_act_fp8(bf16_tensor(X), gd, eps, f16_tensor(U))
        T = _sync_np(T)
        assert np.all(np.abs(T - T_o) <= 2.0 ** -18 * Tabs + 1e-30)
    else:
        Xq, sx = zqfp.rmsnorm_quantize_act_fp8(bf16_tensor(X), gd, eps)
    Xq, sx = _sync_np(Xq), _sync_np(sx)
    assert bits_equal_f32(sx, sx_o)
    assert np.array_equal(Xq, Xq_o)
    assert np.all(Xq[M // 2] == 0) and sx[M // 2] == 1.0


@pytest.mark.gpu
def test_fused_rmsnorm_quantizer_argument_checks():
    X = bf16_tensor(inputs.make_x(CFG["tiny"], 4))
    g = bf16_tensor(_gain_bits(256).reshape(1, -1)).reshape(-1).contiguous()
    with pytest.raises(zqfp.ZqfpError):
        zqfp.rmsnorm_quantize_act_fp8(X, g, 0.0)
    with pytest.raises(zqfp.ZqfpError):
        zqfp.rmsnorm_quantize_act_fp8(X, g[:128].contiguous(), 1e-5)


def _bias_bits(K):
    rng = np.random.default_rng(4243)
    return inputs.f32_to_bf16_bits((0.05 * rng.standard_normal(K)).astype(np.float32))


@pytest.mark.gpu
@pytest.mark.parametrize("name,M,eps,shift", [("tiny", 16, 1e-5, 0.0), ("opt1p3b_fc1", 300, 1e-5, 0.25),
                                              ("llama7b_qkv", 77, 1e-6, -3.0), ("llama13b_ffn_lorc", 16, 1e-5, 0.5),
                                              ("llama70b_ffn_decode", 64, 1e-5, 0.0),
                                              ("llama70b_ffn_decode", 130, 1e-2, 40.0),
                                              # many tokens without LoRC: the wave-per-token kernel
                                              ("opt1p3b_fc1", 1027, 1e-5, 1.0), ("llama7b_qkv", 1100, 1e-5, 0.0)])
def test_fused_layernorm_quantizer_equals_the_unfused_sequence_bit_for_bit(name, M, eps, shift):
    """Layer normalisation (gain and bias) fused in front of the quantizer: codes and scales are those of the
    oracle's normalisation (bf16 result) followed by the oracle's quantizer; rows carry a common offset so that
    the mean matters, one token is all zero (its normalised row is the bias) and one is constant (variance 0)."""
    cfg = CFG[name]
    X = inputs.make_x(cfg, M)
    if shift:
        rows = np.linspace(-shift, shift, M, dtype=np.float32).reshape(-1, 1)
        X = inputs.f32_to_bf16_bits(inputs.bf16_bits_to_f32(X) + rows)
    X[M // 2] = 0
    X[M // 3] = inputs.f32_to_bf16_bits(np.full(cfg.K, 1.5, np.float32))
    g, b = _gain_bits(cfg.K), _bias_bits(cfg.K)
    Yn = oracle.layernorm_bf16(X, g, b, eps)
    Xq_o, sx_o = oracle.quantize_act(Yn)
    gd = bf16_tensor(g.reshape(1, -1)).reshape(-1).contiguous()
    bd = bf16_tensor(b.reshape(1, -1)).reshape(-1).contiguous()
    if cfg.rank:
        U, _ = inputs.make_uv(cfg)
        T_o, Tabs = oracle.lorc_left(Yn, U)
        Xq, sx, T = zqfp.layernorm_quantize_act_fp8(bf16_tensor(X), gd, bd, eps, f16_tensor(U))
        T = _sync_np(T)
        assert np.all(np.abs(T - T_o) <= 2.0 ** -18 * Tabs + 1e-30)
    else:
        Xq, sx = zqfp.layernorm_quantize_act_fp8(bf16_tensor(X), gd, bd, eps)
    Xq, sx = _sync_np(Xq), _sync_np(sx)
    assert bits_equal_f32(sx, sx_o)
    assert np.array_equal(Xq, Xq_o)
    # all-zero and constant tokens normalise to the bias alone
    Xq_b, sx_b = oracle.quantize_act(b.reshape(1, -1))
    for m in (M // 2, M // 3):
        assert np.array_equal(Xq[m], Xq_b[0]) and bits_equal_f32(sx[m:m + 1], sx_b)


@pytest.mark.gpu
@pytest.mark.parametrize("K,M,rank", [(11008, 5, 0), (28672, 3, 8), (32768, 2, 0), (8320, 70, 8), (128, 9, 0)])
def test_fused_normalisations_on_rows_beyond_the_register_budget_of_256_threads(K, M, rank):
    """Rows of up to 32768 elements (the documented limit) and the shortest row, both normalisations."""
    import dataclasses
    cfg = dataclasses.replace(CFG["llama7b_qkv"], K=K, N=64, G=64, rank=rank, seed=K + M)
    X = inputs.f32_to_bf16_bits(inputs.bf16_bits_to_f32(inputs.make_x(cfg, M)) + np.float32(0.75))
    g, b = _gain_bits(K), _bias_bits(K)
    gd = bf16_tensor(g.reshape(1, -1)).reshape(-1).contiguous()
    bd = bf16_tensor(b.reshape(1, -1)).reshape(-1).contiguous()
    U = inputs.make_uv(cfg)[0] if rank else None
    Ud = f16_tensor(U) if rank else None
    for Yn, out in ((oracle.rmsnorm_bf16(X, g, 1e-5), zqfp.rmsnorm_quantize_act_fp8(bf16_tensor(X), gd, 1e-5, Ud)),
                    (oracle.layernorm_bf16(X, g, b, 1e-5),
                     zqfp.layernorm_quantize_act_fp8(bf16_tensor(X), gd, bd, 1e-5, Ud))):
        Xq_o, sx_o = oracle.quantize_act(Yn)
        assert bits_equal_f32(_sync_np(out[1]), sx_o)
        assert np.array_equal(_sync_np(out[0]), Xq_o)
        if rank:
            T_o, Tabs = oracle.lorc_left(Yn, U)
            assert np.all(np.abs(_sync_np(out[2]) - T_o) <= 2.0 ** -18 * Tabs + 1e-30)


def _check_quantized(out, Y, U):
    """out = (Xq, sx[, T]) of a fused quantizer call against the oracle's quantizer applied to the oracle's Y."""
    Xq_o, sx_o = oracle.quantize_act(Y)
    assert bits_equal_f32(_sync_np(out[1]), sx_o)
    assert np.array_equal(_sync_np(out[0]), Xq_o)
    if U is not None:
        T_o, Tabs = oracle.lorc_left(Y, U)
        assert np.all(np.abs(_sync_np(out[2]) - T_o) <= 2.0 ** -18 * Tabs + 1e-30)


def _producer_case(K, M, rank, seed):
    import dataclasses
    cfg = dataclasses.replace(CFG["llama7b_qkv"], K=K, N=64, G=64, rank=rank, seed=seed)
    X = inputs.make_x(cfg, M)
    R = inputs.make_x(dataclasses.replace(cfg, seed=seed + 1), M)
    U = inputs.make_uv(cfg)[0] if rank else None
    return X, R, U


PRODUCER_SHAPES = [(256, 16, 0), (2048, 300, 0), (4096, 77, 8), (8192, 1030, 0), (4096, 1100, 0), (2048, 1027, 0),
                   (4096, 1100, 8), (8192, 1025, 8), (5120, 1024, 8),
                   (11008, 40, 8), (28672, 3, 0), (32768, 2, 0), (128, 9, 0), (8320, 70, 8)]


@pytest.mark.gpu
@pytest.mark.parametrize("K,M,rank", PRODUCER_SHAPES)
def test_residual_add_fused_in_front_of_both_normalisations(K, M, rank):
    """h = bf16(X + R) is written out bit-exactly and is what gets normalised and quantized; H may be R itself."""
    X, R, U = _producer_case(K, M, rank, 100 + M)
    g, b = _gain_bits(K), _bias_bits(K)
    gd = bf16_tensor(g.reshape(1, -1)).reshape(-1).contiguous()
    bd = bf16_tensor(b.reshape(1, -1)).reshape(-1).contiguous()
    Ud = f16_tensor(U) if rank else None
    H_o = oracle.add_bf16(X, R)
    for bias_dev, Yn in ((None, oracle.rmsnorm_bf16(H_o, g, 1e-5)), (bd, oracle.layernorm_bf16(H_o, g, b, 1e-5))):
        out = zqfp.add_norm_quantize_act_fp8(bf16_tensor(X), bf16_tensor(R), gd, 1e-5, bias=bias_dev, U=Ud)
        assert np.array_equal(_sync_np(out[0].view(torch.int16)).view(np.uint16), H_o)
        _check_quantized(out[1:], Yn, U)
    # in place: the residual stream is overwritten by the sum; rows of X taken from a wider tensor
    wide = torch.zeros((M, K + 64), dtype=torch.bfloat16, device="cuda")
    wide[:, :K] = bf16_tensor(X)
    Rd = bf16_tensor(R)
    out = zqfp.add_norm_quantize_act_fp8(wide[:, :K], Rd, gd, 1e-5, U=Ud, H=Rd)
    assert out[0].data_ptr() == Rd.data_ptr()
    assert np.array_equal(_sync_np(Rd.view(torch.int16)).view(np.uint16), H_o)
    _check_quantized(out[1:], oracle.rmsnorm_bf16(H_o, g, 1e-5), U)


@pytest.mark.gpu
@pytest.mark.parametrize("K,M,rank", PRODUCER_SHAPES)
def test_relu_fused_in_front_of_the_quantizer(K, M, rank):
    X, _, U = _producer_case(K, M, rank, 200 + M)
    X[M // 2] = inputs.f32_to_bf16_bits(-np.abs(inputs.bf16_bits_to_f32(X[M // 2])))  # a token that ReLU voids entirely
    out = zqfp.relu_quantize_act_fp8(bf16_tensor(X), f16_tensor(U) if rank else None)
    _check_quantized(out, oracle.relu_bf16(X), U)
    assert np.all(_sync_np(out[0])[M // 2] == 0) and _sync_np(out[1])[M // 2] == 1.0


@pytest.mark.gpu
@pytest.mark.parametrize("K,M,rank", PRODUCER_SHAPES)
def test_gated_silu_fused_in_front_of_the_quantizer(K, M, rank):
    """silu(gate) * up with gate and up taken as the two halves of one [M, 2K] tensor, as a fused gate/up
    projection would leave them."""
    G, Up, U = _producer_case(K, M, rank, 300 + M)
    G = inputs.f32_to_bf16_bits(inputs.bf16_bits_to_f32(G) * np.float32(0.5))
    both = torch.cat([bf16_tensor(G), bf16_tensor(Up)], dim=1)
    out = zqfp.swiglu_quantize_act_fp8(both[:, :K], both[:, K:], f16_tensor(U) if rank else None)
    _check_quantized(out, oracle.swiglu_bf16(G, Up), U)


@pytest.mark.gpu
def test_gated_silu_every_gate_value_bit_exact():
    """The product silu(g) * u as the kernel rounds it to bf16 (returned through H), for every finite bf16
    gate value against a spread of up values: ordinary ones, powers of two at the ends of the binary32
    range, subnormals, values one bf16 step from 1, and random bit patterns.  The kernel evaluates most
    values in binary32 and only those near a rounding boundary or outside its safe ranges in binary64: all
    must round as the binary64 evaluation does."""
    K = 8192
    gates = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    gates[(gates & 0x7F80) == 0x7F80] = 0x3F80          # infinities and NaNs: 1.0 instead
    gates = gates.reshape(8, K)
    fixed = np.array([1.0, -1.0, 0.5, -0.5, 3.140625, -2.71875, 1.0078125, 0.99609375, 1e-3, -1e3, 2.0 ** -30, 2.0 ** -31,
                      2.0 ** 30, 2.0 ** 31, 2.0 ** -126, 2.0 ** -130, -2.0 ** -133, 2.0 ** 100, -2.0 ** 127, 2.0 ** -60,
                      0.0, -0.0, 6.0, 448.0], dtype=np.float32)
    ups = list(inputs.f32_to_bf16_bits(fixed))
    rng = np.random.default_rng(77)
    G_rows, U_rows = [], []
    for u in ups:
        for b in range(8):
            G_rows.append(gates[b]); U_rows.append(np.full(K, u, np.uint16))
    for j in range(24):                                   # random up values against every gate value
        r = rng.integers(0, 65536, size=(8, K), dtype=np.uint32).astype(np.uint16)
        r[(r & 0x7F80) == 0x7F80] ^= 0x4000
        if j >= 12:                                       # half of them of ordinary magnitude (exponent field 112 .. 135)
            r = (r & 0x807F) | (rng.integers(112, 136, size=(8, K), dtype=np.uint32).astype(np.uint16) << 7)
        for b in range(8):
            G_rows.append(gates[b]); U_rows.append(r[b])
    G = np.ascontiguousarray(np.stack(G_rows)); Up = np.ascontiguousarray(np.stack(U_rows))
    H = torch.empty(G.shape, dtype=torch.bfloat16, device="cuda")
    zqfp.swiglu_quantize_act_fp8(bf16_tensor(G), bf16_tensor(Up), H=H)
    got = _sync_np(H.view(torch.int16)).view(np.uint16)
    want = oracle.swiglu_bf16(G, Up)
    bad = np.argwhere(got != want)
    assert bad.size == 0, (len(bad), [(hex(G[i, j]), hex(Up[i, j]), hex(got[i, j]), hex(want[i, j])) for i, j in bad[:8]])


@pytest.mark.gpu
def test_fused_producer_argument_checks():
    X = bf16_tensor(inputs.make_x(CFG["tiny"], 4))
    g = bf16_tensor(_gain_bits(256).reshape(1, -1)).reshape(-1).contiguous()
    with pytest.raises(zqfp.ZqfpError):
        zqfp.add_norm_quantize_act_fp8(X, X[:2].contiguous(), g, 1e-5)
    with pytest.raises(zqfp.ZqfpError):
        zqfp.add_norm_quantize_act_fp8(X, X, g, 0.0)
    with pytest.raises(zqfp.ZqfpError):
        zqfp.swiglu_quantize_act_fp8(X, X[:, :128])
    lib = zqfp.lib()
    assert lib.zqfp_swiglu_quantize_act_fp8(X.data_ptr(), None, 256, None, 4, 256, 256, None, None, None, 0, None, None) != 0
    assert lib.zqfp_relu_quantize_act_fp8(X.data_ptr(), 4, 65536, 65536, X.data_ptr(), X.data_ptr(), None, 0, None, None) != 0


@pytest.mark.gpu
def test_fused_layernorm_quantizer_argument_checks():
    X = bf16_tensor(inputs.make_x(CFG["tiny"], 4))
    g = bf16_tensor(_gain_bits(256).reshape(1, -1)).reshape(-1).contiguous()
    b = bf16_tensor(_bias_bits(256).reshape(1, -1)).reshape(-1).contiguous()
    with pytest.raises(zqfp.ZqfpError):
        zqfp.layernorm_quantize_act_fp8(X, g, b, 0.0)
    with pytest.raises(zqfp.ZqfpError):
        zqfp.layernorm_quantize_act_fp8(X, g, b[:128].contiguous(), 1e-5)


def test_gemm_k_split_is_optional_and_agrees_with_the_unsplit_launch():
    """Without a workspace the same call runs un-split; both results meet the parity bar and the
    workspace query names a size exactly when a split is planned."""
    M, K, N, G = 64, 4096, 128, 128
    assert zqfp.gemm_workspace_bytes(M, K, N) == 4 * M * N * 4
    assert zqfp.gemm_workspace_bytes(4096, 4096, 12288) == 0 and zqfp.gemm_workspace_bytes(16, 8192, 28672) == 0
    cfg = inputs.Config("t", K, N, (M,), G, 1, 0.01, 0, 20.0, 0, 0)
    X = inputs.make_x(cfg, M)
    W, packed = _weights(cfg, G, 1)
    Xq_o, sx_o = oracle.quantize_act(X)
    codes_o, exps_o, c_o, _ = oracle.pack_weight(W, G, 1)
    Y_o, Sabs = oracle.gemm(Xq_o, sx_o, codes_o, exps_o, c_o, G)
    Xq, sx = zqfp.quantize_act_fp8(bf16_tensor(X))
    Y_split = _sync_np(zqfp.w4a8_gemm(Xq, sx, packed, N, G))
    Y_plain = _sync_np(zqfp.w4a8_gemm(Xq, sx, packed, N, G, workspace=False))
    check_gemm(Y_split, Y_o, Sabs, "K split")
    check_gemm(Y_plain, Y_o, Sabs, "no workspace")
    # M <= 16 beyond 64 k-tiles: a workspace is named; with few strips both calls take the streaming kernel
    assert zqfp.gemm_workspace_bytes(8, 8320, 128) == 2 * 8 * 128 * 4
    Yd = _sync_np(zqfp.w4a8_gemm(Xq[:8].contiguous(), sx[:8].contiguous(), packed, N, G))
    Yd0 = _sync_np(zqfp.w4a8_gemm(Xq[:8].contiguous(), sx[:8].contiguous(), packed, N, G,
                                  workspace=False))
    check_gemm(Yd, Y_o[:8], Sabs[:8], "decode")
    check_gemm(Yd0, Y_o[:8], Sabs[:8], "decode, no workspace")


def test_binding_and_library_refuse_mismatched_blob_workspace_and_output():
    """What would otherwise become out-of-bounds device accesses: a blob packed for other sizes, a short
    workspace, an output of the wrong shape.  Refused on the host, nothing is enqueued."""
    M, K, N, G = 64, 4096, 128, 128
    cfg = inputs.Config("t", K, N, (M,), G, 1, 0.01, 0, 20.0, 0, 0)
    W, packed = _weights(cfg, G, 1)
    Xq, sx = zqfp.quantize_act_fp8(bf16_tensor(inputs.make_x(cfg, M)))
    zqfp.packed_weight_check(packed, K, N, G)
    for k, n, g in ((K, N, 256), (K, N - 1, G), (2 * K, N // 2, G)):
        with pytest.raises(zqfp.ZqfpError) as e:
            zqfp.packed_weight_check(packed, k, n, g)
        assert e.value.code == -7
    with pytest.raises(zqfp.ZqfpError) as e:
        zqfp.w4a8_gemm(Xq, sx, packed, N, 256)            # blob size differs for G = 256
    assert e.value.code == -2
    with pytest.raises(zqfp.ZqfpError) as e:
        zqfp.w4a8_gemm(Xq, sx, packed, N, G, workspace=torch.empty(4 * M * N * 4 - 16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -6
    with pytest.raises(zqfp.ZqfpError) as e:              # the library's own check, past the binding's
        zqfp._check(zqfp.lib().zqfp_w4a8_gemm(Xq.data_ptr(), sx.data_ptr(), M, K, packed.data_ptr(), N, G,
                                              torch.empty((M, N), device="cuda").data_ptr(), N, 0, 0,
                                              torch.empty(1024, dtype=torch.uint8, device="cuda").data_ptr(), 1024, None))
    assert e.value.code == -6 and "workspace" in str(e.value)
    for bad in (torch.empty((M, N + 8), device="cuda"), torch.empty((M, N), device="cuda", dtype=torch.float16),
                torch.empty((N, M), device="cuda").t(), torch.empty((M, N))):
        with pytest.raises(zqfp.ZqfpError):
            zqfp.w4a8_gemm(Xq, sx, packed, N, G, out=bad)
    with pytest.raises(zqfp.ZqfpError):
        zqfp.unpack_codes(packed, K, N, 256)
    Y = zqfp.w4a8_gemm(Xq, sx, packed, N, G, out=torch.empty((M, N + 8), device="cuda")[:, :N])  # a row stride is fine
    assert torch.equal(Y, zqfp.w4a8_gemm(Xq, sx, packed, N, G))


@pytest.mark.parametrize("M,K,N,G,mode,r", [(16, 8320, 8192, 64, 2, 8),     # 65 k-tiles: chunks of 33 and 32
                                            (5, 16640, 5504, 128, 1, 0),    # 130 k-tiles: three chunks of 44, 44, 42
                                            (7, 14080, 8192, 128, 1, 8)])   # 110 k-tiles: two chunks of 55
def test_gemm_decode_long_k_in_chunks(M, K, N, G, mode, r):
    """Decode form with more than 64 k-tiles and strips enough for the chunked path (partial sums
    through the workspace, scales and LoRC in the reduce kernel); sampled outputs."""
    assert zqfp.gemm_workspace_bytes(M, K, N) == -(-K // 128 // 64) * M * N * 4
    Y, Y_o, Sabs = _gemm_case(M, K, N, G, mode, r, seed_cfg="llama70b_ffn_decode", full=False, nsamples=2048)
    check_gemm(Y, Y_o, Sabs, f"decode chunks M{M} K{K} N{N}")


def test_gemm_seeded_sweep_of_small_shapes():
    """Forty seeded random shapes across every dispatch branch (decode form, chunked K, streaming
    fallback, the three tile shapes' smallest members, K split), each compared in full with the oracle."""
    rng = np.random.default_rng(20230719)
    done = 0
    while done < 40:
        M = int(rng.choice([1, 2, 7, 16, 17, 31, 64, 65, 100, 129, 257]))
        K = 128 * int(rng.integers(1, 72))
        N = int(rng.choice([1, 15, 16, 63, 64, 65, 127, 128, 200, 272, 513]))
        Gs = [g for g in (32, 64, 128, 256, 384, K) if K % g == 0 and K // g <= 256]
        G = int(rng.choice(Gs))
        mode = int(rng.integers(1, 3))
        r = int(rng.choice([0, 0, 3, 8, 16]))
        if M * K * N > 3.0e8:
            continue
        Y, Y_o, Sabs = _gemm_case(M, K, N, G, mode, r)
        check_gemm(Y, Y_o, Sabs, f"sweep M{M} K{K} N{N} G{G} mode{mode} r{r}")
        done += 1


# ------------------------------------------------------------------ every tile shape the tiled form has
@pytest.mark.parametrize("bm,bn,kg", [(64, 128, 1), (64, 128, 2), (64, 192, 1), (64, 192, 2), (64, 256, 1), (64, 256, 2),
                                      (128, 128, 1), (128, 192, 1), (128, 256, 1), (256, 256, 1)])
def test_gemm_every_tile_shape_with_and_without_a_k_split(bm, bn, kg):
    """The planner picks a tile shape from the problem size; here every shape (and both wave-group counts of the
    64-row tiles) is forced in turn onto one ragged problem, unsplit and with K cut in 2 and 3 slices, LoRC in the
    tile epilogue or in the reduce kernel, float32 and bfloat16 output."""
    M, K, N, G, mode, r = 300, 1536, 1000, 128, 2, 8
    try:
        for ksplit in (1, 2, 3):
            zqfp.probe_force_tile_plan(bm, bn, ksplit, kg)
            assert (zqfp.gemm_workspace_bytes(M, K, N) > 0) == (ksplit > 1)
            Y, Y_o, Sabs = _gemm_case(M, K, N, G, mode, r)
            check_gemm(Y, Y_o, Sabs, f"{bm}x{bn} tiles, {kg} wave group(s), K in {ksplit}")
        zqfp.probe_force_tile_plan(bm, bn, 2, kg)
        Y, Y_o, Sabs = _gemm_case(M, K, N, G, mode, r, out_dtype=torch.bfloat16)
        _check_bf16(Y, Y_o, Sabs, f"{bm}x{bn} bf16")
    finally:
        zqfp.probe_force_tile_plan(0, 0, 0)


@pytest.mark.parametrize("bm,bn,kg", [(64, 128, 1), (64, 128, 2), (64, 192, 1), (64, 192, 2), (64, 256, 1), (64, 256, 2),
                                      (128, 128, 1), (128, 192, 1), (128, 256, 1), (256, 256, 1)])
def test_gemm_every_tile_shape_on_pipelines_shorter_than_the_stages(bm, bn, kg):
    """Four k-tiles in all, cut so that a wave group multiplies four, two or a single one: fewer than the LDS
    stages it keeps in flight (two or three), the case in which the pipeline's first step is also its last."""
    M, K, N, G, mode, r = 300, 512, 1000, 128, 1, 0
    try:
        for ksplit in ((1, 2, 4) if kg == 1 else (1, 2)):
            zqfp.probe_force_tile_plan(bm, bn, ksplit, kg)
            for rep in range(2):  # a fragment register read before its data arrived would differ from run to run
                Y, Y_o, Sabs = _gemm_case(M, K, N, G, mode, r)
                check_gemm(Y, Y_o, Sabs, f"{bm}x{bn} tiles, {kg} wave group(s), {K // 128 // ksplit // kg} k-tile(s) per group")
    finally:
        zqfp.probe_force_tile_plan(0, 0, 0)


def test_gemm_repeated_launches_give_the_same_bits_on_every_tile_shape():
    """A register or an LDS stage read before its data has arrived shows as results that differ from launch to
    launch; so every tile shape (FP4 and FP8 weights, both accumulation modes, unsplit and with K in slices) is
    launched several times on ragged problems with long and with very short pipelines and the outputs are
    compared bit for bit.  (What the bits should be is the other tests' business.)"""
    shapes4 = [(64, 128, 1), (64, 128, 2), (64, 192, 1), (64, 192, 2), (64, 256, 1), (64, 256, 2),
               (128, 128, 1), (128, 192, 1), (128, 256, 1), (256, 256, 1)]
    shapes8 = [(64, 128, 1), (64, 128, 2), (128, 128, 1)]
    try:
        for M, K, N in ((300, 1536, 1000), (531, 256, 520), (77, 128, 200), (260, 2304, 264)):
            cfg = inputs.Config("d", K, N, (M,), 128, 1, 0.01, 0, 20.0, 0, 5)
            W = bf16_tensor(inputs.make_w(cfg))
            Xq, sx = zqfp.quantize_act_fp8(bf16_tensor(inputs.make_x(cfg, M)))
            p4, p8 = zqfp.pack_weight_fp4(W, 128, 1), zqfp.pack_weight_fp8(W, 128, 1)
            for wb, shapes in ((4, shapes4), (8, shapes8)):
                for bm, bn, kg in shapes:
                    for ksplit in ((1, 2, 3) if wb == 4 else (1,)):
                        if K // 128 < ksplit * kg:
                            continue
                        for accum in (zqfp.ACCUM_EXACT, zqfp.ACCUM_FAST):
                            zqfp.probe_force_tile_plan(bm, bn, ksplit, kg)
                            outs = [zqfp.w4a8_gemm(Xq, sx, p4, N, 128, accum=accum) if wb == 4
                                    else zqfp.w8a8_gemm(Xq, sx, p8, N, 128, accum=accum) for _ in range(5)]
                            torch.cuda.synchronize()
                            assert all(torch.equal(outs[0], o) for o in outs[1:]), \
                                f"wb {wb} M {M} K {K} N {N}: {bm}x{bn} tiles, {kg} group(s), K in {ksplit}, accum {accum}"
    finally:
        zqfp.probe_force_tile_plan(0, 0, 0)
