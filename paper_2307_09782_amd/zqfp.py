"""Thin Python binding of libzqfp (the C ABI in ``include/zqfp.h``).

Argument marshalling only: every function takes torch tensors that live on
the GPU, checks dtypes / contiguity, allocates the outputs with torch and
passes raw device pointers plus the current HIP stream to the library.  No
step of the path is computed here and there is no fallback: if the library
is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# ZQFP_LIB_PATH names another build of the same library (e.g. one whose host code is compiled with sanitizers)
LIB_PATH = os.environ.get("ZQFP_LIB_PATH") or os.path.join(_HERE, "libzqfp.so")

SCALE_M1, SCALE_M2 = 1, 2
OUT_F32, OUT_BF16 = 0, 1
ACCUM_EXACT, ACCUM_FAST = 0, 1

_ERR = {-1: "ZQFP_E_NULL", -2: "ZQFP_E_SHAPE", -3: "ZQFP_E_ALIGN", -4: "ZQFP_E_MODE", -5: "ZQFP_E_HIP",
        -6: "ZQFP_E_WORKSPACE", -7: "ZQFP_E_BLOB"}
BLOB_HEADER_BYTES = 256

_lib = None


class ZqfpError(RuntimeError):
    def __init__(self, code, detail=""):
        self.code = code
        super().__init__(f"libzqfp: {_ERR.get(code, code)} {detail}".strip())


def lib():
    """Load libzqfp.so (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2307_09782_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        c, p, i64 = ctypes, ctypes.c_void_p, ctypes.c_int64
        L.zqfp_version.restype = c.c_int
        L.zqfp_last_hip_error.restype = c.c_char_p
        L.zqfp_quantize_act_fp8.restype = c.c_int
        L.zqfp_quantize_act_fp8.argtypes = [p, i64, i64, i64, p, p, p, c.c_int, p, p]
        L.zqfp_packed_weight_bytes.restype = c.c_size_t
        L.zqfp_packed_weight_bytes.argtypes = [i64, i64, c.c_int]
        L.zqfp_pack_weight_fp4.restype = c.c_int
        L.zqfp_pack_weight_fp4.argtypes = [p, i64, i64, i64, c.c_int, c.c_int, p, p]
        L.zqfp_unpack_codes.restype = c.c_int
        L.zqfp_unpack_codes.argtypes = [p, i64, i64, c.c_int, p, p, p, p]
        L.zqfp_gemm_workspace_bytes.restype = c.c_size_t
        L.zqfp_gemm_workspace_bytes.argtypes = [i64, i64, i64]
        L.zqfp_w4a8_gemm.restype = c.c_int
        L.zqfp_w4a8_gemm.argtypes = [p, p, i64, i64, p, i64, c.c_int, p, i64, c.c_int, c.c_int, p, c.c_size_t, p]
        L.zqfp_w4a8_gemm_lorc.restype = c.c_int
        L.zqfp_w4a8_gemm_lorc.argtypes = [p, p, i64, i64, p, i64, c.c_int, p, p, c.c_int, p, i64, c.c_int, c.c_int, p,
                                          c.c_size_t, p]
        L.zqfp_w4a8_gemm_lorc_static.restype = c.c_int
        L.zqfp_w4a8_gemm_lorc_static.argtypes = [p, p, i64, i64, p, i64, c.c_int, p, p, c.c_int, p, i64, c.c_int, c.c_int, p]
        L.zqfp_w4a8_linear.restype = c.c_int
        L.zqfp_w4a8_linear.argtypes = [p, i64, i64, i64, p, i64, c.c_int, p, p, c.c_int, p, p, p, p, i64, c.c_int, c.c_int, p,
                                       c.c_size_t, p]
        L.zqfp_packed_weight_fp8_bytes.restype = c.c_size_t
        L.zqfp_packed_weight_fp8_bytes.argtypes = [i64, i64, c.c_int]
        L.zqfp_pack_weight_fp8.restype = c.c_int
        L.zqfp_pack_weight_fp8.argtypes = [p, i64, i64, i64, c.c_int, c.c_int, p, p]
        L.zqfp_unpack_codes_fp8.restype = c.c_int
        L.zqfp_unpack_codes_fp8.argtypes = [p, i64, i64, c.c_int, p, p, p, p]
        L.zqfp_w8a8_gemm.restype = c.c_int
        L.zqfp_w8a8_gemm.argtypes = [p, p, i64, i64, p, i64, c.c_int, p, p, c.c_int, p, i64, c.c_int, c.c_int, p]
        L.zqfp_packed_weight_check.restype = c.c_int
        L.zqfp_packed_weight_check.argtypes = [p, i64, i64, c.c_int]
        L.zqfp_rmsnorm_quantize_act_fp8.restype = c.c_int
        L.zqfp_rmsnorm_quantize_act_fp8.argtypes = [p, p, c.c_float, i64, i64, i64, p, p, p, c.c_int, p, p]
        L.zqfp_layernorm_quantize_act_fp8.restype = c.c_int
        L.zqfp_layernorm_quantize_act_fp8.argtypes = [p, p, p, c.c_float, i64, i64, i64, p, p, p, c.c_int, p, p]
        L.zqfp_add_rmsnorm_quantize_act_fp8.restype = c.c_int
        L.zqfp_add_rmsnorm_quantize_act_fp8.argtypes = [p, p, i64, p, p, c.c_float, i64, i64, i64, p, p, p, c.c_int, p, p]
        L.zqfp_add_layernorm_quantize_act_fp8.restype = c.c_int
        L.zqfp_add_layernorm_quantize_act_fp8.argtypes = [p, p, i64, p, p, p, c.c_float, i64, i64, i64, p, p, p, c.c_int, p, p]
        L.zqfp_relu_quantize_act_fp8.restype = c.c_int
        L.zqfp_relu_quantize_act_fp8.argtypes = [p, i64, i64, i64, p, p, p, c.c_int, p, p]
        L.zqfp_swiglu_quantize_act_fp8.restype = c.c_int
        L.zqfp_swiglu_quantize_act_fp8.argtypes = [p, p, i64, p, i64, i64, i64, p, p, p, c.c_int, p, p]
        L.zqfp_lorc_workspace_bytes.restype = c.c_size_t
        L.zqfp_lorc_workspace_bytes.argtypes = [i64, i64, c.c_int]
        L.zqfp_lorc_factorize.restype = c.c_int
        L.zqfp_lorc_factorize.argtypes = [p, i64, i64, i64, p, c.c_int, c.c_int, p, c.c_int, p, p, p, p, p]
        L.zqfp_gptq_workspace_bytes.restype = c.c_size_t
        L.zqfp_gptq_workspace_bytes.argtypes = [i64, i64, c.c_int]
        L.zqfp_gptq_pack_weight_fp4.restype = c.c_int
        L.zqfp_gptq_pack_weight_fp4.argtypes = [p, i64, i64, i64, p, c.c_int, c.c_int, p, p, p]
        L.zqfp_probe_stream_read.restype = c.c_int
        L.zqfp_probe_stream_read.argtypes = [p, i64, p, c.c_int, p]
        L.zqfp_probe_force_tile_plan.restype = c.c_int
        L.zqfp_probe_force_tile_plan.argtypes = [c.c_int, c.c_int, c.c_int, c.c_int]
        L.zqfp_probe_force_decode_waves.restype = c.c_int
        L.zqfp_probe_force_decode_waves.argtypes = [c.c_int]
        L.zqfp_probe_mfma.restype = c.c_int
        L.zqfp_probe_mfma.argtypes = [p, p, c.c_int, c.c_int, p]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise ZqfpError(rc, lib().zqfp_last_hip_error().decode() if rc in (-5, -6) else "")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(t):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _dev(t, dtype, ndim):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.dim() == ndim and t.is_contiguous()):
        raise TypeError(f"expected a contiguous CUDA tensor of dtype {dtype} and {ndim} dims")
    return t


def _rows(t, dtype):
    """A 2-D CUDA tensor whose rows are contiguous (the row stride may exceed the row length)."""
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.dim() == 2 and t.stride(1) == 1):
        raise TypeError(f"expected a 2-D CUDA tensor of dtype {dtype} with contiguous rows")
    return t


def quantize_act_fp8(X, U=None):
    """X [M,K] bf16 (U [K,r] fp16) -> Xq [M,K] uint8 E4M3 codes, sx [M] f32 (, T [M,r] f32)."""
    _dev(X, torch.bfloat16, 2)
    M, K = X.shape
    Xq = torch.empty((M, K), dtype=torch.uint8, device=X.device)
    sx = torch.empty((M,), dtype=torch.float32, device=X.device)
    T, r = None, 0
    if U is not None:
        _dev(U, torch.float16, 2)
        r = U.shape[1]
        T = torch.empty((M, r), dtype=torch.float32, device=X.device)
    _check(lib().zqfp_quantize_act_fp8(_ptr(X), M, K, X.stride(0), _ptr(Xq), _ptr(sx), _ptr(U), r, _ptr(T),
                                       _stream(X)))
    return (Xq, sx) if U is None else (Xq, sx, T)


def rmsnorm_quantize_act_fp8(X, gain, eps, U=None):
    """RMS normalisation (gain [K] bf16, eps > 0) fused in front of quantize_act_fp8; same outputs."""
    _dev(X, torch.bfloat16, 2), _dev(gain, torch.bfloat16, 1)
    M, K = X.shape
    if gain.shape[0] != K:
        raise ZqfpError(-2, "gain length")
    Xq = torch.empty((M, K), dtype=torch.uint8, device=X.device)
    sx = torch.empty((M,), dtype=torch.float32, device=X.device)
    T, r = None, 0
    if U is not None:
        _dev(U, torch.float16, 2)
        r = U.shape[1]
        T = torch.empty((M, r), dtype=torch.float32, device=X.device)
    _check(lib().zqfp_rmsnorm_quantize_act_fp8(_ptr(X), _ptr(gain), float(eps), M, K, X.stride(0), _ptr(Xq), _ptr(sx),
                                               _ptr(U), r, _ptr(T), _stream(X)))
    return (Xq, sx) if U is None else (Xq, sx, T)


def layernorm_quantize_act_fp8(X, gain, bias, eps, U=None):
    """Layer normalisation (gain, bias [K] bf16, eps > 0) fused in front of quantize_act_fp8; same outputs."""
    _dev(X, torch.bfloat16, 2), _dev(gain, torch.bfloat16, 1), _dev(bias, torch.bfloat16, 1)
    M, K = X.shape
    if gain.shape[0] != K or bias.shape[0] != K:
        raise ZqfpError(-2, "gain / bias length")
    Xq = torch.empty((M, K), dtype=torch.uint8, device=X.device)
    sx = torch.empty((M,), dtype=torch.float32, device=X.device)
    T, r = None, 0
    if U is not None:
        _dev(U, torch.float16, 2)
        r = U.shape[1]
        T = torch.empty((M, r), dtype=torch.float32, device=X.device)
    _check(lib().zqfp_layernorm_quantize_act_fp8(_ptr(X), _ptr(gain), _ptr(bias), float(eps), M, K, X.stride(0), _ptr(Xq),
                                                 _ptr(sx), _ptr(U), r, _ptr(T), _stream(X)))
    return (Xq, sx) if U is None else (Xq, sx, T)


def _quant_outputs(X, U):
    M, K = X.shape
    Xq = torch.empty((M, K), dtype=torch.uint8, device=X.device)
    sx = torch.empty((M,), dtype=torch.float32, device=X.device)
    T, r = None, 0
    if U is not None:
        _dev(U, torch.float16, 2)
        r = U.shape[1]
        T = torch.empty((M, r), dtype=torch.float32, device=X.device)
    return Xq, sx, T, r


def add_norm_quantize_act_fp8(X, R, gain, eps, bias=None, U=None, H=None):
    """h = bf16(X + R), then RMS (bias None) or layer normalisation and the quantizer.  Returns (H, Xq, sx[, T]);
    pass H=R to update the residual stream in place."""
    _rows(X, torch.bfloat16), _rows(R, torch.bfloat16), _dev(gain, torch.bfloat16, 1)
    M, K = X.shape
    if tuple(R.shape) != (M, K) or gain.shape[0] != K or (bias is not None and bias.shape[0] != K):
        raise ZqfpError(-2, "residual / gain / bias shape")
    if H is None:
        H = torch.empty((M, K), dtype=torch.bfloat16, device=X.device)
    if tuple(H.shape) != (M, K) or not H.is_contiguous():
        raise ZqfpError(-2, "H must be a dense [M, K] tensor")
    Xq, sx, T, r = _quant_outputs(X, U)
    if bias is None:
        _check(lib().zqfp_add_rmsnorm_quantize_act_fp8(_ptr(X), _ptr(R), R.stride(0), _ptr(H), _ptr(gain), float(eps), M, K,
                                                       X.stride(0), _ptr(Xq), _ptr(sx), _ptr(U), r, _ptr(T), _stream(X)))
    else:
        _dev(bias, torch.bfloat16, 1)
        _check(lib().zqfp_add_layernorm_quantize_act_fp8(_ptr(X), _ptr(R), R.stride(0), _ptr(H), _ptr(gain), _ptr(bias),
                                                         float(eps), M, K, X.stride(0), _ptr(Xq), _ptr(sx), _ptr(U), r,
                                                         _ptr(T), _stream(X)))
    return (H, Xq, sx) if U is None else (H, Xq, sx, T)


def relu_quantize_act_fp8(X, U=None):
    """ReLU fused in front of quantize_act_fp8; same outputs."""
    _rows(X, torch.bfloat16)
    M, K = X.shape
    Xq, sx, T, r = _quant_outputs(X, U)
    _check(lib().zqfp_relu_quantize_act_fp8(_ptr(X), M, K, X.stride(0), _ptr(Xq), _ptr(sx), _ptr(U), r, _ptr(T), _stream(X)))
    return (Xq, sx) if U is None else (Xq, sx, T)


def swiglu_quantize_act_fp8(G, Up, U=None, H=None):
    """bf16(silu(G) * Up) fused in front of quantize_act_fp8; same outputs.  H (dense [M, K] bf16, optional)
    receives the unquantized product."""
    _rows(G, torch.bfloat16), _rows(Up, torch.bfloat16)
    M, K = G.shape
    if tuple(Up.shape) != (M, K):
        raise ZqfpError(-2, "gate / up shapes differ")
    if H is not None and (tuple(H.shape) != (M, K) or not H.is_contiguous() or H.dtype != torch.bfloat16):
        raise ZqfpError(-2, "H must be a dense [M, K] bf16 tensor")
    Xq, sx, T, r = _quant_outputs(G, U)
    _check(lib().zqfp_swiglu_quantize_act_fp8(_ptr(G), _ptr(Up), Up.stride(0), _ptr(H), M, K, G.stride(0), _ptr(Xq), _ptr(sx),
                                              _ptr(U), r, _ptr(T), _stream(G)))
    return (Xq, sx) if U is None else (Xq, sx, T)


def packed_weight_bytes(K, N, G):
    return int(lib().zqfp_packed_weight_bytes(K, N, G))


def pack_weight_fp4(W, G, mode):
    """W [K,N] bf16 -> opaque packed blob (uint8 tensor)."""
    _dev(W, torch.bfloat16, 2)
    K, N = W.shape
    nbytes = packed_weight_bytes(K, N, G)
    if nbytes == 0:
        raise ZqfpError(-2, f"(K={K}, N={N}, G={G})")
    packed = torch.empty((nbytes,), dtype=torch.uint8, device=W.device)
    _check(lib().zqfp_pack_weight_fp4(_ptr(W), K, N, W.stride(0), G, mode, _ptr(packed), _stream(W)))
    return packed


def unpack_codes(packed, K, N, G):
    """packed blob -> codes [K,N] uint8, exps [K/G,N] uint8, colscale [N] f32."""
    _dev(packed, torch.uint8, 1)
    if packed.numel() != packed_weight_bytes(K, N, G) or packed.numel() == 0:
        raise ZqfpError(-2, f"packed blob has {packed.numel()} bytes, a blob of (K={K}, N={N}, G={G}) has "
                            f"{packed_weight_bytes(K, N, G)}")
    codes = torch.empty((K, N), dtype=torch.uint8, device=packed.device)
    exps = torch.empty((K // G, N), dtype=torch.uint8, device=packed.device)
    colscale = torch.empty((N,), dtype=torch.float32, device=packed.device)
    _check(lib().zqfp_unpack_codes(_ptr(packed), K, N, G, _ptr(codes), _ptr(exps), _ptr(colscale), _stream(packed)))
    return codes, exps, colscale


def gemm_workspace_bytes(M, K, N):
    return int(lib().zqfp_gemm_workspace_bytes(M, K, N))


def _workspace(M, K, N, device):
    n = gemm_workspace_bytes(M, K, N)
    return torch.empty((n,), dtype=torch.uint8, device=device) if n else None


def check_gemm_args(M, K, N, G, packed_numel, workspace_numel, out_shape, out_dtype, out_stride, out_is_cuda=True):
    """Host-side refusals of the GEMM wrappers, on plain numbers (the library cannot look into device memory
    without a synchronization, so sizes that it takes on trust are compared here): raises ZqfpError(-2 / -6 / -4)
    for a blob whose size is not that of (K, N, G), a workspace smaller than the query's answer, an output that
    is not a [M, N] float32 / bfloat16 tensor with contiguous rows."""
    need = packed_weight_bytes(K, N, G)
    if need == 0:
        raise ZqfpError(-2, f"(K={K}, N={N}, G={G}) outside the shape limits")
    if packed_numel != need:
        raise ZqfpError(-2, f"packed blob has {packed_numel} bytes, a blob of (K={K}, N={N}, G={G}) has {need}")
    if workspace_numel is not None and workspace_numel < gemm_workspace_bytes(M, K, N):
        raise ZqfpError(-6, f"workspace has {workspace_numel} bytes, zqfp_gemm_workspace_bytes says "
                            f"{gemm_workspace_bytes(M, K, N)}")
    if out_dtype not in (torch.float32, torch.bfloat16):
        raise ZqfpError(-4, f"output dtype {out_dtype}: float32 or bfloat16")
    if not out_is_cuda or tuple(out_shape) != (M, N) or (N > 1 and out_stride[1] != 1) or (M > 1 and out_stride[0] < N):
        raise ZqfpError(-2, f"output must be a CUDA [M={M}, N={N}] tensor with contiguous rows")


def packed_weight_check(packed, K, N, G):
    """Copies the blob's header to the host (this synchronizes) and asks the library whether it is a blob of
    (K, N, G); raises ZqfpError(-7) if not.  Meant to be called once per blob, after packing."""
    _dev(packed, torch.uint8, 1)
    if packed.numel() < BLOB_HEADER_BYTES:
        raise ZqfpError(-7, "shorter than a header")
    host = packed[:BLOB_HEADER_BYTES].cpu().numpy().tobytes()
    _check(lib().zqfp_packed_weight_check(host, K, N, G))


def _gemm_call(Xq, sx, packed, N, G, T, V, out_dtype, accum, out, workspace):
    _dev(Xq, torch.uint8, 2), _dev(sx, torch.float32, 1), _dev(packed, torch.uint8, 1)
    M, K = Xq.shape
    if sx.shape[0] != M:
        raise ZqfpError(-2, "one token scale per row of Xq")
    r = 0
    if T is not None:
        _dev(T, torch.float32, 2), _dev(V, torch.float16, 2)
        r = T.shape[1]
        if T.shape[0] != M or tuple(V.shape) != (r, N):
            raise ZqfpError(-2, "LoRC factor shapes")
    Y = torch.empty((M, N), dtype=out_dtype, device=Xq.device) if out is None else out
    no_ws = workspace is False  # run without the K-split (the library accepts NULL)
    if workspace is not None and not no_ws:
        _dev(workspace, torch.uint8, 1)
    check_gemm_args(M, K, N, G, packed.numel(), None if (workspace is None or no_ws) else workspace.numel(), Y.shape,
                    Y.dtype, Y.stride(), Y.is_cuda)
    code = OUT_F32 if Y.dtype == torch.float32 else OUT_BF16
    ws = None if no_ws else workspace if workspace is not None else _workspace(M, K, N, Xq.device)
    nws = 0 if ws is None else ws.numel()
    if r:
        _check(lib().zqfp_w4a8_gemm_lorc(_ptr(Xq), _ptr(sx), M, K, _ptr(packed), N, G, _ptr(T), _ptr(V), r, _ptr(Y),
                                         Y.stride(0), code, accum, _ptr(ws), nws, _stream(Xq)))
    else:
        _check(lib().zqfp_w4a8_gemm(_ptr(Xq), _ptr(sx), M, K, _ptr(packed), N, G, _ptr(Y), Y.stride(0), code, accum,
                                    _ptr(ws), nws, _stream(Xq)))
    return Y


STATIC_SCRATCH_BYTES = 32 << 20


def w4a8_gemm_lorc_static(Xq, sx, packed, N, G, out, T=None, V=None, accum=ACCUM_EXACT):
    """zqfp_w4a8_gemm_lorc_static: the GEMM (with LoRC when T, V are given) into the caller's `out`, partial
    results through the library's built-in scratch array; the call allocates nothing on either side."""
    _dev(Xq, torch.uint8, 2), _dev(sx, torch.float32, 1), _dev(packed, torch.uint8, 1)
    M, K = Xq.shape
    r = 0
    if T is not None:
        _dev(T, torch.float32, 2), _dev(V, torch.float16, 2)
        r = T.shape[1]
        if T.shape[0] != M or tuple(V.shape) != (r, N):
            raise ZqfpError(-2, "LoRC factor shapes")
    check_gemm_args(M, K, N, G, packed.numel(), None, out.shape, out.dtype, out.stride(), out.is_cuda)
    code = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
    _check(lib().zqfp_w4a8_gemm_lorc_static(_ptr(Xq), _ptr(sx), M, K, _ptr(packed), N, G, _ptr(T), _ptr(V), r, _ptr(out),
                                            out.stride(0), code, accum, _stream(Xq)))
    return out


def w4a8_gemm(Xq, sx, packed, N, G, out_dtype=torch.float32, accum=ACCUM_EXACT, out=None, workspace=None):
    """Y [M,N] = (sx c) * (Xq . Wq).  workspace: None = allocated here when the shape needs one, a uint8 tensor of
    at least gemm_workspace_bytes(M, K, N) bytes, or False = none (K is then not split)."""
    return _gemm_call(Xq, sx, packed, N, G, None, None, out_dtype, accum, out, workspace)


def w4a8_gemm_lorc(Xq, sx, packed, N, G, T, V, out_dtype=torch.float32, accum=ACCUM_EXACT, out=None, workspace=None):
    """Y [M,N] = (sx c) * (Xq . Wq) + T . V."""
    if T is None or V is None:
        raise ZqfpError(-1, "T and V are required")
    return _gemm_call(Xq, sx, packed, N, G, T, V, out_dtype, accum, out, workspace)


def linear_is_fused(M, K, r=0):
    """Whether w4a8_linear runs as one kernel (the decode GEMM quantizing in its prologue)."""
    return 1 <= M <= 16 and K <= 4096 and r == 0


def w4a8_linear(X, packed, N, G, U=None, V=None, out_dtype=torch.float32, accum=ACCUM_EXACT, out=None, want_codes=False):
    """Y = Q8(X) . Q4(W) (+ (X.U).V) from bfloat16 X in one call (one kernel for at most 16 tokens, K <= 4096 and no
    LoRC).  Returns Y, or (Y, Xq, sx) with want_codes."""
    _rows(X, torch.bfloat16), _dev(packed, torch.uint8, 1)
    M, K = X.shape
    r = 0
    if U is not None:
        _dev(U, torch.float16, 2), _dev(V, torch.float16, 2)
        r = U.shape[1]
        if U.shape[0] != K or tuple(V.shape) != (r, N):
            raise ZqfpError(-2, "LoRC factor shapes")
    Y = torch.empty((M, N), dtype=out_dtype, device=X.device) if out is None else out
    check_gemm_args(M, K, N, G, packed.numel(), None, Y.shape, Y.dtype, Y.stride(), Y.is_cuda)
    fused = linear_is_fused(M, K, r)
    Xq = sx = T = None
    if want_codes or not fused:
        Xq = torch.empty((M, K), dtype=torch.uint8, device=X.device)
        sx = torch.empty((M,), dtype=torch.float32, device=X.device)
    if r:
        T = torch.empty((M, r), dtype=torch.float32, device=X.device)
    ws = None if fused else _workspace(M, K, N, X.device)
    code = OUT_F32 if Y.dtype == torch.float32 else OUT_BF16
    _check(lib().zqfp_w4a8_linear(_ptr(X), X.stride(0), M, K, _ptr(packed), N, G, _ptr(U), _ptr(V), r, _ptr(Xq), _ptr(sx),
                                  _ptr(T), _ptr(Y), Y.stride(0), code, accum, _ptr(ws), 0 if ws is None else ws.numel(),
                                  _stream(X)))
    return (Y, Xq, sx) if want_codes else Y


def pack_weight_fp8(W, G, mode):
    """W [K,N] bf16 -> packed blob of E4M3 weights with power-of-two group scales (W8A8; G a multiple of 128)."""
    _rows(W, torch.bfloat16)
    K, N = W.shape
    nbytes = int(lib().zqfp_packed_weight_fp8_bytes(K, N, G))
    if nbytes == 0:
        raise ZqfpError(-2, f"(K={K}, N={N}, G={G})")
    packed = torch.empty((nbytes,), dtype=torch.uint8, device=W.device)
    _check(lib().zqfp_pack_weight_fp8(_ptr(W), K, N, W.stride(0), G, mode, _ptr(packed), _stream(W)))
    return packed


def unpack_codes_fp8(packed, K, N, G):
    """packed E4M3 blob -> codes [K,N] uint8 (E4M3), exps [K/G,N] uint8, colscale [N] f32."""
    _dev(packed, torch.uint8, 1)
    if packed.numel() != int(lib().zqfp_packed_weight_fp8_bytes(K, N, G)) or packed.numel() == 0:
        raise ZqfpError(-2, "blob size is not that of an E4M3 blob of (K, N, G)")
    codes = torch.empty((K, N), dtype=torch.uint8, device=packed.device)
    exps = torch.empty((K // G, N), dtype=torch.uint8, device=packed.device)
    colscale = torch.empty((N,), dtype=torch.float32, device=packed.device)
    _check(lib().zqfp_unpack_codes_fp8(_ptr(packed), K, N, G, _ptr(codes), _ptr(exps), _ptr(colscale), _stream(packed)))
    return codes, exps, colscale


def w8a8_gemm(Xq, sx, packed, N, G, T=None, V=None, out_dtype=torch.float32, accum=ACCUM_EXACT, out=None):
    """Y [M,N] = (sx c) * (Xq . Wq8) (+ T . V): E4M3 weights."""
    _dev(Xq, torch.uint8, 2), _dev(sx, torch.float32, 1), _dev(packed, torch.uint8, 1)
    M, K = Xq.shape
    if packed.numel() != int(lib().zqfp_packed_weight_fp8_bytes(K, N, G)) or packed.numel() == 0 or sx.shape[0] != M:
        raise ZqfpError(-2, "blob size is not that of an E4M3 blob of (K, N, G)")
    r = 0
    if T is not None:
        _dev(T, torch.float32, 2), _dev(V, torch.float16, 2)
        r = T.shape[1]
        if T.shape[0] != M or tuple(V.shape) != (r, N):
            raise ZqfpError(-2, "LoRC factor shapes")
    Y = torch.empty((M, N), dtype=out_dtype, device=Xq.device) if out is None else out
    if Y.dtype not in (torch.float32, torch.bfloat16) or tuple(Y.shape) != (M, N) or not Y.is_cuda or (N > 1 and Y.stride(1) != 1):
        raise ZqfpError(-2, "output must be a CUDA [M, N] float32 / bfloat16 tensor with contiguous rows")
    code = OUT_F32 if Y.dtype == torch.float32 else OUT_BF16
    _check(lib().zqfp_w8a8_gemm(_ptr(Xq), _ptr(sx), M, K, _ptr(packed), N, G, _ptr(T), _ptr(V), r, _ptr(Y), Y.stride(0),
                                code, accum, _stream(Xq)))
    return Y


def gptq_pack_weight_fp4(W, Hinv_u, G, mode):
    """GPTQ on the E2M1 grid: W [K,N] bf16, Hinv_u [K,K] f32 (upper Cholesky factor of the inverse Hessian)
    -> the packed blob (same format as pack_weight_fp4)."""
    _rows(W, torch.bfloat16), _dev(Hinv_u, torch.float32, 2)
    K, N = W.shape
    if tuple(Hinv_u.shape) != (K, K):
        raise ZqfpError(-2, "Hinv_u must be [K, K]")
    nbytes = packed_weight_bytes(K, N, G)
    wsb = int(lib().zqfp_gptq_workspace_bytes(K, N, G))
    if nbytes == 0 or wsb == 0:
        raise ZqfpError(-2, "shape / group size")
    packed = torch.empty((nbytes,), dtype=torch.uint8, device=W.device)
    ws = torch.empty((wsb + 256,), dtype=torch.uint8, device=W.device)
    off = (-ws.data_ptr()) % 256
    _check(lib().zqfp_gptq_pack_weight_fp4(_ptr(W), K, N, W.stride(0), _ptr(Hinv_u), G, mode, _ptr(packed),
                                           ws.data_ptr() + off, _stream(W)))
    return packed


def lorc_factorize(W, packed, G, r, Omega, power_iters=2):
    """LoRC factors of W minus what `packed` de-quantizes to: U [K,r] fp16, V [r,N] fp16, sigma [r] f32.
    Omega [N, r+8] float32 holds the caller's standard normal draws."""
    _rows(W, torch.bfloat16), _dev(packed, torch.uint8, 1), _dev(Omega, torch.float32, 2)
    K, N = W.shape
    if tuple(Omega.shape) != (N, r + 8):
        raise ZqfpError(-2, "Omega must be [N, r + 8]")
    U = torch.empty((K, r), dtype=torch.float16, device=W.device)
    V = torch.empty((r, N), dtype=torch.float16, device=W.device)
    sigma = torch.empty((r,), dtype=torch.float32, device=W.device)
    ws = torch.empty((int(lib().zqfp_lorc_workspace_bytes(K, N, r)) + 256,), dtype=torch.uint8, device=W.device)
    off = (-ws.data_ptr()) % 256
    _check(lib().zqfp_lorc_factorize(_ptr(W), K, N, W.stride(0), _ptr(packed), G, r, _ptr(Omega), power_iters, _ptr(U),
                                     _ptr(V), _ptr(sigma), ws.data_ptr() + off, _stream(W)))
    return U, V, sigma


def probe_stream_read(src, sink, workgroups):
    """Enqueue a plain streaming read of the uint8 tensor `src` (measurement probe; the caller times it)."""
    _dev(src, torch.uint8, 1), _dev(sink, torch.int32, 1)
    if sink.numel() < workgroups:
        raise ZqfpError(-2, "sink smaller than the workgroup count")
    _check(lib().zqfp_probe_stream_read(_ptr(src), src.numel(), _ptr(sink), workgroups, _stream(src)))


def probe_mfma(operands, sink, iters, workgroups):
    """Enqueue `iters` rounds of 32 FP8 x FP4 matrix instructions per wave on `workgroups` workgroups of 8
    waves (measurement probe; the caller times it).  Returns the floating-point operations enqueued."""
    _dev(operands, torch.int32, 1), _dev(sink, torch.float32, 1)
    if operands.numel() < 1024 or sink.numel() < 512 * workgroups:
        raise ZqfpError(-2, "probe buffers too small")
    _check(lib().zqfp_probe_mfma(_ptr(operands), _ptr(sink), iters, workgroups, _stream(operands)))
    return 2.0 * 16 * 16 * 128 * 32 * 8 * iters * workgroups


def probe_force_tile_plan(bm=0, bn=0, ksplit=0, kg=1):
    """Tuning hook: fix tile shape, wave groups and number of K slices of the tiled GEMM for the calls that follow
    (0, 0, 0 = plan automatically again)."""
    _check(lib().zqfp_probe_force_tile_plan(bm, bn, ksplit, kg if bm else 0))


def probe_force_decode_waves(nw=8):
    """Tuning hook: 8 or 16 waves per workgroup of the decode GEMM (K <= 4096)."""
    _check(lib().zqfp_probe_force_decode_waves(nw))
