"""ctypes front end of the CPU oracle (``zqfp_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg.  Nothing here touches the HIP library and the
HIP package never imports this module.  All arithmetic lives in the C file;
this module only marshals numpy arrays.

Array conventions (all C-contiguous numpy arrays):
  X      uint16 [M, K]   bfloat16 bit patterns
  W      uint16 [K, N]   bfloat16 bit patterns (input feature k, output channel n)
  U, V   uint16 [K, r], [r, N]  binary16 bit patterns
  Xq     uint8  [M, K]   E4M3 codes;  sx float32 [M]
  codes  uint8  [K, N]   one E2M1 code per byte
  exps   uint8  [K/G, N] exponent byte (n + 127 for a scale c[n] * 2^n)
  c      float32 [N]     per-output-channel real scale (1 under M1)
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zqfp_oracle.c")
_LIB = os.path.join(_HERE, "libzqfp_oracle.so")

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
          "-Wall", "-Wextra", "-shared", "-fPIC"]


def build_oracle():
    """Compile the oracle with gcc (always recompiles)."""
    subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


def build_oracle_sanitized(out, cc="/opt/rocm/llvm/bin/clang"):
    """The same source under AddressSanitizer + UndefinedBehaviorSanitizer, for the test that re-runs the pins on
    it (clang, so that one sanitizer runtime serves this library and the sanitized host build of the HIP library;
    single-threaded: the OpenMP pragmas are ignored).  The process that loads it needs the runtime preloaded."""
    flags = [f for f in CFLAGS if f not in ("-fopenmp", "-O2")]
    subprocess.check_call([cc, "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-Wno-unknown-pragmas", "-Wno-source-uses-openmp", *flags,
                           "-o", out, _SRC, "-lm"])
    return out


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = os.environ.get("ZQFP_ORACLE_LIB")  # another build of this same source (the sanitizer run sets it)
        if not path:
            if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
                build_oracle()
            path = _LIB
        L = ctypes.CDLL(path)
        c = ctypes
        p = c.c_void_p
        L.orc_e4m3_decode.restype = c.c_double
        L.orc_e4m3_decode.argtypes = [c.c_uint8]
        L.orc_e5m2_decode.restype = c.c_double
        L.orc_e5m2_decode.argtypes = [c.c_uint8]
        L.orc_e2m1_decode.restype = c.c_double
        L.orc_e2m1_decode.argtypes = [c.c_uint8]
        L.orc_e4m3_encode.restype = c.c_uint8
        L.orc_e4m3_encode.argtypes = [c.c_float]
        L.orc_e2m1_encode.restype = c.c_uint8
        L.orc_e2m1_encode.argtypes = [c.c_double]
        L.orc_fp4_to_fp8_shift.restype = c.c_int
        L.orc_fp4_to_fp8_shift.argtypes = [c.c_uint8, c.c_int, c.c_int, c.POINTER(c.c_uint8)]
        L.orc_quantize_act.restype = None
        L.orc_quantize_act.argtypes = [p, c.c_int64, c.c_int64, c.c_int64, p, p]
        L.orc_pack_weight.restype = c.c_int64
        L.orc_pack_weight.argtypes = [p, c.c_int64, c.c_int64, c.c_int64, c.c_int, c.c_int, p, p, p]
        L.orc_gemm.restype = None
        L.orc_gemm.argtypes = [p, p, c.c_int64, c.c_int64, p, p, p, c.c_int64, c.c_int,
                               p, p, c.c_int, p, p, c.c_int]
        L.orc_gemm_samples.restype = None
        L.orc_gemm_samples.argtypes = [p, p, c.c_int64, c.c_int64, p, p, p, c.c_int64, c.c_int,
                                       p, p, c.c_int, p, p, c.c_int64, p, p]
        L.orc_pack_weight_fp8.restype = c.c_int64
        L.orc_pack_weight_fp8.argtypes = [p, c.c_int64, c.c_int64, c.c_int64, c.c_int, c.c_int, p, p, p, p]
        L.orc_gemm_w8_samples.restype = None
        L.orc_gemm_w8_samples.argtypes = [p, p, c.c_int64, c.c_int64, p, p, p, p, c.c_int64, c.c_int, p, p, c.c_int,
                                          p, p, c.c_int64, p, p]
        L.orc_lorc_left.restype = None
        L.orc_lorc_left.argtypes = [p, c.c_int64, c.c_int64, c.c_int64, p, c.c_int, p, p]
        L.orc_rmsnorm_bf16.restype = None
        L.orc_rmsnorm_bf16.argtypes = [p, c.c_int64, c.c_int64, c.c_int64, p, c.c_float, p]
        L.orc_add_bf16.restype = None
        L.orc_add_bf16.argtypes = [p, p, c.c_int64, c.c_int64, c.c_int64, c.c_int64, p]
        L.orc_relu_bf16.restype = None
        L.orc_relu_bf16.argtypes = [p, c.c_int64, c.c_int64, c.c_int64, p]
        L.orc_swiglu_bf16.restype = None
        L.orc_swiglu_bf16.argtypes = [p, p, c.c_int64, c.c_int64, c.c_int64, c.c_int64, p]
        L.orc_layernorm_bf16.restype = None
        L.orc_layernorm_bf16.argtypes = [p, c.c_int64, c.c_int64, c.c_int64, p, p, c.c_float, p]
        L.orc_max_threads.restype = c.c_int
        L.orc_max_threads.argtypes = []
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, ndim):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.ndim == ndim, (a.dtype, a.shape)
    assert a.flags["C_CONTIGUOUS"]
    return a


# ---- scalar format functions -------------------------------------------------
def e4m3_decode(code):
    return lib().orc_e4m3_decode(int(code))


def e5m2_decode(code):
    return lib().orc_e5m2_decode(int(code))


def e2m1_decode(code):
    return lib().orc_e2m1_decode(int(code))


def e4m3_encode(y):
    return lib().orc_e4m3_encode(float(np.float32(y)))


def e2m1_encode(y):
    return lib().orc_e2m1_encode(float(y))


def fp4_to_fp8_shift(code4, n, container):
    """container: 'e4m3' or 'e5m2'.  Returns the FP8 code or None if the shifted
    exponent is outside the container's normal range."""
    out = ctypes.c_uint8(0)
    rc = lib().orc_fp4_to_fp8_shift(int(code4), int(n), 1 if container == "e5m2" else 0,
                                    ctypes.byref(out))
    return None if rc else out.value


# ---- array functions -----------------------------------------------------------
def quantize_act(X):
    _chk(X, np.uint16, 2)
    M, K = X.shape
    Xq = np.empty((M, K), np.uint8)
    sx = np.empty((M,), np.float32)
    lib().orc_quantize_act(_ptr(X), M, K, K, _ptr(Xq), _ptr(sx))
    return Xq, sx


def rmsnorm_bf16(X, g, eps):
    """RMS normalisation of bf16 rows (bits) with bf16 gain g, result rounded to bf16 (bits)."""
    _chk(X, np.uint16, 2), _chk(g, np.uint16, 1)
    M, K = X.shape
    if g.shape[0] != K or not eps > 0:
        raise ValueError("gain length / eps")
    Y = np.empty((M, K), np.uint16)
    lib().orc_rmsnorm_bf16(_ptr(X), M, K, K, _ptr(g), float(eps), _ptr(Y))
    return Y


def layernorm_bf16(X, g, b, eps):
    """Layer normalisation of bf16 rows (bits) with bf16 gain g and bias b, result rounded to bf16 (bits)."""
    _chk(X, np.uint16, 2), _chk(g, np.uint16, 1), _chk(b, np.uint16, 1)
    M, K = X.shape
    if g.shape[0] != K or b.shape[0] != K or not eps > 0:
        raise ValueError("gain / bias length or eps")
    Y = np.empty((M, K), np.uint16)
    lib().orc_layernorm_bf16(_ptr(X), M, K, K, _ptr(g), _ptr(b), float(eps), _ptr(Y))
    return Y


def add_bf16(X, R):
    """h = bf16(x + r) on bf16 bits (one binary32 addition, round to nearest even)."""
    _chk(X, np.uint16, 2), _chk(R, np.uint16, 2)
    if X.shape != R.shape:
        raise ValueError("shapes differ")
    M, K = X.shape
    H = np.empty((M, K), np.uint16)
    lib().orc_add_bf16(_ptr(X), _ptr(R), M, K, K, K, _ptr(H))
    return H


def relu_bf16(X):
    """y = x if x > 0 else +0, on bf16 bits."""
    _chk(X, np.uint16, 2)
    M, K = X.shape
    Y = np.empty((M, K), np.uint16)
    lib().orc_relu_bf16(_ptr(X), M, K, K, _ptr(Y))
    return Y


def swiglu_bf16(G, U):
    """y = bf16(silu(g) * u) on bf16 bits, evaluated in binary64."""
    _chk(G, np.uint16, 2), _chk(U, np.uint16, 2)
    if G.shape != U.shape:
        raise ValueError("shapes differ")
    M, K = G.shape
    Y = np.empty((M, K), np.uint16)
    lib().orc_swiglu_bf16(_ptr(G), _ptr(U), M, K, K, K, _ptr(Y))
    return Y


def pack_weight(W, G, mode):
    """mode 1 = M1, 2 = M2.  Returns codes, exps, c, number of saturated elements."""
    _chk(W, np.uint16, 2)
    K, N = W.shape
    assert K % G == 0 and mode in (1, 2)
    codes = np.empty((K, N), np.uint8)
    exps = np.empty((K // G, N), np.uint8)
    c = np.empty((N,), np.float32)
    clipped = lib().orc_pack_weight(_ptr(W), K, N, N, G, mode, _ptr(codes), _ptr(exps), _ptr(c))
    return codes, exps, c, int(clipped)


def pack_weight_fp8(W, G, mode):
    """E4M3 weights (W8A8).  mode 0 = real group scales (the paper's W8A8 rows), 1 = M1, 2 = M2.
    Returns codes [K,N] (E4M3), exps [K/G,N], c [N], gscale [K/G,N] (each group's whole scale), saturated count."""
    _chk(W, np.uint16, 2)
    K, N = W.shape
    assert K % G == 0 and mode in (0, 1, 2)
    codes = np.empty((K, N), np.uint8)
    exps = np.empty((K // G, N), np.uint8)
    c = np.empty((N,), np.float32)
    gscale = np.empty((K // G, N), np.float32)
    clipped = lib().orc_pack_weight_fp8(_ptr(W), K, N, N, G, mode, _ptr(codes), _ptr(exps), _ptr(c), _ptr(gscale))
    return codes, exps, c, gscale, int(clipped)


def gemm_w8(Xq, sx, codes, exps, c, G, gscale=None, T=None, V=None, ms=None, ns=None):
    """W8A8 layer: Y (and Sabs) for the sampled outputs (ms, ns), or for the whole [M,N] matrix when none are given.
    gscale: real group scales (mode 0), else the power-of-two exponents `exps` are used."""
    _chk(Xq, np.uint8, 2), _chk(sx, np.float32, 1), _chk(codes, np.uint8, 2), _chk(exps, np.uint8, 2), _chk(c, np.float32, 1)
    M, K = Xq.shape
    N = codes.shape[1]
    assert codes.shape[0] == K and exps.shape == (K // G, N)
    T, V, r = _lorc_args(T, V, M, N)
    full = ms is None
    if full:
        ms, ns = np.divmod(np.arange(M * N, dtype=np.int64), N)
    ms = np.ascontiguousarray(ms, np.int64)
    ns = np.ascontiguousarray(ns, np.int64)
    if gscale is not None:
        _chk(gscale, np.float32, 2)
    Y = np.empty(ms.shape, np.float32)
    Sabs = np.empty(ms.shape, np.float64)
    lib().orc_gemm_w8_samples(_ptr(Xq), _ptr(sx), M, K, _ptr(codes), _ptr(exps), _ptr(c), _ptr(gscale), N, G,
                              _ptr(T), _ptr(V), r, _ptr(ms), _ptr(ns), ms.size, _ptr(Y), _ptr(Sabs))
    return (Y.reshape(M, N), Sabs.reshape(M, N)) if full else (Y, Sabs)


def _lorc_args(T, V, M, N):
    if T is None:
        return None, None, 0
    _chk(T, np.float32, 2)
    _chk(V, np.uint16, 2)
    r = T.shape[1]
    assert T.shape[0] == M and V.shape == (r, N)
    return T, V, r


def gemm(Xq, sx, codes, exps, c, G, T=None, V=None, want_abs=True, threads=0):
    """Y [M,N] float32 (and Sabs [M,N] float64, the sum of absolute terms)."""
    _chk(Xq, np.uint8, 2), _chk(sx, np.float32, 1), _chk(codes, np.uint8, 2)
    _chk(exps, np.uint8, 2), _chk(c, np.float32, 1)
    M, K = Xq.shape
    N = codes.shape[1]
    assert codes.shape[0] == K and exps.shape == (K // G, N) and c.shape == (N,)
    T, V, r = _lorc_args(T, V, M, N)
    Y = np.empty((M, N), np.float32)
    Sabs = np.empty((M, N), np.float64) if want_abs else None
    lib().orc_gemm(_ptr(Xq), _ptr(sx), M, K, _ptr(codes), _ptr(exps), _ptr(c), N, G,
                   _ptr(T), _ptr(V), r, _ptr(Y), _ptr(Sabs), int(threads))
    return (Y, Sabs) if want_abs else Y


def gemm_samples(Xq, sx, codes, exps, c, G, ms, ns, T=None, V=None):
    _chk(Xq, np.uint8, 2), _chk(sx, np.float32, 1), _chk(codes, np.uint8, 2)
    M, K = Xq.shape
    N = codes.shape[1]
    T, V, r = _lorc_args(T, V, M, N)
    ms = np.ascontiguousarray(ms, np.int64)
    ns = np.ascontiguousarray(ns, np.int64)
    Y = np.empty(ms.shape, np.float32)
    Sabs = np.empty(ms.shape, np.float64)
    lib().orc_gemm_samples(_ptr(Xq), _ptr(sx), M, K, _ptr(codes), _ptr(exps), _ptr(c), N, G,
                           _ptr(T), _ptr(V), r, _ptr(ms), _ptr(ns), ms.size, _ptr(Y), _ptr(Sabs))
    return Y, Sabs


def lorc_left(X, U):
    """T = X.U (float32 [M,r]) and Tabs = sum |x.u| (float64 [M,r])."""
    _chk(X, np.uint16, 2), _chk(U, np.uint16, 2)
    M, K = X.shape
    r = U.shape[1]
    assert U.shape[0] == K
    T = np.empty((M, r), np.float32)
    Tabs = np.empty((M, r), np.float64)
    lib().orc_lorc_left(_ptr(X), M, K, K, _ptr(U), r, _ptr(T), _ptr(Tabs))
    return T, Tabs


def max_threads():
    return lib().orc_max_threads()


# ---- LoRC factorisation (offline step; plain numpy in float64) -------------------
def _bf16_bits_to_f64(bits):
    return (np.asarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def dequant_weight(codes, exps, c, G):
    """The quantized weight the GEMM multiplies with, W^[k,n] = c[n] * 2^(exps[k/G,n] - 127) * e2m1(codes[k,n])
    (Section 3, "Casting the FP4 to FP8": S = 2^n, methods M1 / M2), as float64 [K,N]."""
    _chk(codes, np.uint8, 2), _chk(exps, np.uint8, 2), _chk(c, np.float32, 1)
    K, N = codes.shape
    table = np.array([e2m1_decode(q) for q in range(16)], np.float64)
    scale = np.exp2(exps.astype(np.float64) - 127.0)           # [K/G, N]
    return table[codes] * np.repeat(scale, G, axis=0) * c.astype(np.float64)[None, :]


def lorc_factors(W, codes, exps, c, G, r):
    """LoRC (Section 3): singular value decomposition of the error matrix E = W - W^ (original minus
    quantized weight), E = P diag(s) Q^T; the two low-rank matrices are the r leading singular triplets
    with the singular values shared evenly, U = P_r diag(s_r)^(1/2), V = diag(s_r)^(1/2) Q_r^T, so that U V is the
    best rank-r approximation of E.  W: bf16 bits [K,N].  Returns U [K,r], V [r,N], s [min(K,N)] (float64)
    and E."""
    _chk(W, np.uint16, 2)
    E = _bf16_bits_to_f64(W) - dequant_weight(codes, exps, c, G)
    P, s, Qt = np.linalg.svd(E, full_matrices=False)
    root = np.sqrt(s[:r])
    return P[:, :r] * root[None, :], root[:, None] * Qt[:r], s, E


# ---- GPTQ with the E2M1 grid and power-of-two scales (offline step; plain numpy in float64) -------
_E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def e2m1_encode_array(y):
    """Nearest E2M1 code of every element (ties to the even code, saturating at 6, sign bit copied from y):
    the array form of orc_e2m1_encode, written out as the definition."""
    y = np.asarray(y, np.float64)
    a = np.abs(y)
    d = np.abs(a[..., None] - _E2M1_GRID)                 # distance to the eight magnitudes
    best = d.min(axis=-1)
    cand = d == best[..., None]                           # one or (on a tie) two neighbouring codes
    lo = cand.argmax(axis=-1)
    hi = 7 - cand[..., ::-1].argmax(axis=-1)
    mag = np.where(lo % 2 == 0, lo, hi)                   # the even one of the two
    return (mag | (np.signbit(y).astype(np.int64) << 3)).astype(np.uint8)


def gptq_fp4(W, Hinv_u, G, mode):
    """GPTQ (the weight quantizer the paper runs, Section 3 and Appendix A) on the E2M1 grid with the
    power-of-two scales of "Casting the FP4 to FP8" (mode 1 = M1, 2 = M2).

    W: bf16 bits [K, N] (input channels x output channels).  Hinv_u: the upper Cholesky factor of the inverse
    Hessian, inv(H) = Hinv_u^T Hinv_u, float64 [K, K].  Input channels are quantized one at a time, in order;
    after channel k its scaled error is pushed onto the channels not yet quantized:
        q_k = S * e2m1(w_k / S);   err = (w_k - q_k) / Hinv_u[k, k];   w_j -= Hinv_u[k, j] * err  for j > k.
    A group's scale is fixed when its first channel is reached, from the weights as they stand then
    (M1: S = 2^n, least n with amax <= 6 * 2^n; M2: S = c * 2^-k with c = column absmax of the ORIGINAL W / 6,
    least k >= 0 with amax_max <= amax * 2^k, at most 15).  The value that is encoded is w / S; under M2 it is
    formed as the plain packer forms it, fl32(fl32(w) / c) * 2^k: one binary32 division, then an exact shift.
    Returns codes [K,N] u8, exps [K/G,N] u8, c [N] f32 and the final de-quantized weight [K,N] f64."""
    _chk(W, np.uint16, 2)
    K, N = W.shape
    Wf = _bf16_bits_to_f64(W).copy()
    codes = np.zeros((K, N), np.uint8)
    exps = np.zeros((K // G, N), np.uint8)
    Q = np.zeros((K, N))
    c = np.ones(N, np.float32)
    colmax = np.abs(Wf).max(axis=0)
    if mode == 2:
        c = np.where(colmax > 0, (colmax.astype(np.float32) / np.float32(6.0)), np.float32(1.0)).astype(np.float32)
    S = np.ones(N)
    for k in range(K):
        if k % G == 0:
            amax = np.abs(Wf[k:k + G]).max(axis=0)
            if mode == 1:
                n = np.zeros(N, np.int64)
                nz = amax > 0
                n[nz] = np.ceil(np.log2(amax[nz] / 6.0)).astype(np.int64)
                # the logarithm can be off by one at exact powers of two: settle it by the definition
                n[nz & (amax > 6.0 * np.exp2(n))] += 1
                n[nz & (amax <= 6.0 * np.exp2(n - 1.0))] -= 1
                n = np.clip(n, -126, 127)
                exps[k // G] = (n + 127).astype(np.uint8)
                S = np.exp2(n.astype(np.float64))
            else:
                kg = np.full(N, 15, np.int64)
                nz = amax > 0
                for t in range(14, -1, -1):
                    kg[nz & (colmax <= amax * 2.0 ** t)] = t
                exps[k // G] = (127 - kg).astype(np.uint8)
                S = c.astype(np.float64) * np.exp2(-kg.astype(np.float64))
        if mode == 1:
            y = Wf[k] / S                                   # a power of two: exact
        else:
            # the plain packer's rule (orc_pack_weight): the working weight rounded to binary32, ONE binary32
            # division by the column scale, then the exact shift by 2^k -- so that H = I gives the packer's codes
            y = (Wf[k].astype(np.float32) / c).astype(np.float64) * np.exp2(kg.astype(np.float64))
        codes[k] = e2m1_encode_array(y)
        Q[k] = np.where(codes[k] & 8, -1.0, 1.0) * _E2M1_GRID[codes[k] & 7] * S
        err = (Wf[k] - Q[k]) / Hinv_u[k, k]
        if k + 1 < K:
            Wf[k + 1:] -= np.outer(Hinv_u[k, k + 1:], err)
    return codes, exps, c, Q


# ---- format ablation helpers (Appendix A, Table A.1: E2M1 against E3M0 weights; Section 4: E4M3 against E5M2) ----
def format_values(name):
    """Non-negative values of a small floating-point format, ascending, index = magnitude code.
    e2m1, e4m3, e5m2: decoded by the C oracle.  e3m0: sign, three exponent bits (bias 3), no mantissa bit --
    0, then 2^(E - 3) for E = 1..7 (the paper's alternative 4-bit format; it names the format only, the bias is
    immaterial under an absmax scale)."""
    if name == "e2m1":
        return np.array([e2m1_decode(q) for q in range(8)])
    if name == "e3m0":
        return np.array([0.0] + [2.0 ** (e - 3) for e in range(1, 8)])
    if name == "e4m3":
        return np.array([e4m3_decode(q) for q in range(0x7F)])          # 0x7F is NaN
    if name == "e5m2":
        return np.array([e5m2_decode(q) for q in range(0x7C)])          # 0x7C.. are infinity / NaN
    raise ValueError(name)


def quantize_to_format(y, name):
    """Nearest value of the format for every element of y (ties to the even magnitude code, saturating at the
    largest value, sign kept): the definition written out over the value table.  Returns the values (float64)."""
    tab = format_values(name)
    y = np.asarray(y, np.float64)
    a = np.minimum(np.abs(y), tab[-1])
    hi = np.clip(np.searchsorted(tab, a, side="left"), 1, len(tab) - 1)
    lo = hi - 1
    dl, dh = a - tab[lo], tab[hi] - a
    pick_hi = (dh < dl) | ((dh == dl) & (hi % 2 == 0))
    return np.copysign(np.where(pick_hi, tab[hi], tab[lo]), y)
