// C ABI of libzqfp (declared in include/zqfp.h): argument checks and kernel
// dispatch.  No call here synchronizes, allocates or frees device memory.
#include "../../include/zqfp.h"
#include "../../include/zqfp_probe.h"

#include <cstring>
#include <mutex>
#include <string>

#include "zqfp_internal.h"

namespace {

thread_local std::string g_last_error;

int hip_fail(hipError_t e)
{
    g_last_error = hipGetErrorString(e);
    return ZQFP_E_HIP;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// bytes of float32 partial results the GEMM of (M, K, N) hands through a workspace (0: none)
size_t gemm_workspace_need(int64_t M, int64_t K, int64_t N)
{
    if (M <= 0 || N <= 0 || K <= 0 || K % 128 != 0) return 0;
    const int64_t Np = (N + 15) / 16 * 16;
    if (M <= 16) {  // decode form: K beyond 64 k-tiles is served in chunks
        const zqfp::DecodePlan d = zqfp::plan_decode(K / 128);
        return d.chunks > 1 ? (size_t)d.chunks * (size_t)M * (size_t)Np * sizeof(float) : 0;
    }
    if (N < 64) return 0;
    const zqfp::TilePlan p = zqfp::effective_tile_plan(M, Np, K / 128);
    return p.ksplit > 1 ? (size_t)p.ksplit * (size_t)M * (size_t)Np * sizeof(float) : 0;
}

int gemm_common(const uint8_t* Xq, const float* sx, int64_t M, int64_t K, const void* packed, int64_t N, int G,
                const float* T, const void* V, int r, void* Y, int64_t ldy, int out_dtype, int accum, void* workspace,
                size_t workspace_bytes, void* stream)
{
    if (M < 0 || N < 0 || r < 0 || r > 64) return ZQFP_E_SHAPE;
    zqfp::BlobLayout L;
    if (!zqfp::make_layout(K, N, G, &L)) return ZQFP_E_SHAPE;
    if (out_dtype != ZQFP_OUT_F32 && out_dtype != ZQFP_OUT_BF16) return ZQFP_E_MODE;
    if (accum != ZQFP_ACCUM_EXACT && accum != ZQFP_ACCUM_FAST) return ZQFP_E_MODE;
    if (M == 0 || N == 0) return ZQFP_OK;
    if (!Xq || !sx || !packed || !Y) return ZQFP_E_NULL;
    if (r > 0 && (!T || !V)) return ZQFP_E_NULL;
    if (ldy < N) return ZQFP_E_SHAPE;
    if (workspace != nullptr && workspace_bytes < gemm_workspace_need(M, K, N)) {
        g_last_error = "workspace smaller than zqfp_gemm_workspace_bytes(M, K, N)";
        return ZQFP_E_WORKSPACE;
    }
    if (!aligned16(Xq) || !aligned16(Y) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(packed) & 255u) != 0)
        return ZQFP_E_ALIGN;
    zqfp::Lorc lorc{r > 0 ? T : nullptr, r > 0 ? static_cast<const uint16_t*>(V) : nullptr, r};
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint8_t* blob = static_cast<const uint8_t*>(packed);
    hipError_t e = zqfp::gemm_decode_supported(M, L, workspace)
                       ? zqfp::launch_gemm_decode(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, accum, workspace, s)
                   : zqfp::gemm_tile_supported(M, L)
                       ? zqfp::launch_gemm_tile(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, accum, workspace, s)
                       : zqfp::launch_gemm_stream(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, accum, s);
    return e == hipSuccess ? ZQFP_OK : hip_fail(e);
}

// argument checks shared by the quantizer entry points; `normalised` rows are limited to what registers hold
int quantize_common(const void* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, float* sx, const void* U, int r,
                           float* T, const zqfp::Producer& pr, void* stream)
{
    if (M < 0 || K <= 0 || K % 128 != 0 || ldx < K || r < 0 || r > 64) return ZQFP_E_SHAPE;
    if (pr.kind != 0 && K > 32768) return ZQFP_E_SHAPE;
    if ((pr.kind == 1 || pr.kind == 2) && !(pr.eps > 0.0f)) return ZQFP_E_SHAPE;
    if (pr.other != nullptr && pr.ld_other < K) return ZQFP_E_SHAPE;
    if (M == 0) return ZQFP_OK;
    if (!X || !Xq || !sx) return ZQFP_E_NULL;
    if ((U != nullptr) != (r > 0) || (r > 0 && !T)) return ZQFP_E_NULL;
    if ((pr.kind == 1 || pr.kind == 2) && !pr.gain) return ZQFP_E_NULL;
    if (pr.kind == 2 && !pr.bias) return ZQFP_E_NULL;
    if (pr.kind == 4 && !pr.other) return ZQFP_E_NULL;
    if ((pr.kind == 1 || pr.kind == 2) && pr.other != nullptr && !pr.H) return ZQFP_E_NULL;
    if (!aligned16(X) || !aligned16(Xq) || (ldx % 8) != 0 || (r > 0 && !aligned16(U))) return ZQFP_E_ALIGN;
    if (!aligned16(pr.gain) || !aligned16(pr.bias) || !aligned16(pr.other) || !aligned16(pr.H) || (pr.ld_other % 8) != 0)
        return ZQFP_E_ALIGN;
    hipError_t e = zqfp::launch_quantize_act(static_cast<const uint16_t*>(X), M, K, ldx, Xq, sx,
                                             static_cast<const uint16_t*>(U), r, T, pr, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQFP_OK : hip_fail(e);
}

const uint16_t* u16(const void* p) { return static_cast<const uint16_t*>(p); }

// ---- the built-in scratch array of zqfp_w4a8_gemm_lorc_static.  Every device that loads this library holds
// its own copy at its own address until the process ends.  In host code the array's NAME is only a handle
// for hipGetSymbolAddress: the device address is asked for once per device, with that device current, and
// from then on only that address is used (kernel arguments take it as they take a caller's workspace).
static __device__ __align__(256) unsigned char scratch[ZQFP_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // per device; guarded by g_scratch_mutex

int static_scratch(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) {
        g_last_error = "device ordinal beyond the per-device table of the static scratch array";
        return ZQFP_E_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (p == nullptr) {
            g_last_error = "hipGetSymbolAddress returned no address for the static scratch array";
            return ZQFP_E_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ZQFP_OK;
}

}  // namespace

extern "C" {

int zqfp_version(void) { return 106; }

const char* zqfp_last_hip_error(void) { return g_last_error.c_str(); }

int zqfp_quantize_act_fp8(const void* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, float* sx, const void* U,
                          int r, float* T, void* stream)
{
    return quantize_common(X, M, K, ldx, Xq, sx, U, r, T, zqfp::Producer{0, nullptr, nullptr, nullptr, 0, nullptr, 0.0f}, stream);
}

int zqfp_rmsnorm_quantize_act_fp8(const void* X, const void* gain, float eps, int64_t M, int64_t K, int64_t ldx,
                                  uint8_t* Xq, float* sx, const void* U, int r, float* T, void* stream)
{
    return quantize_common(X, M, K, ldx, Xq, sx, U, r, T, zqfp::Producer{1, u16(gain), nullptr, nullptr, 0, nullptr, eps}, stream);
}

int zqfp_layernorm_quantize_act_fp8(const void* X, const void* gain, const void* bias, float eps, int64_t M, int64_t K,
                                    int64_t ldx, uint8_t* Xq, float* sx, const void* U, int r, float* T, void* stream)
{
    return quantize_common(X, M, K, ldx, Xq, sx, U, r, T, zqfp::Producer{2, u16(gain), u16(bias), nullptr, 0, nullptr, eps}, stream);
}

int zqfp_add_rmsnorm_quantize_act_fp8(const void* X, const void* R, int64_t ldr, void* H, const void* gain, float eps,
                                      int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, float* sx, const void* U, int r,
                                      float* T, void* stream)
{
    if (!R && M > 0) return ZQFP_E_NULL;
    return quantize_common(X, M, K, ldx, Xq, sx, U, r, T,
                           zqfp::Producer{1, u16(gain), nullptr, u16(R), ldr, static_cast<uint16_t*>(H), eps}, stream);
}

int zqfp_add_layernorm_quantize_act_fp8(const void* X, const void* R, int64_t ldr, void* H, const void* gain,
                                        const void* bias, float eps, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq,
                                        float* sx, const void* U, int r, float* T, void* stream)
{
    if (!R && M > 0) return ZQFP_E_NULL;
    return quantize_common(X, M, K, ldx, Xq, sx, U, r, T,
                           zqfp::Producer{2, u16(gain), u16(bias), u16(R), ldr, static_cast<uint16_t*>(H), eps}, stream);
}

int zqfp_relu_quantize_act_fp8(const void* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, float* sx, const void* U,
                               int r, float* T, void* stream)
{
    return quantize_common(X, M, K, ldx, Xq, sx, U, r, T, zqfp::Producer{3, nullptr, nullptr, nullptr, 0, nullptr, 0.0f}, stream);
}

int zqfp_swiglu_quantize_act_fp8(const void* G, const void* Up, int64_t ldu, void* H, int64_t M, int64_t K, int64_t ldg,
                                 uint8_t* Xq, float* sx, const void* U, int r, float* T, void* stream)
{
    return quantize_common(G, M, K, ldg, Xq, sx, U, r, T,
                           zqfp::Producer{4, nullptr, nullptr, u16(Up), ldu, static_cast<uint16_t*>(H), 0.0f}, stream);
}

size_t zqfp_packed_weight_bytes(int64_t K, int64_t N, int G)
{
    zqfp::BlobLayout L;
    return zqfp::make_layout(K, N, G, &L) ? L.total : 0;
}

int zqfp_pack_weight_fp4(const void* W, int64_t K, int64_t N, int64_t ldw, int G, int mode, void* packed, void* stream)
{
    zqfp::BlobLayout L;
    if (!zqfp::make_layout(K, N, G, &L) || ldw < N) return ZQFP_E_SHAPE;
    if (mode != ZQFP_SCALE_M1 && mode != ZQFP_SCALE_M2) return ZQFP_E_MODE;
    if (!packed || (N > 0 && !W)) return ZQFP_E_NULL;
    if ((reinterpret_cast<uintptr_t>(packed) & 255u) != 0) return ZQFP_E_ALIGN;
    if (N == 0) return ZQFP_OK;
    hipError_t e = zqfp::launch_pack_weight(static_cast<const uint16_t*>(W), ldw, L, mode, static_cast<uint8_t*>(packed),
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQFP_OK : hip_fail(e);
}

size_t zqfp_packed_weight_fp8_bytes(int64_t K, int64_t N, int G)
{
    zqfp::BlobLayout L;
    return zqfp::make_layout(K, N, G, &L, 8) ? L.total : 0;
}

int zqfp_pack_weight_fp8(const void* W, int64_t K, int64_t N, int64_t ldw, int G, int mode, void* packed, void* stream)
{
    zqfp::BlobLayout L;
    if (!zqfp::make_layout(K, N, G, &L, 8) || ldw < N) return ZQFP_E_SHAPE;
    if (mode != ZQFP_SCALE_M1 && mode != ZQFP_SCALE_M2) return ZQFP_E_MODE;
    if (!packed || (N > 0 && !W)) return ZQFP_E_NULL;
    if ((reinterpret_cast<uintptr_t>(packed) & 255u) != 0) return ZQFP_E_ALIGN;
    if (N == 0) return ZQFP_OK;
    hipError_t e = zqfp::launch_pack_weight(static_cast<const uint16_t*>(W), ldw, L, mode, static_cast<uint8_t*>(packed),
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQFP_OK : hip_fail(e);
}

int zqfp_unpack_codes_fp8(const void* packed, int64_t K, int64_t N, int G, uint8_t* codes, uint8_t* exps, float* colscale,
                          void* stream)
{
    zqfp::BlobLayout L;
    if (!zqfp::make_layout(K, N, G, &L, 8)) return ZQFP_E_SHAPE;
    if (N == 0) return ZQFP_OK;
    if (!packed || !codes || !exps || !colscale) return ZQFP_E_NULL;
    hipError_t e = zqfp::launch_unpack(static_cast<const uint8_t*>(packed), L, codes, exps, colscale,
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQFP_OK : hip_fail(e);
}

int zqfp_w8a8_gemm(const uint8_t* Xq, const float* sx, int64_t M, int64_t K, const void* packed, int64_t N, int G,
                   const float* T, const void* V, int r, void* Y, int64_t ldy, int out_dtype, int accum, void* stream)
{
    if (M < 0 || N < 0 || r < 0 || r > 64) return ZQFP_E_SHAPE;
    zqfp::BlobLayout L;
    if (!zqfp::make_layout(K, N, G, &L, 8)) return ZQFP_E_SHAPE;
    if (out_dtype != ZQFP_OUT_F32 && out_dtype != ZQFP_OUT_BF16) return ZQFP_E_MODE;
    if (accum != ZQFP_ACCUM_EXACT && accum != ZQFP_ACCUM_FAST) return ZQFP_E_MODE;
    if (M == 0 || N == 0) return ZQFP_OK;
    if (!Xq || !sx || !packed || !Y) return ZQFP_E_NULL;
    if (r > 0 && (!T || !V)) return ZQFP_E_NULL;
    if (ldy < N) return ZQFP_E_SHAPE;
    if (!aligned16(Xq) || !aligned16(Y) || (reinterpret_cast<uintptr_t>(packed) & 255u) != 0) return ZQFP_E_ALIGN;
    zqfp::Lorc lorc{r > 0 ? T : nullptr, r > 0 ? static_cast<const uint16_t*>(V) : nullptr, r};
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint8_t* blob = static_cast<const uint8_t*>(packed);
    // the streaming kernel: at most 16 tokens, fewer than 64 output channels, or up to 32 tokens on a small matrix (measured: 7B QKV
    // at 17 tokens 17.6 us against the tiled kernel's 20.3; on the 70B FFN matrix the tiled kernel wins from 17 tokens on, 39 us against 64)
    const bool small = M <= 32 && K * N <= (int64_t)1 << 26;
    hipError_t e = zqfp::gemm_w8_decode_supported(M, L)
                       ? zqfp::launch_gemm_w8_decode(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, accum, s)
                   : !zqfp::gemm_tile_supported(M, L) || small
                       ? zqfp::launch_gemm_stream(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, accum, s)
                       : zqfp::launch_gemm_w8_tile(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, accum, s);
    return e == hipSuccess ? ZQFP_OK : hip_fail(e);
}

int zqfp_packed_weight_check(const void* header, int64_t K, int64_t N, int G)
{
    static_assert(sizeof(zqfp::BlobHeader) <= ZQFP_BLOB_HEADER_BYTES, "header size");
    if (!header) return ZQFP_E_NULL;
    zqfp::BlobHeader h;
    std::memcpy(&h, header, sizeof h);
    zqfp::BlobLayout L;
    if (!zqfp::make_layout(K, N, G, &L, h.wbits == 8 ? 8 : 4)) return ZQFP_E_SHAPE;
    const bool ok = (h.wbits == 4 || h.wbits == 8) && h.magic == zqfp::kBlobMagic && h.version == zqfp::kBlobVersion && h.K == L.K && h.N == L.N &&
                    h.Np == L.Np && h.G == L.G && h.Gs == L.Gs && h.ngs == L.ngs && h.ngq == L.ngq &&
                    (h.mode == ZQFP_SCALE_M1 || h.mode == ZQFP_SCALE_M2) && h.off_codes == L.off_codes &&
                    h.off_exps == L.off_exps && h.off_colscale == L.off_colscale && h.total == L.total;
    return ok ? ZQFP_OK : ZQFP_E_BLOB;
}

int zqfp_unpack_codes(const void* packed, int64_t K, int64_t N, int G, uint8_t* codes, uint8_t* exps, float* colscale,
                      void* stream)
{
    zqfp::BlobLayout L;
    if (!zqfp::make_layout(K, N, G, &L)) return ZQFP_E_SHAPE;
    if (N == 0) return ZQFP_OK;
    if (!packed || !codes || !exps || !colscale) return ZQFP_E_NULL;
    hipError_t e = zqfp::launch_unpack(static_cast<const uint8_t*>(packed), L, codes, exps, colscale,
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQFP_OK : hip_fail(e);
}

size_t zqfp_gemm_workspace_bytes(int64_t M, int64_t K, int64_t N) { return gemm_workspace_need(M, K, N); }

int zqfp_w4a8_gemm(const uint8_t* Xq, const float* sx, int64_t M, int64_t K, const void* packed, int64_t N, int G,
                   void* Y, int64_t ldy, int out_dtype, int accum, void* workspace, size_t workspace_bytes, void* stream)
{
    return gemm_common(Xq, sx, M, K, packed, N, G, nullptr, nullptr, 0, Y, ldy, out_dtype, accum, workspace, workspace_bytes,
                       stream);
}

int zqfp_w4a8_gemm_lorc(const uint8_t* Xq, const float* sx, int64_t M, int64_t K, const void* packed, int64_t N, int G,
                        const float* T, const void* V, int r, void* Y, int64_t ldy, int out_dtype, int accum,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    return gemm_common(Xq, sx, M, K, packed, N, G, T, V, r, Y, ldy, out_dtype, accum, workspace, workspace_bytes, stream);
}

int zqfp_w4a8_gemm_lorc_static(const uint8_t* Xq, const float* sx, int64_t M, int64_t K, const void* packed, int64_t N,
                               int G, const float* T, const void* V, int r, void* Y, int64_t ldy, int out_dtype,
                               int accum, void* stream)
{
    const size_t need = gemm_workspace_need(M, K, N);
    if (need > (size_t)ZQFP_STATIC_SCRATCH_BYTES) {
        g_last_error = "partial results of this (M, K, N) need " + std::to_string(need) +
                       " bytes, the built-in scratch array has " + std::to_string((size_t)ZQFP_STATIC_SCRATCH_BYTES) +
                       ": use zqfp_w4a8_gemm_lorc with a workspace";
        return ZQFP_E_WORKSPACE;
    }
    void* ws = nullptr;
    if (need > 0) {  // shapes without a K-split never touch the array
        const int rc = static_scratch(&ws);
        if (rc != ZQFP_OK) return rc;
    }
    return gemm_common(Xq, sx, M, K, packed, N, G, T, V, r, Y, ldy, out_dtype, accum, ws, ws ? (size_t)ZQFP_STATIC_SCRATCH_BYTES : 0,
                       stream);
}

int zqfp_w4a8_linear(const void* X, int64_t ldx, int64_t M, int64_t K, const void* packed, int64_t N, int G, const void* U,
                     const void* V, int r, uint8_t* Xq, float* sx, float* T, void* Y, int64_t ldy, int out_dtype, int accum,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (M < 0 || N < 0 || r < 0 || r > 64) return ZQFP_E_SHAPE;
    zqfp::BlobLayout L;
    if (!zqfp::make_layout(K, N, G, &L) || ldx < K) return ZQFP_E_SHAPE;
    if (out_dtype != ZQFP_OUT_F32 && out_dtype != ZQFP_OUT_BF16) return ZQFP_E_MODE;
    if (accum != ZQFP_ACCUM_EXACT && accum != ZQFP_ACCUM_FAST) return ZQFP_E_MODE;
    if (M == 0 || N == 0) return ZQFP_OK;
    if (zqfp::gemm_decode_fused_supported(M, L, r)) {
        // one kernel: the decode GEMM quantizes the tokens in its prologue
        if (!X || !packed || !Y) return ZQFP_E_NULL;
        if (ldy < N) return ZQFP_E_SHAPE;
        if (!aligned16(X) || (ldx % 8) != 0 || !aligned16(Xq) || !aligned16(Y) ||
            (reinterpret_cast<uintptr_t>(packed) & 255u) != 0)
            return ZQFP_E_ALIGN;
        hipError_t e = zqfp::launch_gemm_decode(nullptr, nullptr, M, static_cast<const uint8_t*>(packed), L,
                                                zqfp::Lorc{nullptr, nullptr, 0}, Y, ldy, out_dtype, accum, nullptr,
                                                static_cast<hipStream_t>(stream), u16(X), ldx, Xq, sx);
        return e == hipSuccess ? ZQFP_OK : hip_fail(e);
    }
    // two kernels: the quantizer (with the LoRC left factor), then the GEMM; the intermediate buffers are the caller's
    if (!Xq || !sx) return ZQFP_E_NULL;
    const int rc = quantize_common(X, M, K, ldx, Xq, sx, U, r, T, zqfp::Producer{0, nullptr, nullptr, nullptr, 0, nullptr, 0.0f}, stream);
    if (rc != ZQFP_OK) return rc;
    return gemm_common(Xq, sx, M, K, packed, N, G, T, V, r, Y, ldy, out_dtype, accum, workspace, workspace_bytes, stream);
}

size_t zqfp_lorc_workspace_bytes(int64_t K, int64_t N, int r)
{
    if (K <= 0 || N <= 0 || r < 1 || r > 64) return 0;
    return zqfp::lorc_workspace_bytes(K, N, r);
}

int zqfp_lorc_factorize(const void* W, int64_t K, int64_t N, int64_t ldw, const void* packed, int G, int r,
                        const float* Omega, int power_iters, void* U, void* V, float* sigma, void* workspace, void* stream)
{
    zqfp::BlobLayout L;
    if (!zqfp::make_layout(K, N, G, &L) || N == 0 || ldw < N) return ZQFP_E_SHAPE;
    if (r < 1 || r > 64 || r + 8 > K || r + 8 > N || power_iters < 0 || power_iters > 8) return ZQFP_E_SHAPE;
    if (!W || !packed || !Omega || !U || !V || !sigma || !workspace) return ZQFP_E_NULL;
    if ((reinterpret_cast<uintptr_t>(packed) & 255u) != 0 || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 ||
        !aligned16(Omega))
        return ZQFP_E_ALIGN;
    hipError_t e = zqfp::launch_lorc_factorize(static_cast<const uint16_t*>(W), ldw, static_cast<const uint8_t*>(packed), L, r,
                                               Omega, power_iters, static_cast<uint16_t*>(U), static_cast<uint16_t*>(V),
                                               sigma, workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQFP_OK : hip_fail(e);
}

size_t zqfp_gptq_workspace_bytes(int64_t K, int64_t N, int G)
{
    zqfp::BlobLayout L;
    if (!zqfp::make_layout(K, N, G, &L) || N == 0 || (G != 32 && G != 64 && G != 128 && G != 256)) return 0;
    return zqfp::gptq_workspace_bytes(K, N, G);
}

int zqfp_gptq_pack_weight_fp4(const void* W, int64_t K, int64_t N, int64_t ldw, const float* Hinv_u, int G, int mode,
                              void* packed, void* workspace, void* stream)
{
    zqfp::BlobLayout L;
    if (!zqfp::make_layout(K, N, G, &L) || N == 0 || ldw < N) return ZQFP_E_SHAPE;
    if (G != 32 && G != 64 && G != 128 && G != 256) return ZQFP_E_SHAPE;
    if (mode != ZQFP_SCALE_M1 && mode != ZQFP_SCALE_M2) return ZQFP_E_MODE;
    if (!W || !Hinv_u || !packed || !workspace) return ZQFP_E_NULL;
    if ((reinterpret_cast<uintptr_t>(packed) & 255u) != 0 || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return ZQFP_E_ALIGN;
    hipError_t e = zqfp::launch_gptq_pack(static_cast<const uint16_t*>(W), ldw, L, mode, Hinv_u, static_cast<uint8_t*>(packed),
                                          workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQFP_OK : hip_fail(e);
}

int zqfp_probe_stream_read(const void* src, int64_t bytes, void* sink, int workgroups, void* stream)
{
    if (bytes <= 0 || workgroups <= 0) return ZQFP_E_SHAPE;
    if (!src || !sink) return ZQFP_E_NULL;
    if (!aligned16(src)) return ZQFP_E_ALIGN;
    hipError_t e = zqfp::launch_probe_read(src, bytes, static_cast<uint32_t*>(sink), workgroups,
                                           static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQFP_OK : hip_fail(e);
}

int zqfp_probe_force_tile_plan(int bm, int bn, int ksplit, int kg)
{
    return zqfp::force_tile_plan(bm, bn, ksplit, kg) ? ZQFP_OK : ZQFP_E_SHAPE;
}

int zqfp_probe_force_decode_waves(int nw)
{
    if (nw != 8 && nw != 16) return ZQFP_E_SHAPE;
    zqfp::force_decode_waves(nw);
    return ZQFP_OK;
}

int zqfp_probe_mfma(const void* operands, void* sink, int iters, int workgroups, void* stream)
{
    if (iters <= 0 || workgroups <= 0) return ZQFP_E_SHAPE;
    if (!operands || !sink) return ZQFP_E_NULL;
    hipError_t e = zqfp::launch_probe_mfma(static_cast<const uint32_t*>(operands), static_cast<float*>(sink), iters,
                                           workgroups, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ZQFP_OK : hip_fail(e);
}

}  // extern "C"
