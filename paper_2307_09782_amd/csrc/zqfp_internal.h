// Internal declarations shared by the HIP translation units of libzqfp.
// Nothing here is part of the ABI (see include/zqfp.h for that).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

namespace zqfp {

// One-time set-up that several host threads may reach together (raising a kernel's dynamic-LDS limit is a
// per-function setting): the first caller runs `f`, the others wait for it and all see its status.
struct OnceStatus {
    std::once_flag flag;
    hipError_t err = hipSuccess;
};
template <class F>
inline hipError_t run_once(OnceStatus& o, F&& f)
{
    std::call_once(o.flag, [&] { o.err = f(); });
    return o.err;
}

// ---------------------------------------------------------------------------
// Packed weight blob
//
//   [0, 256)            header (BlobHeader, little endian)
//   codes               Np/16 strips x K/128 k-tiles x 1024 B "fragments".
//                       A fragment is the B operand of one 16x16x128 (or half
//                       of one 32x32x64 pair) block-scaled matrix instruction:
//                       lane l (0..63) owns output channel n = 16*strip + l%16
//                       and the 32 consecutive k = 128*ktile + 32*(l/16) + p,
//                       p = 0..31, stored as 16 bytes, code p in byte p/2, even
//                       p in the low nibble.  The fragment stores lane 0's 16
//                       bytes first, so a wave reads it with one 16 B/lane load.
//   exps                E8M0 exponent bytes, [Np/16][ngq][16 columns][4]: the
//                       dword of (strip, quad q, column c) holds the bytes of
//                       stored groups 4q..4q+3.  Stored groups have size Gs
//                       (= G when G is a multiple of 128, else gcd(G,128)); a
//                       real group larger than Gs repeats its byte.
//   colscale            Np float32 (per-output-channel real scale; 1 under M1).
//
// Np = N rounded up to 16; padding columns hold zero codes, exponent byte 127
// and colscale 0.
// ---------------------------------------------------------------------------
struct BlobHeader {
    uint32_t magic;    // 'ZQF4'
    uint32_t version;  // layout version
    int64_t K, N, Np;
    int32_t G, Gs, mode, ngs, ngq;
    uint32_t wbits;    // 4: E2M1 codes, 8: E4M3 codes
    uint64_t off_codes, off_exps, off_colscale, total;
};
constexpr uint32_t kBlobMagic = 0x3446515Au;  // "ZQF4"
constexpr uint32_t kBlobVersion = 1;

struct BlobLayout {
    int64_t K, N, Np, nstrips, nkt;
    int G, Gs, ngs, ngq;
    int wbits;      // weight code width: 4 (E2M1) or 8 (E4M3: fragments of 2 KB, [half][64 lanes][16 B], where half h
                    // of lane l holds k = 128*ktile + 64*h + 16*(l/16) + [0,16) -- the FP8 operand order of the
                    // matrix instruction, each half one contiguous 1 KB read)
    int gsb;        // 32-element blocks per stored group (Gs / 32)
    int gsb_shift;  // log2(gsb) if gsb is a power of two, else -1
    uint32_t gq_magic;  // groups of >= 128: stored group of k-tile kt is (kt * gq_magic) >> 20 (exact for kt < 16384)
    size_t off_codes, off_exps, off_colscale, total;
};

inline int gcd_int(int a, int b) { while (b) { int t = a % b; a = b; b = t; } return a; }

// Returns false if (K, N, G) violates the documented shape limits.
inline bool make_layout(int64_t K, int64_t N, int G, BlobLayout* L, int wbits = 4)
{
    if (K <= 0 || N < 0 || G <= 0 || K % 128 != 0 || G % 32 != 0 || K % G != 0) return false;
    if (wbits != 4 && wbits != 8) return false;
    if (wbits == 8 && G % 128 != 0) return false;  // E4M3 weights: one exponent byte per k-tile and column
    L->wbits = wbits;
    if (K / G > 256) return false;
    if (K / 128 >= 4096) return false;  // the k-tile -> group division by multiplication (gq_magic) is exact below this
    L->K = K; L->N = N; L->Np = (N + 15) / 16 * 16;
    L->nstrips = L->Np / 16; L->nkt = K / 128;
    L->G = G; L->Gs = (G % 128 == 0) ? G : gcd_int(G, 128);
    L->ngs = (int)(K / L->Gs); L->ngq = (L->ngs + 3) / 4;
    L->gsb = L->Gs / 32;
    L->gsb_shift = -1;
    for (int s = 0; s < 16; ++s) if ((1 << s) == L->gsb) L->gsb_shift = s;
    {
        const int gq = L->gsb >= 4 ? L->gsb / 4 : 1;  // k-tiles per stored group
        L->gq_magic = (uint32_t)(((1 << 20) + gq - 1) / gq);  // gq <= 64, so kt * gq_magic < 2^32 for kt < 4096
    }
    L->off_codes = 256;
    L->off_exps = L->off_codes + (size_t)L->Np * (size_t)K * (size_t)wbits / 8;
    size_t exps_bytes = (size_t)L->nstrips * L->ngq * 64;
    L->off_colscale = (L->off_exps + exps_bytes + 255) / 256 * 256;
    L->total = (L->off_colscale + (size_t)L->Np * 4 + 255) / 256 * 256;
    return true;
}

// binary32 -> bfloat16 bits, round to nearest even (finite inputs)
__device__ inline uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// IEEE binary16 bits -> binary32 (exact)
__device__ inline float half_bits_to_f32(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

// Splits the eight dwords of an E4M3 operand into the codes whose exponent field is >= 8
// (bit 6 of the byte set) and the rest; the other bytes of each half are +0.  Inside either
// half the exponents span at most 8 binades, which the matrix core's 8-wide dot unit sums
// without dropping a bit.  One byte permute does the selection: v_perm_b32 picks, per result byte,
// a byte of x or a byte of a zero operand, and the selector is made from bit 6 of each byte.
// Four full-rate operations per dword (shift, and-or, permute, xor).
typedef int zq_v8i __attribute__((ext_vector_type(8)));
__device__ inline void split_exponent_bands_dword(uint32_t x, uint32_t& hi, uint32_t& lo)
{
    // byte selector i (byte i of x) for bytes with bit 6 clear, 4 + i (byte i of the zero operand) for the others
    const uint32_t sel = ((x >> 4) & 0x04040404u) | 0x03020100u;
    lo = __builtin_amdgcn_perm(0u, x, sel);
    hi = x ^ lo;
}
__device__ inline void split_exponent_bands(const zq_v8i& a, zq_v8i& hi, zq_v8i& lo)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t h, l;
        split_exponent_bands_dword((uint32_t)a[i], h, l);
        hi[i] = (int)h;
        lo[i] = (int)l;
    }
}

// ---------------------------------------------------------------------------
// Token-wise E4M3 quantizer arithmetic, shared by the quantizer kernels and the decode GEMM that quantizes in
// its prologue: the same binary32 sequence everywhere, so that the codes have one right answer.
// ---------------------------------------------------------------------------
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ inline uint32_t absmax_bits(uint32_t acc, uint4 v)
{
    // |bf16| ordering equals the ordering of the 15 magnitude bits
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t lo = w[i] & 0x7FFFu, hi = (w[i] >> 16) & 0x7FFFu;
        acc = max(acc, max(lo, hi));
    }
    return acc;
}

__device__ inline float clamp448(float y) { return fminf(fmaxf(y, -448.0f), 448.0f); }

// 8 bf16 -> 8 E4M3 codes (two dwords)
__device__ inline uint2 encode8(uint4 v, float inv)
{
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float y[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        y[2 * i] = clamp448(bf16_lo(w[i]) * inv);
        y[2 * i + 1] = clamp448(bf16_hi(w[i]) * inv);
    }
    int p0 = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], 0, false);
    p0 = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], p0, true);
    int p1 = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], 0, false);
    p1 = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], p1, true);
    return make_uint2((uint32_t)p0, (uint32_t)p1);
}

// token scale and its reciprocal from the row's absmax (15 magnitude bits of a bf16): IEEE binary32 divisions;
// an all-zero (or vanishing, < 2^-96) token gets scale 1 and signed-zero codes
__device__ inline void token_scale(uint32_t absmax_bf16_bits, float& scale, float& inv)
{
    const float amax = __uint_as_float(absmax_bf16_bits << 16);
    scale = 1.0f;
    inv = 0.0f;
    if (amax >= 0x1p-96f) {
        scale = amax / 448.0f;
        inv = 448.0f / amax;
    }
}

// ---------------------------------------------------------------------------
// E2M1 and scale helpers shared by the weight-side kernels (packer, GPTQ, LoRC error matrix)
// ---------------------------------------------------------------------------
__device__ inline float bf16_bits_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// least integer n with amax <= 6 * 2^n (= ceil(log2(amax / 6))), clamped to [-126, 127]; 0 for a zero group
__device__ inline int m1_exponent(float amax)
{
    if (amax == 0.0f) return 0;
    const uint32_t b = __float_as_uint(amax);
    const int ex = (int)(b >> 23);
    if (ex == 0) return -126;  // below 2^-126: far under the clamp
    const uint32_t man = b & 0x7FFFFFu;
    const int n = (ex - 127) - ((man <= 0x400000u) ? 2 : 1);  // significand <= 1.5 ?
    return min(127, max(-126, n));
}

// the same for E4M3 weights: least integer n with amax <= 448 * 2^n (448 = 1.75 * 2^8)
__device__ inline int m1_exponent_e4m3(float amax)
{
    if (amax == 0.0f) return 0;
    const uint32_t b = __float_as_uint(amax);
    const int ex = (int)(b >> 23);
    if (ex == 0) return -126;
    const uint32_t man = b & 0x7FFFFFu;
    const int n = (ex - 127) - ((man <= 0x600000u) ? 8 : 7);  // significand <= 1.75 ?
    return min(127, max(-126, n));
}

// least k >= 0 with amax_max <= amax_g * 2^k (= ceil(log2(S_max / S_g))), clamped to 15
__device__ inline int m2_shift(float amax_max, float amax_g)
{
    if (amax_g == 0.0f) return 15;
    int k = 0;
    while (k < 15 && amax_max > ldexpf(amax_g, k)) ++k;
    return k;
}

// round to nearest E2M1 magnitude, ties to the even code, saturating at 6; sign bit copied
__device__ inline uint32_t e2m1_encode(float y)
{
    const float a = fabsf(y);
    const uint32_t c = a <= 0.25f ? 0u : a < 0.75f ? 1u : a <= 1.25f ? 2u : a < 1.75f ? 3u
                     : a <= 2.5f ? 4u : a < 3.5f ? 5u : a <= 5.0f ? 6u : 7u;
    return c | ((__float_as_uint(y) >> 28) & 8u);
}

// value of an E2M1 code (sign . 2 exponent bits . 1 mantissa bit, bias 1): 0, 0.5, 1, 1.5, 2, 3, 4, 6
__device__ inline float e2m1_value(uint32_t code)
{
    const uint32_t mag = code & 7u;
    const float v = mag < 2u ? 0.5f * (float)mag : (float)(2u + (mag & 1u)) * (float)(1u << ((mag >> 1) - 1u)) * 0.5f;
    return (code & 8u) ? -v : v;
}

// Tile shape, wave groups and K-split of the tiled GEMM for a problem (the launcher and the workspace query
// must agree; gemm_tile.hip plans them).  `kg` wave groups of four waves share a tile and take its k-tiles in
// turn (two waves per SIMD from one workgroup per compute unit).  When even the smallest tiles fill less than a
// third of the chip (few output channels, long K: down-projections at small M), K is cut into `ksplit` slices
// of `kslice` k-tiles, each tile-slice goes to its own workgroup, and the float32 partial tiles meet in a
// workspace (ksplit * M * Np floats) that a second kernel sums in fixed order.
struct TilePlan {
    int bm, bn;       // tile shape
    int kg;           // wave groups per workgroup (1 or 2)
    int ksplit;       // number of K slices (1: none)
    int kslice;       // k-tiles per slice
    bool forced = false;  // set through the tuning hook (zqfp_probe_force_tile_plan), not planned
};
TilePlan plan_tiles(int64_t M, int64_t Np, int64_t nkt);

// The decode GEMM keeps a wave's activation fragments in registers, at most 8 k-tiles per wave and
// 64 per workgroup.  A longer K is cut into `chunks` pieces of `len` k-tiles; a workgroup serves one
// piece, and the float32 partial results meet in the caller's workspace ([chunks][M][Np]) like
// the K slices of the tiled form.
struct DecodePlan { int chunks, len; };
inline DecodePlan plan_decode(int64_t nkt)
{
    DecodePlan p;
    p.chunks = (int)((nkt + 63) / 64);
    p.len = (int)((nkt + p.chunks - 1) / p.chunks);
    return p;
}

// LoRC arguments of the GEMM epilogue (r == 0: none)
struct Lorc {
    const float* T;     // [M, r]
    const uint16_t* V;  // [r, N] binary16 bits
    int r;
};

// Launchers (each enqueues on `s` and returns the launch status).
// What is fused in front of the activation quantizer (rows with a producer: K <= 32768).
struct Producer {
    int kind;               // 0 none, 1 RMS normalisation, 2 layer normalisation, 3 ReLU, 4 gated SiLU
    const uint16_t* gain;   // [K] bf16 (kinds 1, 2)
    const uint16_t* bias;   // [K] bf16 (kind 2)
    const uint16_t* other;  // [M, K] bf16, row stride ld_other: residual added first (kinds 1, 2; may be null),
    int64_t ld_other;       //   or the operand multiplied with silu(X) (kind 4)
    uint16_t* H;            // [M, K] bf16 dense: X + other rounded to bf16 (kinds 1, 2 with a residual)
    float eps;              // kinds 1, 2
};
hipError_t launch_quantize_act(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq,
                               float* sx, const uint16_t* U, int r, float* T, const Producer& pr, hipStream_t s);
hipError_t launch_pack_weight(const uint16_t* W, int64_t ldw, const BlobLayout& L, int mode,
                              uint8_t* blob, hipStream_t s);
hipError_t launch_unpack(const uint8_t* blob, const BlobLayout& L, uint8_t* codes, uint8_t* exps,
                         float* colscale, hipStream_t s);
hipError_t launch_gemm_stream(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob,
                              const BlobLayout& L, Lorc lorc, void* Y, int64_t ldy, int out_dtype,
                              int accum, hipStream_t s);
// W8A8 (E4M3 weights, L.wbits == 8), at most 16 tokens: the persistent weight-streaming kernel
bool gemm_w8_decode_supported(int64_t M, const BlobLayout& L);
hipError_t launch_gemm_w8_decode(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob,
                                 const BlobLayout& L, Lorc lorc, void* Y, int64_t ldy, int out_dtype,
                                 int accum, hipStream_t s);
// W8A8 (E4M3 weights, L.wbits == 8), more than 16 tokens: the tiled kernel with two-register-quad B operands,
// 128 x 128 or 64 x 128 tiles
hipError_t launch_gemm_w8_tile(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob,
                               const BlobLayout& L, Lorc lorc, void* Y, int64_t ldy, int out_dtype,
                               int accum, hipStream_t s);
// workspace: device memory of plan_tiles(...).ksplit * M * Np floats, or nullptr (then K is not split)
hipError_t launch_gemm_tile(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob,
                            const BlobLayout& L, Lorc lorc, void* Y, int64_t ldy, int out_dtype,
                            int accum, void* workspace, hipStream_t s);
bool gemm_tile_supported(int64_t M, const BlobLayout& L);
// The plan the tiled form runs for a problem: plan_tiles, unless the tuning hook has fixed one (tile shape and
// number of K slices for every following call; 0, 0, 0 returns to automatic planning; false = not a shape the kernel has).
TilePlan effective_tile_plan(int64_t M, int64_t Np, int64_t nkt);
bool force_tile_plan(int bm, int bn, int ksplit, int kg);

// workspace: plan_decode(nkt).chunks * M * Np floats when K has more than 64 k-tiles (else unused)
// X != nullptr: the fused form (gemm_decode_fused_supported): bfloat16 activations, quantized in the kernel's
// prologue; Xq and sx are then unused, Xq_out / sx_out (may be null) receive the codes and scales.
hipError_t launch_gemm_decode(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob,
                              const BlobLayout& L, Lorc lorc, void* Y, int64_t ldy, int out_dtype,
                              int accum, void* workspace, hipStream_t s, const uint16_t* X = nullptr,
                              int64_t ldx = 0, uint8_t* Xq_out = nullptr, float* sx_out = nullptr);
bool gemm_decode_fused_supported(int64_t M, const BlobLayout& L, int r);
void force_decode_waves(int nw);  // tuning hook: 8 or 16 waves per workgroup of the decode form
bool gemm_decode_supported(int64_t M, const BlobLayout& L, const void* workspace);
int compute_units();  // of the current device (asked once)
// Y[m,n] = (sx[m] c[n]) * sum_s partial[s][m][n] (+ T.V): the second kernel of every K-split
hipError_t launch_splitk_reduce(const float* partial, int slices, int64_t M, const uint8_t* blob, const BlobLayout& L,
                                const float* sx, Lorc lorc, void* Y, int64_t ldy, int out_dtype, hipStream_t s);
// LoRC factorisation of W - W^ (offline): U [K, r], V [r, N] binary16, sigma [r]; Omega [N, r + 8] float32
size_t lorc_workspace_bytes(int64_t K, int64_t N, int r);
hipError_t launch_lorc_factorize(const uint16_t* W, int64_t ldw, const uint8_t* blob, const BlobLayout& L, int r,
                                 const float* Omega, int power_iters, uint16_t* U, uint16_t* V, float* sigma,
                                 void* workspace, hipStream_t s);
// GPTQ with the E2M1 grid (offline): U = upper Cholesky factor of the inverse Hessian, [K][K] float32; G in {32, 64, 128, 256}
size_t gptq_workspace_bytes(int64_t K, int64_t N, int G);
hipError_t launch_gptq_pack(const uint16_t* W, int64_t ldw, const BlobLayout& L, int mode, const float* U, uint8_t* blob,
                            void* workspace, hipStream_t s);
hipError_t launch_probe_read(const void* src, int64_t bytes, uint32_t* sink, int workgroups, hipStream_t s);
hipError_t launch_probe_mfma(const uint32_t* operands, float* sink, int iters, int workgroups, hipStream_t s);

}  // namespace zqfp
