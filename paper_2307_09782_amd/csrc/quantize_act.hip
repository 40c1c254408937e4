// Token-wise FP8 (E4M3) activation quantizer, with the optional LoRC left
// factor T = X.U computed in the same sweep (paper Section 3: token-wise
// activation quantization, LoRC; Appendix A).
//
// One workgroup of 256 threads per token (1024 for a handful of tokens).  The row is read once with 16-byte
// loads (8 bf16 per lane), kept in registers across the absmax reduction
// (rows up to 8192 elements; longer rows are re-read, from L2), scaled,
// converted with the hardware FP8 conversion (round to nearest even) after an
// explicit clamp to +-448, and written with 8-byte stores.  HBM-bound: 2 B read
// and 1 B written per element.
#include "zqfp_internal.h"

namespace zqfp {
namespace {

constexpr int kRegChunks = 4;  // 16-byte chunks per thread kept in registers

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

__device__ inline float half_bits_to_float(uint32_t h) { return half_bits_to_f32((uint16_t)h); }

// acc[j] += sum_i x_i * U[k_i][j] for the 8 elements (x_i, k_i = kbase + 64 i) that a lane picked up
// from its wave's 512-element slice: consecutive lanes own consecutive k, so a wave's load of U
// rows is one contiguous run (r = 8: 1 KB per instruction) instead of 64 scattered 16-byte pieces.
template <int RP>
__device__ inline void lorc_accumulate(float (&acc)[RP], const float (&x)[8], const uint16_t* U, int64_t kbase, int64_t K, int r)
{
    // K is a multiple of 128, not of 512: elements past the row's end are zero and meet a zeroed row of U
    if ((r & 7) == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const bool live = kbase + 64 * i < K;
            const uint4* urow = reinterpret_cast<const uint4*>(U + (live ? kbase + 64 * i : 0) * r);
#pragma unroll
            for (int jb = 0; jb < RP / 8; ++jb) {
                if (jb * 8 < r) {
                    uint4 u = urow[jb];
                    uint32_t uw[4] = {live ? u.x : 0u, live ? u.y : 0u, live ? u.z : 0u, live ? u.w : 0u};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        acc[jb * 8 + 2 * q] = fmaf(x[i], half_bits_to_float(uw[q] & 0xFFFFu), acc[jb * 8 + 2 * q]);
                        acc[jb * 8 + 2 * q + 1] = fmaf(x[i], half_bits_to_float(uw[q] >> 16), acc[jb * 8 + 2 * q + 1]);
                    }
                }
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < RP; ++j)
                if (j < r && kbase + 64 * i < K) acc[j] = fmaf(x[i], half_bits_to_float(U[(kbase + 64 * i) * r + j]), acc[j]);
    }
}

// NT threads per token: 256 when there are tokens enough to fill the chip, 1024 for a handful of
// tokens (decode), where one row's latency chain is all there is.
__device__ inline uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest even (finite inputs)
    return u >> 16;
}

// 8 bf16 -> 8 bf16: (x * rstd) * g, each product one binary32 operation, rounded to bf16
__device__ inline uint4 normalize8(uint4 v, uint4 g, float rstd)
{
    uint32_t w[4] = {v.x, v.y, v.z, v.w}, gw[4] = {g.x, g.y, g.z, g.w}, o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo = (bf16_lo(w[i]) * rstd) * bf16_lo(gw[i]);
        const float hi = (bf16_hi(w[i]) * rstd) * bf16_hi(gw[i]);
        o[i] = f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}

__device__ inline double sum_squares(double acc, uint4 v)
{
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const double lo = (double)bf16_lo(w[i]), hi = (double)bf16_hi(w[i]);
        acc += lo * lo;  // each square is exact in binary64
        acc += hi * hi;
    }
    return acc;
}

template <int RP, int NT, bool NORM>
__global__ __launch_bounds__(NT) void k_quantize_act(const uint16_t* __restrict__ X, int64_t K, int64_t ldx,
                                                         uint8_t* __restrict__ Xq, float* __restrict__ sx,
                                                         const uint16_t* __restrict__ U, int r, float* __restrict__ T,
                                                         const uint16_t* __restrict__ gain, float eps)
{
    constexpr int kThreads = NT, kWaves = NT / 64;
    __shared__ uint32_t s_amax[kWaves];
    __shared__ float s_t[kWaves][RP > 0 ? RP : 1];
    __shared__ __attribute__((aligned(16))) uint16_t s_x[RP > 0 ? kWaves : 1][512];  // per wave: its current 512-element slice
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x;
    const uint4* xrow = reinterpret_cast<const uint4*>(X + row * ldx);
    uint2* qrow = reinterpret_cast<uint2*>(Xq + row * K);
    const int nchunk = (int)(K / 8);

    uint4 v[kRegChunks];
#pragma unroll
    for (int c = 0; c < kRegChunks; ++c) {
        int idx = tid + c * kThreads;
        v[c] = make_uint4(0, 0, 0, 0);
        if (idx < nchunk) v[c] = xrow[idx];
    }
    if constexpr (NORM) {
        // the whole row sits in registers (the launcher guarantees K <= 8 * kRegChunks * NT): sum of
        // squares in binary64, waves meet in LDS and every thread adds the partial sums in the same
        // order; then the normalised row replaces the row
        __shared__ double s_ss[kWaves];
        const uint4* grow = reinterpret_cast<const uint4*>(gain);
        uint4 g[kRegChunks];
        double ss = 0.0;
#pragma unroll
        for (int c = 0; c < kRegChunks; ++c) {
            int idx = tid + c * kThreads;
            g[c] = make_uint4(0, 0, 0, 0);
            if (idx < nchunk) g[c] = grow[idx];
            ss = sum_squares(ss, v[c]);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
        if ((tid & 63) == 0) s_ss[tid >> 6] = ss;
        __syncthreads();
        ss = s_ss[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) ss += s_ss[w];
        const float ms = (float)(ss / (double)K);
        const float rstd = 1.0f / sqrtf(ms + eps);  // IEEE binary32 add, square root, division
#pragma unroll
        for (int c = 0; c < kRegChunks; ++c) v[c] = normalize8(v[c], g[c], rstd);
    }
    uint32_t am = 0;
#pragma unroll
    for (int c = 0; c < kRegChunks; ++c) am = absmax_bits(am, v[c]);
    if constexpr (!NORM)
        for (int idx = tid + kRegChunks * kThreads; idx < nchunk; idx += kThreads) am = absmax_bits(am, xrow[idx]);

    // LoRC left factor first: its loads of U overlap the row's own loads and the absmax reduction.
    // A lane holds 8 consecutive elements; for the product with U it trades them, through a
    // wave-private LDS slice, for the 8 elements lane, lane + 64, ... of the wave's 512.
    float acc[RP > 0 ? RP : 1];
    if constexpr (RP > 0) {
        const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
        for (int j = 0; j < RP; ++j) acc[j] = 0.0f;
        auto one_chunk = [&](uint4 vc, int idx) {
            *reinterpret_cast<uint4*>(&s_x[wave][lane * 8]) = vc;  // same wave writes and reads: no barrier
            float x[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = __uint_as_float((uint32_t)s_x[wave][lane + 64 * i] << 16);
            lorc_accumulate<RP>(acc, x, U, (int64_t)(idx - lane) * 8 + lane, K, r);
        };
#pragma unroll
        for (int c = 0; c < kRegChunks; ++c) {
            int idx = tid + c * kThreads;
            if (idx - lane < nchunk) one_chunk(idx < nchunk ? v[c] : make_uint4(0, 0, 0, 0), idx);
        }
        if constexpr (!NORM)
            for (int idx = tid + kRegChunks * kThreads; idx - lane < nchunk; idx += kThreads)
                one_chunk(idx < nchunk ? xrow[idx] : make_uint4(0, 0, 0, 0), idx);
    }

#pragma unroll
    for (int off = 32; off > 0; off >>= 1) am = max(am, (uint32_t)__shfl_xor((int)am, off));
    if ((tid & 63) == 0) s_amax[tid >> 6] = am;
    __syncthreads();
    am = s_amax[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) am = max(am, s_amax[w]);

    const float amax = __uint_as_float(am << 16);
    float scale = 1.0f, inv = 0.0f;  // all-zero (or vanishing) token: signed-zero codes, scale 1
    if (amax >= 0x1p-96f) {
        scale = amax / 448.0f;  // IEEE binary32 division
        inv = 448.0f / amax;    // IEEE binary32 division
    }
    if (tid == 0) sx[row] = scale;

#pragma unroll
    for (int c = 0; c < kRegChunks; ++c) {
        int idx = tid + c * kThreads;
        if (idx < nchunk) qrow[idx] = encode8(v[c], inv);
    }
    if constexpr (!NORM)
        for (int idx = tid + kRegChunks * kThreads; idx < nchunk; idx += kThreads) qrow[idx] = encode8(xrow[idx], inv);

    if constexpr (RP > 0) {
#pragma unroll
        for (int j = 0; j < RP; ++j) {
            float a = acc[j];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off);
            if ((tid & 63) == 0) s_t[tid >> 6][j] = a;
        }
        __syncthreads();
        if (tid < r) {  // fixed order: pairs of waves, then the pairs in sequence
            float t = 0.0f;
#pragma unroll
            for (int w = 0; w < kWaves; w += 2) t += s_t[w][tid] + s_t[w + 1][tid];
            T[row * r + tid] = t;
        }
    }
}

// ---------------------------------------------------------------------------
// Wave-per-token form for many tokens without the LoRC factor: a row of up to 8 * 64 * MAXC
// elements sits in one wave's registers (16 B per lane per load, 1 KB contiguous per instruction),
// the reductions are wave shuffles only, and no barrier or LDS is involved; 16 waves per compute
// unit keep 8 * MAXC KB of loads in flight each.
// ---------------------------------------------------------------------------
template <int MAXC, bool NORM>
__global__ __launch_bounds__(256) void k_quantize_rows(const uint16_t* __restrict__ X, int64_t M, int64_t K, int64_t ldx,
                                                     uint8_t* __restrict__ Xq, float* __restrict__ sx,
                                                     const uint16_t* __restrict__ gain, float eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;  // whole waves leave; nothing below synchronises across waves
    const uint4* xrow = reinterpret_cast<const uint4*>(X + row * ldx);
    uint2* qrow = reinterpret_cast<uint2*>(Xq + row * K);
    const int nchunk = (int)(K / 8);

    uint4 v[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int idx = c * 64 + lane;
        v[c] = make_uint4(0, 0, 0, 0);
        if (idx < nchunk) v[c] = xrow[idx];
    }
    if constexpr (NORM) {
        double ss = 0.0;
#pragma unroll
        for (int c = 0; c < MAXC; ++c) ss = sum_squares(ss, v[c]);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);  // every lane ends with the same sum
        const float ms = (float)(ss / (double)K);
        const float rstd = 1.0f / sqrtf(ms + eps);  // IEEE binary32 add, square root, division
        const uint4* grow = reinterpret_cast<const uint4*>(gain);
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int idx = c * 64 + lane;
            if (idx < nchunk) v[c] = normalize8(v[c], grow[idx], rstd);
        }
    }
    uint32_t am = 0;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) am = absmax_bits(am, v[c]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) am = max(am, (uint32_t)__shfl_xor((int)am, off));
    const float amax = __uint_as_float(am << 16);
    float scale = 1.0f, inv = 0.0f;  // all-zero (or vanishing) token: signed-zero codes, scale 1
    if (amax >= 0x1p-96f) {
        scale = amax / 448.0f;  // IEEE binary32 division
        inv = 448.0f / amax;    // IEEE binary32 division
    }
    if (lane == 0) sx[row] = scale;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int idx = c * 64 + lane;
        if (idx < nchunk) qrow[idx] = encode8(v[c], inv);
    }
}

}  // namespace

hipError_t launch_quantize_act(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, float* sx,
                               const uint16_t* U, int r, float* T, const uint16_t* gain, float eps, hipStream_t s)
{
    if (M == 0) return hipSuccess;
    const bool norm = gain != nullptr;
    if (r == 0 && M >= 1024 && K <= 8192) {  // many tokens, no LoRC factor: one wave per token
        const dim3 g4((unsigned)((M + 3) / 4));
#define ZQ_ROWS(MAXC)                                                                                                  \
    do {                                                                                                               \
        if (norm) hipLaunchKernelGGL((k_quantize_rows<MAXC, true>), g4, dim3(256), 0, s, X, M, K, ldx, Xq, sx, gain, eps);  \
        else hipLaunchKernelGGL((k_quantize_rows<MAXC, false>), g4, dim3(256), 0, s, X, M, K, ldx, Xq, sx, gain, eps);      \
    } while (0)
        if (K <= 2048) ZQ_ROWS(4);
        else if (K <= 4096) ZQ_ROWS(8);
        else ZQ_ROWS(16);
#undef ZQ_ROWS
        return hipGetLastError();
    }
    const dim3 grid((unsigned)M);
    // 1024 threads per token for a handful of tokens, and for normalised rows too long for 256 threads' registers
    const bool wide = (M <= 64 && K >= 2048) || (norm && K > 8 * kRegChunks * 256);
#define ZQ_QUANT(RP)                                                                                                       \
    do {                                                                                                                   \
        if (norm && wide) hipLaunchKernelGGL((k_quantize_act<RP, 1024, true>), grid, dim3(1024), 0, s, X, K, ldx, Xq, sx, U, r, T, gain, eps); \
        else if (norm) hipLaunchKernelGGL((k_quantize_act<RP, 256, true>), grid, dim3(256), 0, s, X, K, ldx, Xq, sx, U, r, T, gain, eps);      \
        else if (wide) hipLaunchKernelGGL((k_quantize_act<RP, 1024, false>), grid, dim3(1024), 0, s, X, K, ldx, Xq, sx, U, r, T, gain, eps);   \
        else hipLaunchKernelGGL((k_quantize_act<RP, 256, false>), grid, dim3(256), 0, s, X, K, ldx, Xq, sx, U, r, T, gain, eps);               \
    } while (0)
    if (r == 0) ZQ_QUANT(0);
    else if (r <= 8) ZQ_QUANT(8);
    else if (r <= 16) ZQ_QUANT(16);
    else if (r <= 32) ZQ_QUANT(32);
    else ZQ_QUANT(64);
#undef ZQ_QUANT
    return hipGetLastError();
}

}  // namespace zqfp
