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
template <int RP, int NT>
__global__ __launch_bounds__(NT) void k_quantize_act(const uint16_t* __restrict__ X, int64_t K, int64_t ldx,
                                                         uint8_t* __restrict__ Xq, float* __restrict__ sx,
                                                         const uint16_t* __restrict__ U, int r, float* __restrict__ T)
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
    uint32_t am = 0;
#pragma unroll
    for (int c = 0; c < kRegChunks; ++c) {
        int idx = tid + c * kThreads;
        v[c] = make_uint4(0, 0, 0, 0);
        if (idx < nchunk) v[c] = xrow[idx];
        am = absmax_bits(am, v[c]);
    }
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

}  // namespace

hipError_t launch_quantize_act(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, float* sx,
                               const uint16_t* U, int r, float* T, hipStream_t s)
{
    if (M == 0) return hipSuccess;
    const dim3 grid((unsigned)M);
#define ZQ_QUANT(RP)                                                                                           \
    do {                                                                                                       \
        if (M <= 64 && K >= 2048) hipLaunchKernelGGL((k_quantize_act<RP, 1024>), grid, dim3(1024), 0, s, X, K, ldx, Xq, sx, U, r, T); \
        else hipLaunchKernelGGL((k_quantize_act<RP, 256>), grid, dim3(256), 0, s, X, K, ldx, Xq, sx, U, r, T);   \
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
