// Token-wise FP8 (E4M3) activation quantizer, with the optional LoRC left
// factor T = X.U computed in the same sweep (paper Section 3: token-wise
// activation quantization, LoRC; Appendix A).
//
// One workgroup of 256 threads per token.  The row is read once with 16-byte
// loads (8 bf16 per lane), kept in registers across the absmax reduction
// (rows up to 8192 elements; longer rows are re-read, from L2), scaled,
// converted with the hardware FP8 conversion (round to nearest even) after an
// explicit clamp to +-448, and written with 8-byte stores.  HBM-bound: 2 B read
// and 1 B written per element.
#include "zqfp_internal.h"

namespace zqfp {
namespace {

constexpr int kThreads = 256;
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

// acc[j] += sum_i x[k0+i] * U[k0+i][j]
template <int RP>
__device__ inline void lorc_accumulate(float (&acc)[RP], uint4 v, const uint16_t* U, int64_t k0, int r)
{
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float x[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) { x[2 * i] = bf16_lo(w[i]); x[2 * i + 1] = bf16_hi(w[i]); }
    if ((r & 7) == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint4* urow = reinterpret_cast<const uint4*>(U + (k0 + i) * r);
#pragma unroll
            for (int jb = 0; jb < RP / 8; ++jb) {
                if (jb * 8 < r) {
                    uint4 u = urow[jb];
                    uint32_t uw[4] = {u.x, u.y, u.z, u.w};
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
                if (j < r) acc[j] = fmaf(x[i], half_bits_to_float(U[(k0 + i) * r + j]), acc[j]);
    }
}

template <int RP>
__global__ __launch_bounds__(kThreads) void k_quantize_act(const uint16_t* __restrict__ X, int64_t K, int64_t ldx,
                                                         uint8_t* __restrict__ Xq, float* __restrict__ sx,
                                                         const uint16_t* __restrict__ U, int r, float* __restrict__ T)
{
    __shared__ uint32_t s_amax[kThreads / 64];
    __shared__ float s_t[kThreads / 64][RP > 0 ? RP : 1];
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

#pragma unroll
    for (int off = 32; off > 0; off >>= 1) am = max(am, (uint32_t)__shfl_xor((int)am, off));
    if ((tid & 63) == 0) s_amax[tid >> 6] = am;
    __syncthreads();
    am = max(max(s_amax[0], s_amax[1]), max(s_amax[2], s_amax[3]));

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
        float acc[RP];
#pragma unroll
        for (int j = 0; j < RP; ++j) acc[j] = 0.0f;
#pragma unroll
        for (int c = 0; c < kRegChunks; ++c) {
            int idx = tid + c * kThreads;
            if (idx < nchunk) lorc_accumulate<RP>(acc, v[c], U, (int64_t)idx * 8, r);
        }
        for (int idx = tid + kRegChunks * kThreads; idx < nchunk; idx += kThreads)
            lorc_accumulate<RP>(acc, xrow[idx], U, (int64_t)idx * 8, r);
#pragma unroll
        for (int j = 0; j < RP; ++j) {
            float a = acc[j];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off);
            if ((tid & 63) == 0) s_t[tid >> 6][j] = a;
        }
        __syncthreads();
        if (tid < r) T[row * r + tid] = (s_t[0][tid] + s_t[1][tid]) + (s_t[2][tid] + s_t[3][tid]);
    }
}

}  // namespace

hipError_t launch_quantize_act(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, float* sx,
                               const uint16_t* U, int r, float* T, hipStream_t s)
{
    if (M == 0) return hipSuccess;
    dim3 grid((unsigned)M), block(kThreads);
    if (r == 0) hipLaunchKernelGGL(k_quantize_act<0>, grid, block, 0, s, X, K, ldx, Xq, sx, U, r, T);
    else if (r <= 8) hipLaunchKernelGGL(k_quantize_act<8>, grid, block, 0, s, X, K, ldx, Xq, sx, U, r, T);
    else if (r <= 16) hipLaunchKernelGGL(k_quantize_act<16>, grid, block, 0, s, X, K, ldx, Xq, sx, U, r, T);
    else if (r <= 32) hipLaunchKernelGGL(k_quantize_act<32>, grid, block, 0, s, X, K, ldx, Xq, sx, U, r, T);
    else hipLaunchKernelGGL(k_quantize_act<64>, grid, block, 0, s, X, K, ldx, Xq, sx, U, r, T);
    return hipGetLastError();
}

}  // namespace zqfp
