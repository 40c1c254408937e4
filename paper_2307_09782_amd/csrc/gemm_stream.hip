// W4A8 GEMM, weight-streaming form for small token counts (decode): bound by
// reading the packed FP4 weights once from HBM.
//
//   Y[m,n] = (sx[m] c[n]) * sum_k a[m,k] * q[k,n] * 2^e[g(k),n]   (+ T.V, LoRC)
//
// (paper Sections 1 and 3: FP8 activations x FP4 weights with power-of-two
// group scales.)  The power of two is never multiplied in: the E8M0 exponent
// byte goes to the block-scaled matrix instruction
// v_mfma_scale_f32_16x16x128_f8f6f4 (A = E4M3, B = E2M1), which applies it per
// 32-element block of K inside the matrix core.
//
// Work split: one workgroup (8 waves) per strip of 16 output channels and per
// block of up to 64 tokens; the 8 waves split K (k-tile i goes to wave i % 8)
// and meet in LDS, so the sum needs neither atomics nor a second pass and its
// order is fixed.  Each weight fragment is a contiguous 1 KB read (16 B/lane).
#include "zqfp_internal.h"

namespace zqfp {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kUnroll = 4;  // k-tiles whose loads are issued before their matrix instructions

// W8: the weights are E4M3 codes (W8A8, paper Section 4): a fragment is two 1 KB halves, the B operand has eight
// registers and the instruction's format field says FP8 on both sides.
template <int MT, bool EXACT, bool W8 = false>
__global__ __launch_bounds__(kThreads) void k_gemm_stream(const uint8_t* __restrict__ Xq, const float* __restrict__ sx,
                                                        int64_t M, const uint8_t* __restrict__ blob, BlobLayout L,
                                                        Lorc lorc, void* __restrict__ Y, int64_t ldy, int out_dtype)
{
    __shared__ float s_red[kWaves][MT][64][4];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col = lane & 15, lb = lane >> 4;
    const int64_t strip = blockIdx.x;
    const int64_t m_base = (int64_t)blockIdx.y * (16 * MT);
    const int nkt = (int)L.nkt;

    constexpr int kFragVec = W8 ? 128 : 64;  // 16-byte vectors per fragment
    const u32x4* bfrag = reinterpret_cast<const u32x4*>(blob + L.off_codes) + strip * nkt * kFragVec + lane;
    const uint32_t* ex = reinterpret_cast<const uint32_t*>(blob + L.off_exps) + strip * L.ngq * 16 + col;

    // A operand of the instruction: lane (row = lane%16, lb = lane/16) holds the bytes
    // k = 16*lb + [0,16) and k = 64 + 16*lb + [0,16) of the 128-wide k-tile.
    const uint8_t* arow[MT];
    bool alive[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        int64_t m = m_base + t * 16 + col;
        alive[t] = m < M;
        arow[t] = Xq + (alive[t] ? m : 0) * L.K + 16 * lb;
    }

    v4f acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = (v4f){0.f, 0.f, 0.f, 0.f};

    for (int kt0 = wave; kt0 < nkt; kt0 += kWaves * kUnroll) {
        u32x4 b[kUnroll], b2[W8 ? kUnroll : 1];
        uint32_t e[kUnroll];
        u32x4 a_lo[kUnroll][MT], a_hi[kUnroll][MT];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int kt = kt0 + u * kWaves;
            if (kt < nkt) {
                b[u] = bfrag[(int64_t)kt * kFragVec];
                if constexpr (W8) b2[u] = bfrag[(int64_t)kt * kFragVec + 64];
                const int blk = kt * 4 + lb;  // 32-element block index along K
                const int sg = (L.gsb_shift >= 0) ? (blk >> L.gsb_shift) : (blk / L.gsb);
                e[u] = ex[(sg >> 2) * 16] >> (8 * (sg & 3));
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    if (alive[t]) {
                        a_lo[u][t] = *reinterpret_cast<const u32x4*>(arow[t] + (int64_t)kt * 128);
                        a_hi[u][t] = *reinterpret_cast<const u32x4*>(arow[t] + (int64_t)kt * 128 + 64);
                    } else {
                        a_lo[u][t] = (u32x4){0u, 0u, 0u, 0u};
                        a_hi[u][t] = (u32x4){0u, 0u, 0u, 0u};
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int kt = kt0 + u * kWaves;
            if (kt < nkt) {
                v8i bv = {(int)b[u][0], (int)b[u][1], (int)b[u][2], (int)b[u][3], 0, 0, 0, 0};
                if constexpr (W8) { bv[4] = (int)b2[u][0]; bv[5] = (int)b2[u][1]; bv[6] = (int)b2[u][2]; bv[7] = (int)b2[u][3]; }
                constexpr int kBlgp = W8 ? 0 : 4;  // format of B: 0 = E4M3, 4 = E2M1
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    v8i av = {(int)a_lo[u][t][0], (int)a_lo[u][t][1], (int)a_lo[u][t][2], (int)a_lo[u][t][3],
                              (int)a_hi[u][t][0], (int)a_hi[u][t][1], (int)a_hi[u][t][2], (int)a_hi[u][t][3]};
                    // cbsz 0: A is E4M3; blgp 4: B is E2M1; A scale byte 127 = 2^0; B scale = group exponent
                    if constexpr (EXACT) {
                        v8i hi, lo;
                        split_exponent_bands(av, hi, lo);
                        acc[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(hi, bv, acc[t], 0, kBlgp, 0, 127, 0, (int)e[u]);
                        acc[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(lo, bv, acc[t], 0, kBlgp, 0, 127, 0, (int)e[u]);
                    } else {
                        acc[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[t], 0, kBlgp, 0, 127, 0, (int)e[u]);
                    }
                }
            }
        }
    }

#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) s_red[wave][t][lane][i] = acc[t][i];
    __syncthreads();

    // epilogue: one output element per thread; D[row][col] sits in lane 16*(row/4)+col, register row%4
    const float* colscale = reinterpret_cast<const float*>(blob + L.off_colscale);
    for (int o = tid; o < MT * 256; o += kThreads) {
        const int t = o >> 8, idx = o & 255, r = idx >> 4, c = idx & 15;
        const int64_t m = m_base + t * 16 + r, n = strip * 16 + c;
        if (m >= M || n >= L.N) continue;
        const int src = 16 * (r >> 2) + c, reg = r & 3;
        float a = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) a += s_red[w][t][src][reg];
        float y = (sx[m] * colscale[n]) * a;
        for (int j = 0; j < lorc.r; ++j)
            y = fmaf(lorc.T[m * lorc.r + j], half_bits_to_f32(lorc.V[(int64_t)j * L.N + n]), y);
        if (out_dtype == 0) reinterpret_cast<float*>(Y)[m * ldy + n] = y;
        else reinterpret_cast<uint16_t*>(Y)[m * ldy + n] = f32_to_bf16_bits(y);
    }
}

template <int MT>
void launch_mt(dim3 grid, bool exact, const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob,
               const BlobLayout& L, Lorc lorc, void* Y, int64_t ldy, int out_dtype, hipStream_t s)
{
#define ZQ_STREAM(EX, W8) hipLaunchKernelGGL((k_gemm_stream<MT, EX, W8>), grid, dim3(kThreads), 0, s, Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype)
    if (L.wbits == 8) { if (exact) ZQ_STREAM(true, true); else ZQ_STREAM(false, true); }
    else { if (exact) ZQ_STREAM(true, false); else ZQ_STREAM(false, false); }
#undef ZQ_STREAM
}

}  // namespace

hipError_t launch_gemm_stream(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L,
                              Lorc lorc, void* Y, int64_t ldy, int out_dtype, int accum, hipStream_t s)
{
    if (M == 0 || L.N == 0) return hipSuccess;
    const bool exact = accum == 0;
    const unsigned ns = (unsigned)L.nstrips;
    if (M <= 16) launch_mt<1>(dim3(ns, 1), exact, Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, s);
    else if (M <= 32) launch_mt<2>(dim3(ns, 1), exact, Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, s);
    else launch_mt<4>(dim3(ns, (unsigned)((M + 63) / 64)), exact, Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, s);
    return hipGetLastError();
}

}  // namespace zqfp
