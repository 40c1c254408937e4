// W4A8 GEMM, tiled form for many tokens (prefill): bound by the FP8 matrix
// cores.
//
//   Y[m,n] = (sx[m] c[n]) * sum_k a[m,k] * q[k,n] * 2^e[g(k),n]   (+ T.V, LoRC)
//
// (paper Sections 1 and 3.)  A workgroup of 4 waves (2 x 2) owns a BM x BN
// output tile; each wave owns WTM x WTN tiles of 16 x 16 and walks K in steps
// of 128 with v_mfma_scale_f32_16x16x128_f8f6f4 (A = E4M3 from LDS, B = packed
// E2M1 from LDS, B's E8M0 group exponent straight from global memory into the
// instruction's scale operand -- the FP4 -> FP8 alignment is done by the
// matrix core, no unpack and no multiply).
//
// LDS holds two stages.  A stage keeps the activation tile in "fragment order"
// (per 16-row sub-tile: 2 halves x 64 lanes x 16 B, lane = 16*(k/16 % 4) + row)
// so that every operand read is a conflict-free 16 B/lane read; the weight
// tile already has that order in memory and is copied as is.
#include "zqfp_internal.h"

namespace zqfp {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

__device__ inline uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int WTM, int WTN>
struct TileCfg {
    static constexpr int BM = 2 * WTM * 16, BN = 2 * WTN * 16;
    static constexpr int A_BYTES = BM * 128, B_BYTES = BN * 64;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int A_CHUNKS = A_BYTES / 16 / kThreads;  // 16 B chunks per thread
    static constexpr int B_CHUNKS = B_BYTES / 16 / kThreads;
};

template <int WTM, int WTN, bool EXACT>
__global__ __launch_bounds__(kThreads) void k_gemm_tile(const uint8_t* __restrict__ Xq, const float* __restrict__ sx,
                                                      int64_t M, const uint8_t* __restrict__ blob, BlobLayout L, Lorc lorc,
                                                      void* __restrict__ Y, int64_t ldy, int out_dtype, int tiles_m,
                                                      int tiles_n)
{
    using C = TileCfg<WTM, WTN>;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- workgroup -> tile.  Consecutive workgroup ids go to consecutive XCDs (8 of them, one
    // L2 each), so give every XCD a contiguous range of tiles, walked in column-panels of height 8
    // so that concurrently running workgroups of an XCD share activation and weight panels in L2.
    const int ntiles = tiles_m * tiles_n;
    int pid = blockIdx.x;
    {
        const int per = (ntiles + 7) / 8;
        const int xcd = pid & 7, loc = pid >> 3;
        int id = xcd * per + loc;
        if (id >= ntiles || loc >= per) return;
        pid = id;
    }
    constexpr int GROUP_M = 8;
    const int in_group = GROUP_M * tiles_n;
    const int gid = pid / in_group;
    const int first_m = gid * GROUP_M;
    const int gsz = min(tiles_m - first_m, GROUP_M);
    const int tm = first_m + (pid % in_group) % gsz;
    const int tn = (pid % in_group) / gsz;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int col = lane & 15, lb = lane >> 4;
    const int64_t m0 = (int64_t)tm * C::BM;
    const int64_t strip0 = (int64_t)tn * (C::BN / 16);
    const int nkt = (int)L.nkt;

    const uint8_t* codes = blob + L.off_codes;
    const uint32_t* exq = reinterpret_cast<const uint32_t*>(blob + L.off_exps);

    // ---- global -> register staging
    uint4 ra[C::A_CHUNKS], rb[C::B_CHUNKS];
    uint32_t re[WTN], e_cur[WTN];

    auto gload = [&](int kt) {
#pragma unroll
        for (int i = 0; i < C::A_CHUNKS; ++i) {
            const int cidx = tid + kThreads * i;
            const int r = cidx & 15, j = (cidx >> 4) & 7, sub = cidx >> 7;
            const int64_t m = m0 + sub * 16 + r;
            ra[i] = (m < M) ? *reinterpret_cast<const uint4*>(Xq + m * L.K + (int64_t)kt * 128 + 16 * j)
                            : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < C::B_CHUNKS; ++i) {
            const int cidx = tid + kThreads * i;
            const int64_t strip = strip0 + (cidx >> 6);
            rb[i] = (strip < L.nstrips)
                        ? *reinterpret_cast<const uint4*>(codes + ((strip * nkt + kt) * 64 + (cidx & 63)) * 16)
                        : make_uint4(0, 0, 0, 0);
        }
        const int blk = kt * 4 + lb;
        const int sg = (L.gsb_shift >= 0) ? (blk >> L.gsb_shift) : (blk / L.gsb);
#pragma unroll
        for (int j = 0; j < WTN; ++j) {
            const int64_t strip = strip0 + wn * WTN + j;
            re[j] = (strip < L.nstrips) ? (exq[(strip * L.ngq + (sg >> 2)) * 16 + col] >> (8 * (sg & 3))) : 127u;
        }
    };
    auto lstore = [&](int stage) {
        uint8_t* sa = smem + stage * C::STAGE;
        uint8_t* sb = sa + C::A_BYTES;
#pragma unroll
        for (int i = 0; i < C::A_CHUNKS; ++i) {
            const int cidx = tid + kThreads * i;
            const int r = cidx & 15, j = (cidx >> 4) & 7, sub = cidx >> 7;
            *reinterpret_cast<uint4*>(sa + sub * 2048 + (j >> 2) * 1024 + ((j & 3) * 16 + r) * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < C::B_CHUNKS; ++i) {
            const int cidx = tid + kThreads * i;
            *reinterpret_cast<uint4*>(sb + cidx * 16) = rb[i];
        }
    };

    v4f acc[WTM][WTN];
#pragma unroll
    for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

    gload(0);
    lstore(0);
#pragma unroll
    for (int j = 0; j < WTN; ++j) e_cur[j] = re[j];
    __syncthreads();

    for (int kt = 0; kt < nkt; ++kt) {
        const int stage = kt & 1;
        if (kt + 1 < nkt) gload(kt + 1);

        const uint8_t* sa = smem + stage * C::STAGE + (wm * WTM) * 2048 + lane * 16;
        const uint8_t* sb = smem + stage * C::STAGE + C::A_BYTES + (wn * WTN) * 1024 + lane * 16;
        v8i bfr[WTN];
#pragma unroll
        for (int j = 0; j < WTN; ++j) {
            uint4 b = *reinterpret_cast<const uint4*>(sb + j * 1024);
            bfr[j] = (v8i){(int)b.x, (int)b.y, (int)b.z, (int)b.w, 0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < WTM; ++i) {
            uint4 lo = *reinterpret_cast<const uint4*>(sa + i * 2048);
            uint4 hi = *reinterpret_cast<const uint4*>(sa + i * 2048 + 1024);
            v8i afr = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
            if constexpr (EXACT) {
                v8i hi, lo;
                split_exponent_bands(afr, hi, lo);
#pragma unroll
                for (int j = 0; j < WTN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(hi, bfr[j], acc[i][j], 0, 4, 0, 127, 0,
                                                                                  (int)e_cur[j]);
#pragma unroll
                for (int j = 0; j < WTN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(lo, bfr[j], acc[i][j], 0, 4, 0, 127, 0,
                                                                                  (int)e_cur[j]);
            } else {
#pragma unroll
                for (int j = 0; j < WTN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(afr, bfr[j], acc[i][j], 0, 4, 0, 127, 0,
                                                                                  (int)e_cur[j]);
            }
        }

        if (kt + 1 < nkt) {
            lstore(stage ^ 1);
#pragma unroll
            for (int j = 0; j < WTN; ++j) e_cur[j] = re[j];
        }
        __syncthreads();
    }

    // ---- epilogue: D[row][col] of a 16x16 tile sits in lane 16*(row/4)+col, register row%4
    const float* colscale = reinterpret_cast<const float*>(blob + L.off_colscale);
#pragma unroll
    for (int j = 0; j < WTN; ++j) {
        const int64_t n = (strip0 + wn * WTN + j) * 16 + col;
        if (n >= L.N) continue;
        const float cn = colscale[n];
        float v[8];
        for (int q = 0; q < lorc.r && q < 8; ++q) v[q] = half_bits_to_f32(lorc.V[(int64_t)q * L.N + n]);
#pragma unroll
        for (int i = 0; i < WTM; ++i) {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int64_t m = m0 + (wm * WTM + i) * 16 + 4 * lb + rg;
                if (m >= M) continue;
                float y = (sx[m] * cn) * acc[i][j][rg];
                if (lorc.r > 0) {
                    const float* t = lorc.T + m * lorc.r;
                    if (lorc.r <= 8) {
                        for (int q = 0; q < lorc.r; ++q) y = fmaf(t[q], v[q], y);
                    } else {
                        for (int q = 0; q < lorc.r; ++q)
                            y = fmaf(t[q], half_bits_to_f32(lorc.V[(int64_t)q * L.N + n]), y);
                    }
                }
                if (out_dtype == 0) reinterpret_cast<float*>(Y)[m * ldy + n] = y;
                else reinterpret_cast<uint16_t*>(Y)[m * ldy + n] = f32_to_bf16_bits(y);
            }
        }
    }
}

template <int WTM, int WTN, bool EXACT>
hipError_t launch_cfg(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L, Lorc lorc,
                      void* Y, int64_t ldy, int out_dtype, hipStream_t s)
{
    using C = TileCfg<WTM, WTN>;
    const int tiles_m = (int)((M + C::BM - 1) / C::BM), tiles_n = (int)((L.Np + C::BN - 1) / C::BN);
    const int ntiles = tiles_m * tiles_n;
    const int per = (ntiles + 7) / 8;
    const size_t smem = 2 * C::STAGE;
    auto kern = k_gemm_tile<WTM, WTN, EXACT>;
    static bool attr_done = false;  // raising the dynamic LDS limit is a per-function, per-process setting
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(per * 8)), dim3(kThreads), smem, s, Xq, sx, M, blob, L, lorc, Y, ldy,
                       out_dtype, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

bool gemm_tile_supported(int64_t M, const BlobLayout& L) { return M > 64 && L.N >= 64; }

hipError_t launch_gemm_tile(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L,
                            Lorc lorc, void* Y, int64_t ldy, int out_dtype, int accum, hipStream_t s)
{
    return accum == 0 ? launch_cfg<4, 4, true>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, s)
                      : launch_cfg<4, 4, false>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, s);
}

}  // namespace zqfp
