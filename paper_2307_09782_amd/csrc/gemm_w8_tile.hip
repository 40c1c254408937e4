// W8A8 GEMM (FP8 E4M3 activations x FP8 E4M3 weights with power-of-two group scales), tiled form for more
// than 64 tokens.
//
//   Y[m,n] = (sx[m] c[n]) * sum_k a[m,k] * w[k,n] * 2^e[g(k),n]   (+ T.V, LoRC)
//
// (paper Section 4, Table 2: the W8A8 rows with FP8 on both sides; group-wise weight scales as in Section 3,
// constrained to powers of two as in "Casting the FP4 to FP8", so that the block-scaled matrix instruction
// v_mfma_scale_f32_16x16x128_f8f6f4 applies them and no multiply touches the weights.)
//
// A workgroup of four waves (2 x 2) owns a 128 x 128 output tile; each wave 64 x 64 (4 x 4 blocks of 16 x 16)
// and walks K in steps of 128.  Two LDS stages: while a k-tile is multiplied the next one travels through
// registers into the other stage (plain loads, 16 bytes per lane; the compiler places the waits).  The
// activation tile is stored as rows of 128 bytes with XOR-swizzled 16-byte chunks (conflict-free operand
// reads), the weight tile as it lies in memory: per strip of 16 columns two contiguous 1 KB halves, each the
// first / second four registers of the B operand.  Written for correctness and reasonable speed, without the
// hand-placed waits of the FP4 kernel: the FP8 B operand needs twice the registers and twice the LDS traffic
// of the FP4 one, so the two do not share a schedule.
#include "zqfp_internal.h"

namespace zqfp {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBM = 128, kBN = 128, kThreads = 256;
constexpr int kABytes = kBM * 128, kBBytes = kBN * 128, kStage = kABytes + kBBytes;  // 32 KB
constexpr int kAChunks = kABytes / 16 / kThreads, kBChunks = kBBytes / 16 / kThreads;  // 4 and 4

template <bool EXACT>
__global__ __launch_bounds__(kThreads) void k_gemm_w8_tile(const uint8_t* __restrict__ Xq, const float* __restrict__ sx,
                                                         int64_t M, const uint8_t* __restrict__ blob, BlobLayout L,
                                                         Lorc lorc, void* __restrict__ Y, int64_t ldy, int out_dtype,
                                                         int tiles_m, int tiles_n)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];  // 2 stages; the epilogue reuses them
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int col = lane & 15, lb = lane >> 4;
    // consecutive workgroup ids sit on consecutive XCDs: give each XCD a contiguous range of tiles, walked
    // down the columns so that the workgroups of an XCD share weight panels in its L2
    const int ntiles = tiles_m * tiles_n;
    const int per = (ntiles + 7) / 8;
    const int id = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
    if (id >= ntiles) return;
    const int tn = id / tiles_m, tm = id - tn * tiles_m;
    const int64_t m0 = (int64_t)tm * kBM, strip0 = (int64_t)tn * (kBN / 16);
    const int nkt = (int)L.nkt;
    const int rows_here = (int)min((int64_t)kBM, M - m0);

    // ---- global -> register -> LDS staging.  Activation chunk i of thread t: row (t/8) + 32 i, 16-byte chunk
    // t % 8 of the row's 128 bytes, stored at slot chunk ^ (row % 8).  Rows past M repeat the last row (their
    // products are never stored).  Weight chunk i of thread t: 16-byte vector t + 256 i of the tile's
    // 8 strips x 2 KB, copied as is; strips past the last one repeat it.
    const uint8_t* a_src[kAChunks];
    uint32_t a_dst[kAChunks];
#pragma unroll
    for (int i = 0; i < kAChunks; ++i) {
        const int row = (tid >> 3) + 32 * i, chunk = tid & 7;
        a_src[i] = Xq + (m0 + min(row, rows_here - 1)) * L.K + 16 * chunk;
        a_dst[i] = (uint32_t)(row * 128 + ((chunk ^ (row & 7)) * 16));
    }
    const uint8_t* b_src[kBChunks];
#pragma unroll
    for (int i = 0; i < kBChunks; ++i) {
        const int v = tid + kThreads * i;  // 0..1023: strip v / 128, vector v % 128 of its 2 KB fragment
        const int64_t strip = min(strip0 + (v >> 7), L.nstrips - 1);
        b_src[i] = blob + L.off_codes + (strip * nkt) * 2048 + (v & 127) * 16;
    }
    // exponent dword of this lane's columns (one per 16-column block of the wave): groups are multiples of 128,
    // so every 32-block of a k-tile shares the byte of stored group kt / (Gs / 128)
    const uint32_t* ex[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t strip = min(strip0 + wn * 4 + j, L.nstrips - 1);
        ex[j] = reinterpret_cast<const uint32_t*>(blob + L.off_exps) + strip * L.ngq * 16 + col;
    }
    const int gq = L.gsb >> 2;  // k-tiles per stored group (>= 1)

    u32x4 ra[kAChunks], rb[kBChunks];
    auto fetch = [&](int kt) {
#pragma unroll
        for (int i = 0; i < kAChunks; ++i) ra[i] = *reinterpret_cast<const u32x4*>(a_src[i] + (int64_t)kt * 128);
#pragma unroll
        for (int i = 0; i < kBChunks; ++i) rb[i] = *reinterpret_cast<const u32x4*>(b_src[i] + (int64_t)kt * 2048);
    };
    auto stash = [&](int stage) {
        uint8_t* st = smem + stage * kStage;
#pragma unroll
        for (int i = 0; i < kAChunks; ++i) *reinterpret_cast<u32x4*>(st + a_dst[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < kBChunks; ++i) *reinterpret_cast<u32x4*>(st + kABytes + (tid + kThreads * i) * 16) = rb[i];
    };

    v4f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < nkt; ++kt) {
        const int stage = kt & 1;
        if (kt + 1 < nkt) fetch(kt + 1);  // in flight while this k-tile is multiplied
        const uint8_t* st = smem + stage * kStage;
        const int sg = kt / gq;
        // weight fragments and their exponent bytes: four column blocks, kept for all four row blocks
        v8i bv[4];
        int sc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint8_t* f = st + kABytes + (wn * 4 + j) * 2048 + lane * 16;
            const u32x4 h0 = *reinterpret_cast<const u32x4*>(f), h1 = *reinterpret_cast<const u32x4*>(f + 1024);
            bv[j] = (v8i){(int)h0[0], (int)h0[1], (int)h0[2], (int)h0[3], (int)h1[0], (int)h1[1], (int)h1[2], (int)h1[3]};
            sc[j] = (int)(ex[j][(sg >> 2) * 16] >> (8 * (sg & 3)));
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = (wm * 4 + i) * 16 + col;
            const uint8_t* r = st + row * 128;
            const u32x4 a0 = *reinterpret_cast<const u32x4*>(r + ((lb ^ (row & 7)) * 16));
            const u32x4 a1 = *reinterpret_cast<const u32x4*>(r + (((lb + 4) ^ (row & 7)) * 16));
            const v8i av = {(int)a0[0], (int)a0[1], (int)a0[2], (int)a0[3], (int)a1[0], (int)a1[1], (int)a1[2], (int)a1[3]};
            // cbsz 0, blgp 0: E4M3 on both sides; A scale byte 127 = 2^0; B scale = the group's exponent byte
            if constexpr (EXACT) {
                v8i hi, lo;
                split_exponent_bands(av, hi, lo);
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(hi, bv[j], acc[i][j], 0, 0, 0, 127, 0, sc[j]);
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(lo, bv[j], acc[i][j], 0, 0, 0, 127, 0, sc[j]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv[j], acc[i][j], 0, 0, 0, 127, 0, sc[j]);
            }
        }
        if (kt + 1 < nkt) stash(stage ^ 1);  // nobody reads that stage: its last readers passed the barrier below one step ago
        __syncthreads();
    }

    // ---- epilogue.  D[row][col] of a 16 x 16 block sits in lane 16 (row / 4) + col, register row % 4.  LoRC of
    // rank <= 8: the tile's rows of T and columns of V go through LDS once (zero-padded to 8).
    constexpr int RL = 8;
    float* Ts = reinterpret_cast<float*>(smem);  // [kBM][RL]
    float* Vs = Ts + kBM * RL;                   // [kBN][RL]
    const int rk = lorc.r;
    const bool lorc_lds = rk > 0 && rk <= RL;
    if (lorc_lds) {  // (the loop's last barrier has passed: the stages are free)
        for (int idx = tid; idx < kBM * RL; idx += kThreads) {
            const int row = idx / RL, q = idx % RL;
            Ts[idx] = q < rk ? lorc.T[min(m0 + row, M - 1) * rk + q] : 0.f;
        }
        for (int idx = tid; idx < RL * kBN; idx += kThreads) {
            const int q = idx / kBN, c = idx % kBN;
            const int64_t n = min(strip0 * 16 + c, L.N - 1);
            Vs[c * RL + q] = q < rk ? half_bits_to_f32(lorc.V[(int64_t)q * L.N + n]) : 0.f;
        }
        __syncthreads();
    }
    const float* colscale = reinterpret_cast<const float*>(blob + L.off_colscale);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t n = (strip0 + wn * 4 + j) * 16 + col;
        const float cn = colscale[min(n, L.Np - 1)];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int lrow = (wm * 4 + i) * 16 + 4 * lb + rg;
                const int64_t m = m0 + lrow;
                if (m >= M || n >= L.N) continue;
                float y = (sx[m] * cn) * acc[i][j][rg];
                if (lorc_lds) {
#pragma unroll
                    for (int q = 0; q < RL; ++q) y = fmaf(Ts[lrow * RL + q], Vs[((wn * 4 + j) * 16 + col) * RL + q], y);
                } else {
                    for (int q = 0; q < rk; ++q) y = fmaf(lorc.T[m * rk + q], half_bits_to_f32(lorc.V[(int64_t)q * L.N + n]), y);
                }
                if (out_dtype == 0) reinterpret_cast<float*>(Y)[m * ldy + n] = y;
                else reinterpret_cast<uint16_t*>(Y)[m * ldy + n] = f32_to_bf16_bits(y);
            }
        }
    }
}

}  // namespace

hipError_t launch_gemm_w8_tile(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L,
                               Lorc lorc, void* Y, int64_t ldy, int out_dtype, int accum, hipStream_t s)
{
    if (M == 0 || L.N == 0) return hipSuccess;
    const int tiles_m = (int)((M + kBM - 1) / kBM), tiles_n = (int)((L.Np + kBN - 1) / kBN);
    const int per = (tiles_m * tiles_n + 7) / 8;
    const size_t smem = 2 * kStage;  // 64 KB: above the default dynamic-LDS limit
    static OnceStatus attr;
    if (hipError_t e = run_once(attr, [&] {
            hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_w8_tile<true>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e1 != hipSuccess) return e1;
            return hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_w8_tile<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        }); e != hipSuccess)
        return e;
    if (accum == 0)
        hipLaunchKernelGGL(k_gemm_w8_tile<true>, dim3((unsigned)(per * 8)), dim3(kThreads), smem, s, Xq, sx, M, blob, L, lorc, Y,
                           ldy, out_dtype, tiles_m, tiles_n);
    else
        hipLaunchKernelGGL(k_gemm_w8_tile<false>, dim3((unsigned)(per * 8)), dim3(kThreads), smem, s, Xq, sx, M, blob, L, lorc, Y,
                           ldy, out_dtype, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace zqfp
