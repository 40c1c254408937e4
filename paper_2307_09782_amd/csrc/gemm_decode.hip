// W4A8 GEMM for at most 16 tokens (decode): a persistent weight-streaming
// kernel, bound by reading the packed FP4 weights once from HBM.
//
//   Y[m,n] = (sx[m] c[n]) * sum_k a[m,k] * q[k,n] * 2^e[g(k),n]   (+ T.V, LoRC)
//
// (paper Sections 1 and 3.)  One workgroup of NW = 8 or 16 waves per compute unit
// walks over strips of 16 output channels.  Wave w owns the k-tiles w, w+NW, ... of
// every strip, so its activation fragments (the A operands of
// v_mfma_scale_f32_16x16x128_f8f6f4) are loaded ONCE and stay in registers for the whole
// kernel; the only traffic in the loop is the weight stream: one contiguous
// 1 KB fragment per matrix instruction plus its exponent dword.  The fragments
// of the next strip are in flight while the current strip is multiplied,
// reduced across the waves in LDS (fixed order, no atomics) and stored.
#include <atomic>

#include "zqfp_internal.h"

namespace zqfp {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));


// NW: waves per workgroup (8 or 16); KPW: k-tiles per wave (K / 128 / NW, rounded up); NB: fragment
// buffers, i.e. NB - 1 strips in flight behind the one being multiplied.  One workgroup per compute
// unit: NW / 4 waves per SIMD.
// FUSED: the activations arrive as bfloat16 and are quantized here, token-wise to E4M3 (paper Section 3), in the
// same binary32 sequence as the stand-alone quantizer: every workgroup reads the M x K bfloat16 rows once
// (wave w the slices of its own k-tiles), the row maxima meet in LDS, and each wave encodes its own fragments in
// registers.  One kernel instead of two for a decode step; workgroup 0 also writes the codes and scales out
// when the caller asks for them.
struct FusedIn {
    const uint16_t* X;  // [M, K] bf16, row stride ldx
    int64_t ldx;
    uint8_t* Xq_out;    // [M, K] E4M3 codes, or null
    float* sx_out;      // [M], or null
};

// WB: weight bits.  8 = E4M3 weights (the W8A8 rows of the paper's Table 2 with FP8 on both sides): a strip's
// k-tile is then two 1 KB halves, the first and second four registers of the B operand.
template <int NW, int KPW, int NB, bool EXACT, bool LR, bool FUSED = false, int WB = 4>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(NW / 4, NW / 4))) void k_gemm_decode(
    const uint8_t* __restrict__ Xq, const float* __restrict__ sx, int M, const uint8_t* __restrict__ blob, BlobLayout L,
    Lorc lorc, void* __restrict__ Y, int64_t ldy, int out_dtype, int nchunks, int chunk_len, float* __restrict__ partial,
    FusedIn fin)
{
    constexpr int kWaves = NW;
    constexpr bool HI_LDS = EXACT && KPW >= 8;
    static_assert(!FUSED || (KPW <= 4 && !LR), "the fused form keeps a wave's bfloat16 slices in registers and has no LoRC");
    __shared__ float s_red[2][kWaves][64][4];
    __shared__ uint32_t s_rowmax[FUSED ? kWaves : 1][16];
    __shared__ float s_scale[FUSED ? 16 : 1];
    extern __shared__ __attribute__((aligned(16))) uint8_t s_hi[];  // HI_LDS: NW * KPW * 2048 bytes

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: fragment addresses stay in SGPRs
    const int col = lane & 15, lb = lane >> 4;
    const int64_t nstrips = L.nstrips;
    // A K of more than 64 k-tiles is served in chunks: workgroup b takes chunk b % nchunks, multiplies
    // its k-tiles kt0 .. kt0 + nkt only and leaves raw float32 sums in slice `chunk` of the workspace.
    const int nkt_all = (int)L.nkt;
    const int chunk = nchunks > 1 ? (int)(blockIdx.x % nchunks) : 0;
    const int kt0 = chunk * chunk_len;
    const int nkt = min(chunk_len, nkt_all - kt0);
    const bool raw = nchunks > 1;
    if (raw) {
        Y = partial + (int64_t)chunk * M * L.Np;
        ldy = L.Np;
        out_dtype = 0;
    }

    // ---- activation fragments: lane (row = lane%16, lb) holds bytes k = 16*lb + [0,16) and
    // k = 64 + 16*lb + [0,16) of each of its k-tiles.  The loads are unconditional: a row past M
    // repeats row M - 1 (row m of the product depends on row m of A only, and rows past M are
    // never stored), a k-tile past the end repeats the last one and is zeroed further down, once
    // the first strips' weight loads have been issued behind these.
    u32x4 ax0[KPW], ax1[KPW];
    uint4 xb[FUSED ? KPW : 1][4];  // FUSED: the lane's 32 bfloat16 of k-tile u (k = 16 lb + [0,16) and 64 + 16 lb + [0,16))
    // The fragments are filled from ax0/ax1 below.  In the exact mode they are split into their two
    // exponent bands once (they serve every strip): afr holds the lower band, ahi the upper one,
    // or, when 8 k-tiles per wave leave no registers for it, the wave's own slice of LDS does.
    v8i afr[KPW];
    v8i ahi[(EXACT && !HI_LDS) ? KPW : 1];
#pragma unroll
    for (int u = 0; u < KPW; ++u) {
        const int kt = min(wave + kWaves * u, nkt - 1);
        if constexpr (FUSED) {
            const uint4* p = reinterpret_cast<const uint4*>(fin.X + (int64_t)min(col, M - 1) * fin.ldx + (int64_t)(kt0 + kt) * 128 + 16 * lb);
            xb[u][0] = p[0]; xb[u][1] = p[1];  // k = 16 lb + [0, 16)
            xb[u][2] = p[8]; xb[u][3] = p[9];  // 64 elements (128 bytes) further on
        } else {
            const uint8_t* p = Xq + (int64_t)min(col, M - 1) * L.K + (int64_t)(kt0 + kt) * 128 + 16 * lb;
            ax0[u] = *reinterpret_cast<const u32x4*>(p);
            ax1[u] = *reinterpret_cast<const u32x4*>(p + 64);
        }
    }
    // stored exponent group of this lane's 32-block of its u-th k-tile (recomputed where needed:
    // a few integer operations, cheaper than holding it in registers)
    const bool small_groups = L.gsb < 4;  // groups of 32 or 64: a shift; else one group per k-tile
    auto stored_group = [&](int u) {
        const int kt = kt0 + min(wave + kWaves * u, nkt - 1);
        const int a = (kt * 4 + lb) >> (small_groups ? L.gsb_shift : 0);
        const int b = (int)(((uint32_t)kt * L.gq_magic) >> 20);  // kt / (gsb / 4)
        return small_groups ? a : b;
    };

    const uint8_t* codes = blob + L.off_codes;
    const uint32_t* exq = reinterpret_cast<const uint32_t*>(blob + L.off_exps);
    const float* colscale = reinterpret_cast<const float*>(blob + L.off_colscale);

    u32x4 b[NB][KPW];
    u32x4 bh[WB == 8 ? NB : 1][KPW];  // E4M3 weights: the fragments' second halves
    uint32_t e[NB][KPW];

    // ---- epilogue operands.  Thread t (mod 256) owns output (row t / 16, column t % 16) of every
    // strip: its token scale and LoRC row are loaded once; the column scale and the LoRC column
    // of a strip travel with that strip's fragments, so that no load sits on the path between
    // the reduction and the store.  Every load of the loop is unconditional (addresses are clamped
    // into valid memory instead) and its value is left raw until it is used: the load counter can
    // then be waited on exactly, and a strip's operands never wait for the next strip's.
    constexpr int RMAX = 8;  // LoRC ranks up to 8 are held in registers, larger ones are read in place
    const int er = (tid >> 4) & 15, ec = tid & 15;
    const bool row_live = tid < 256 && er < M;
    const int rk = lorc.r;
    float sx_r = (raw || FUSED) ? 1.0f : sx[min(er, M - 1)], t_r[RMAX];  // raw: scales are applied when the chunks are added up; FUSED: set below
#pragma unroll
    for (int j = 0; j < RMAX; ++j) t_r[j] = 0.f;
    if constexpr (LR) {
#pragma unroll
        for (int j = 0; j < RMAX; ++j) t_r[j] = lorc.T[min(er, M - 1) * rk + min(j, rk - 1)];  // j >= rk: unused
    }
    float cs[NB];
    uint32_t vv[NB][RMAX];  // binary16 bits
#pragma unroll
    for (int r = 0; r < NB; ++r)
#pragma unroll
        for (int j = 0; j < RMAX; ++j) vv[r][j] = 0u;

    auto issue = [&](int buf, int64_t strip_unclamped) {
        const int64_t strip = min(strip_unclamped, nstrips - 1);  // past the end: the last strip again, never used
#pragma unroll
        for (int u = 0; u < KPW; ++u) {
            const int kt = min(wave + kWaves * u, nkt - 1);  // clamped duplicates are multiplied by zero fragments
            if constexpr (WB == 8) {
                const u32x4* f = reinterpret_cast<const u32x4*>(codes + ((strip * nkt_all + kt0 + kt) << 11));
                b[buf][u] = f[lane];
                bh[buf][u] = f[64 + lane];
            } else {
                b[buf][u] = reinterpret_cast<const u32x4*>(codes + ((strip * nkt_all + kt0 + kt) << 10))[lane];
            }
            e[buf][u] = (exq + strip * L.ngq * 16)[(stored_group(u) >> 2) * 16 + col];
        }
        const int64_t n = min(strip * 16 + ec, L.N - 1);
        cs[buf] = colscale[n];
        if constexpr (LR) {
#pragma unroll
            for (int j = 0; j < RMAX; ++j) vv[buf][j] = lorc.V[(int64_t)min(j, rk - 1) * L.N + n];
        }
    };
    auto finish = [&](int buf, int64_t strip, int par) {
        // independent accumulator chains (two; four in the exact mode, one pair per exponent band):
        // a matrix instruction that waits for the previous one's result costs its full latency
        v4f acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f}, acc3 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < KPW; ++u) {
            v8i bv = {(int)b[buf][u][0], (int)b[buf][u][1], (int)b[buf][u][2], (int)b[buf][u][3], 0, 0, 0, 0};
            if constexpr (WB == 8) {
                bv[4] = (int)bh[buf][u][0]; bv[5] = (int)bh[buf][u][1]; bv[6] = (int)bh[buf][u][2]; bv[7] = (int)bh[buf][u][3];
            }
            constexpr int BLGP = WB == 8 ? 0 : 4;  // B is E4M3 or E2M1
            const int sc = (int)(e[buf][u] >> (8 * (stored_group(u) & 3)));
            v4f& acc = (u & 1) ? acc1 : acc0;
            // cbsz 0: A is E4M3; A scale byte 127 = 2^0; B scale = group exponent
            if constexpr (EXACT) {
                v4f& accl = (u & 1) ? acc3 : acc2;
                v8i hi;
                if constexpr (HI_LDS) {
                    const u32x4 h0 = *reinterpret_cast<const u32x4*>(s_hi + ((wave * KPW + u) * 128 + lane) * 16);
                    const u32x4 h1 = *reinterpret_cast<const u32x4*>(s_hi + ((wave * KPW + u) * 128 + 64 + lane) * 16);
                    hi = (v8i){(int)h0[0], (int)h0[1], (int)h0[2], (int)h0[3], (int)h1[0], (int)h1[1], (int)h1[2], (int)h1[3]};
                } else {
                    hi = ahi[u];
                }
                acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(hi, bv, acc, 0, BLGP, 0, 127, 0, sc);
                accl = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(afr[u], bv, accl, 0, BLGP, 0, 127, 0, sc);
            } else {
                acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(afr[u], bv, acc, 0, BLGP, 0, 127, 0, sc);
            }
        }
        *reinterpret_cast<v4f*>(&s_red[par][wave][lane][0]) = EXACT ? (acc0 + acc1) + (acc2 + acc3) : acc0 + acc1;
        __syncthreads();
        // D[row][col] sits in lane 16*(row/4)+col, register row%4.  Every thread sums (the upper
        // half of the workgroup repeats the lower half's work): only the store is predicated, so
        // the loop body stays one basic block and the load counters stay exact.
        const int64_t n = strip * 16 + ec;
        const int src = 16 * (er >> 2) + ec, reg = er & 3;
        float a = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) a += s_red[par][w][src][reg];
        float y = (sx_r * (raw ? 1.0f : cs[buf])) * a;
        if constexpr (LR) {
#pragma unroll
            for (int j = 0; j < RMAX; ++j) y = fmaf(t_r[j], j < rk ? half_bits_to_f32((uint16_t)vv[buf][j]) : 0.f, y);
        }
        if (row_live && n < L.N) {
            if (!LR && rk > 0)  // ranks not held in registers: read in place
                for (int j = 0; j < rk; ++j)
                    y = fmaf(lorc.T[er * rk + j], half_bits_to_f32(lorc.V[(int64_t)j * L.N + n]), y);
            if (out_dtype == 0) reinterpret_cast<float*>(Y)[er * ldy + n] = y;
            else reinterpret_cast<uint16_t*>(Y)[er * ldy + n] = f32_to_bf16_bits(y);
        }
    };

    // ---- strips blockIdx.x, + gridDim.x, ...; NB - 1 strips are in flight behind the current one.
    // The loop is unrolled by NB so that the fragment buffers are addressed statically.  The LDS
    // reduction buffer alternates per strip: it is rewritten two strips later, after a barrier
    // that every reader has passed.
    // Strip order.  Consecutive workgroup ids sit on consecutive XCDs (8 of them, one L2 each).  A
    // strip's 16 output columns are half a 128-byte line of every row of Y, so the two strips of a
    // line go to the same XCD, to neighbouring workgroups in the same step: its L2 then merges the
    // halves and writes whole lines.  Workgroup (xcd, loc) walks q = loc, loc + grid/8, ... of its
    // XCD's list, whose entry q is strip 2 * (8 * (q / 2) + xcd) + q % 2 (increasing in q).
    const bool paired = nchunks == 1 && (gridDim.x & 7) == 0;
    const int64_t stride = paired ? gridDim.x >> 3 : gridDim.x / nchunks;
    int64_t q = paired ? blockIdx.x >> 3 : blockIdx.x / nchunks;
    const int xcd = blockIdx.x & 7;
    auto strip_of = [&](int64_t qq) { return paired ? 2 * (8 * (qq >> 1) + xcd) + (qq & 1) : qq; };
#pragma unroll
    for (int r = 0; r < NB - 1; ++r) issue(r, strip_of(q + r * stride));
    if constexpr (FUSED) {
        // token maxima: this lane's, then the four lanes of its row (same lane % 16), then the waves through LDS
        uint32_t am = 0;
#pragma unroll
        for (int u = 0; u < KPW; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) am = absmax_bits(am, xb[u][c]);  // duplicates of the last k-tile change nothing
        am = max(am, (uint32_t)__shfl_xor((int)am, 16));
        am = max(am, (uint32_t)__shfl_xor((int)am, 32));
        if (lane < 16) s_rowmax[wave][lane] = am;
        __syncthreads();
        am = s_rowmax[0][col];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) am = max(am, s_rowmax[w][col]);
        float scale, inv;
        token_scale(am, scale, inv);
        if (tid < 16) s_scale[tid] = scale;  // tid < 16: lane == col == row
        const bool write_out = blockIdx.x == 0 && col < M;
        if (write_out && fin.sx_out != nullptr && tid < 16) fin.sx_out[col] = scale;
#pragma unroll
        for (int u = 0; u < KPW; ++u) {
            const uint2 c0 = encode8(xb[u][0], inv), c1 = encode8(xb[u][1], inv);
            const uint2 c2 = encode8(xb[u][2], inv), c3 = encode8(xb[u][3], inv);
            ax0[u] = (u32x4){c0.x, c0.y, c1.x, c1.y};
            ax1[u] = (u32x4){c2.x, c2.y, c3.x, c3.y};
            if (write_out && fin.Xq_out != nullptr && wave + kWaves * u < nkt) {
                uint8_t* p = fin.Xq_out + (int64_t)col * L.K + (int64_t)(kt0 + wave + kWaves * u) * 128 + 16 * lb;
                *reinterpret_cast<u32x4*>(p) = ax0[u];
                *reinterpret_cast<u32x4*>(p + 64) = ax1[u];
            }
        }
        __syncthreads();
        sx_r = s_scale[er];
    }
#pragma unroll
    for (int u = 0; u < KPW; ++u) {
        const bool live = wave + kWaves * u < nkt;  // uniform
        const u32x4 x0 = live ? ax0[u] : (u32x4){0u, 0u, 0u, 0u}, x1 = live ? ax1[u] : (u32x4){0u, 0u, 0u, 0u};
        const v8i a = {(int)x0[0], (int)x0[1], (int)x0[2], (int)x0[3], (int)x1[0], (int)x1[1], (int)x1[2], (int)x1[3]};
        if constexpr (EXACT) {
            v8i hi;
            split_exponent_bands(a, hi, afr[u]);
            if constexpr (HI_LDS) {
                *reinterpret_cast<u32x4*>(s_hi + ((wave * KPW + u) * 128 + lane) * 16) = (u32x4){(uint32_t)hi[0], (uint32_t)hi[1], (uint32_t)hi[2], (uint32_t)hi[3]};
                *reinterpret_cast<u32x4*>(s_hi + ((wave * KPW + u) * 128 + 64 + lane) * 16) = (u32x4){(uint32_t)hi[4], (uint32_t)hi[5], (uint32_t)hi[6], (uint32_t)hi[7]};
            } else {
                ahi[u] = hi;
            }
        } else {
            afr[u] = a;
        }
    }
    int par = 0;
    while (true) {
#pragma unroll
        for (int r = 0; r < NB; ++r) {
            issue((r + NB - 1) % NB, strip_of(q + (NB - 1) * stride));
            __builtin_amdgcn_sched_barrier(0);
            finish(r, strip_of(q), par);
            __builtin_amdgcn_sched_barrier(0);
            par ^= 1;
            q += stride;
            if (strip_of(q) >= nstrips) return;
        }
    }
}

template <int NW, int KPW, int NB, int WB = 4>
hipError_t launch_kpw(unsigned grid, bool exact, const uint8_t* Xq, const float* sx, int M, const uint8_t* blob,
                const BlobLayout& L, Lorc lorc, void* Y, int64_t ldy, int out_dtype, int nchunks, int chunk_len,
                float* partial, const FusedIn& fin, hipStream_t s)
{
    // LoRC operands of ranks up to 8 are held in registers
    const bool lr = lorc.r > 0 && lorc.r <= 8;
    // the exact mode with 8 k-tiles per wave keeps the upper-band fragments in LDS (above the 64 KB
    // default limit of dynamic LDS, which is a per-function setting)
    const size_t smem = (exact && KPW >= 8) ? (size_t)NW * KPW * 2048 : 0;
    if (smem > 0) {
        static OnceStatus raised;
        if (hipError_t e = run_once(raised, [&] {
                hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_decode<NW, KPW, NB, true, false, false, WB>),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
                if (e1 != hipSuccess) return e1;
                return hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_decode<NW, KPW, NB, true, true, false, WB>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            }); e != hipSuccess)
            return e;
    }
#define ZQ_LAUNCH(EX, LR, FU) \
    hipLaunchKernelGGL((k_gemm_decode<NW, KPW, NB, EX, LR, FU, WB>), dim3(grid), dim3(64 * NW), smem, s, Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, nchunks, chunk_len, partial, fin)
    if (fin.X != nullptr) {
        if constexpr (KPW <= 4 && WB == 4) {
            if (exact) ZQ_LAUNCH(true, false, true); else ZQ_LAUNCH(false, false, true);
        } else {
            return hipErrorInvalidValue;  // not reached: the caller checks gemm_decode_fused_supported
        }
    } else if (exact) { if (lr) ZQ_LAUNCH(true, true, false); else ZQ_LAUNCH(true, false, false); }
    else       { if (lr) ZQ_LAUNCH(false, true, false); else ZQ_LAUNCH(false, false, false); }
#undef ZQ_LAUNCH
    return hipGetLastError();
}

}  // namespace

std::atomic<int> g_decode_waves{8};  // tuning hook: waves per workgroup of the decode form (8 or 16)
void force_decode_waves(int nw) { g_decode_waves.store(nw == 16 ? 16 : 8); }

// compute units of the (single) device, asked once
int compute_units()
{
    static std::atomic<int> cus{0};
    int n = cus.load(std::memory_order_relaxed);
    if (n == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cus.store(n, std::memory_order_relaxed);
    }
    return n;
}

bool gemm_decode_supported(int64_t M, const BlobLayout& L, const void* workspace)
{
    if (M < 1 || M > 16) return false;
    if (L.nkt <= 64) return true;
    if (plan_decode(L.nkt).chunks > compute_units()) return false;  // every chunk needs a workgroup of its own
    // longer K: in chunks through the workspace, if there are strips enough to give every workgroup
    // several (below that the streaming kernel, one launch and no prologue per chunk, is faster)
    return workspace != nullptr && L.nstrips * plan_decode(L.nkt).chunks >= 1024;
}

// E4M3 weights, at most 16 tokens and 40 k-tiles: a fragment is twice the registers of an FP4 one, so a wave holds at
// most five k-tiles (with two fragment buffers) before it spills, and there are no chunks (the W8A8 entry point takes
// no workspace).  Longer K stays with the streaming kernel.
bool gemm_w8_decode_supported(int64_t M, const BlobLayout& L) { return M >= 1 && M <= 16 && L.nkt <= 40 && L.N >= 16; }

hipError_t launch_gemm_w8_decode(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L,
                                 Lorc lorc, void* Y, int64_t ldy, int out_dtype, int accum, hipStream_t s)
{
    const FusedIn fin{nullptr, 0, nullptr, nullptr};
    if (L.N == 0) return hipSuccess;
    const int cus = compute_units();
    const bool exact = accum == 0;
    const int m = (int)M, len = (int)L.nkt;
    const unsigned grid = (unsigned)(L.nstrips < cus ? L.nstrips : cus);
#define ZQ_W8(KPW, NB) launch_kpw<8, KPW, NB, 8>(grid, exact, Xq, sx, m, blob, L, lorc, Y, ldy, out_dtype, 1, len, nullptr, fin, s)
    if (len <= 8) return ZQ_W8(1, 4);
    if (len <= 16) return ZQ_W8(2, 4);
    if (len <= 24) return ZQ_W8(3, 3);
    if (len <= 32) return ZQ_W8(4, 2);
    return ZQ_W8(5, 2);
#undef ZQ_W8
}

bool gemm_decode_fused_supported(int64_t M, const BlobLayout& L, int r)
{
    return M >= 1 && M <= 16 && L.nkt <= 32 && r == 0;  // at most 4 k-tiles per wave, no LoRC
}

hipError_t launch_gemm_decode(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L,
                              Lorc lorc, void* Y, int64_t ldy, int out_dtype, int accum, void* workspace, hipStream_t s,
                              const uint16_t* X, int64_t ldx, uint8_t* Xq_out, float* sx_out)
{
    const FusedIn fin{X, ldx, Xq_out, sx_out};
    if (L.N == 0) return hipSuccess;
    const int cus = compute_units();
    const bool exact = accum == 0;
    const int m = (int)M;
    const DecodePlan plan = plan_decode(L.nkt);
    const int nch = plan.chunks, len = plan.len;
    float* partial = nch > 1 ? static_cast<float*>(workspace) : nullptr;
    const Lorc none{nullptr, nullptr, 0};
    const Lorc lk = nch > 1 ? none : lorc;  // with chunks, LoRC is added when they are summed
    // one persistent workgroup per compute unit, the same number for every chunk
    const int64_t per_chunk = L.nstrips < cus / nch ? L.nstrips : cus / nch;
    const unsigned grid = (unsigned)(per_chunk * nch);
    hipError_t e;
    // 16 waves (four per SIMD) where a wave then owns at most two k-tiles: more loads in flight per compute unit
    if (g_decode_waves.load(std::memory_order_relaxed) == 16 && len <= 32) {
        if (len <= 16) e = launch_kpw<16, 1, 4>(grid, exact, Xq, sx, m, blob, L, lk, Y, ldy, out_dtype, nch, len, partial, fin, s);
        else e = launch_kpw<16, 2, 4>(grid, exact, Xq, sx, m, blob, L, lk, Y, ldy, out_dtype, nch, len, partial, fin, s);
    } else
    if (len <= 8) e = launch_kpw<8, 1, 4>(grid, exact, Xq, sx, m, blob, L, lk, Y, ldy, out_dtype, nch, len, partial, fin, s);
    else if (len <= 16) e = launch_kpw<8, 2, 4>(grid, exact, Xq, sx, m, blob, L, lk, Y, ldy, out_dtype, nch, len, partial, fin, s);
    else if (len <= 24) e = launch_kpw<8, 3, 4>(grid, exact, Xq, sx, m, blob, L, lk, Y, ldy, out_dtype, nch, len, partial, fin, s);
    else if (len <= 32) e = launch_kpw<8, 4, 4>(grid, exact, Xq, sx, m, blob, L, lk, Y, ldy, out_dtype, nch, len, partial, fin, s);
    else if (len <= 40) e = launch_kpw<8, 5, 3>(grid, exact, Xq, sx, m, blob, L, lk, Y, ldy, out_dtype, nch, len, partial, fin, s);
    else if (len <= 48) e = launch_kpw<8, 6, 2>(grid, exact, Xq, sx, m, blob, L, lk, Y, ldy, out_dtype, nch, len, partial, fin, s);
    else if (len <= 56) e = launch_kpw<8, 7, 2>(grid, exact, Xq, sx, m, blob, L, lk, Y, ldy, out_dtype, nch, len, partial, fin, s);
    else e = launch_kpw<8, 8, 2>(grid, exact, Xq, sx, m, blob, L, lk, Y, ldy, out_dtype, nch, len, partial, fin, s);
    if (e != hipSuccess || nch == 1) return e;
    return launch_splitk_reduce(partial, nch, M, blob, L, sx, lorc, Y, ldy, out_dtype, s);
}

}  // namespace zqfp
