// Token-wise FP8 (E4M3) activation quantizer, with the optional LoRC left
// factor T = X.U computed in the same sweep (paper Section 3: token-wise
// activation quantization, LoRC; Appendix A).  The normalisation whose output
// the quantizer sees (Section 3 names the layer normalisation in front of the
// quantized linear layers; LLaMA uses the RMS form) can run in the same sweep.
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

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

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

// two binary32 values -> two bf16 in one dword (round to nearest even): the packed hardware conversion
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack_bf16_rne(float lo, float hi)
{
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}


// 8 bf16 -> 8 bf16: (x * rstd) * g, each product one binary32 operation, rounded to bf16
__device__ inline uint4 normalize8(uint4 v, uint4 g, float rstd)
{
    uint32_t w[4] = {v.x, v.y, v.z, v.w}, gw[4] = {g.x, g.y, g.z, g.w}, o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo = (bf16_lo(w[i]) * rstd) * bf16_lo(gw[i]);
        const float hi = (bf16_hi(w[i]) * rstd) * bf16_hi(gw[i]);
        o[i] = pack_bf16_rne(lo, hi);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}

// 8 bf16 -> 8 bf16: ((x - mu) * rstd) * g + b, four separately rounded binary32 operations (the
// product and the sum must not fuse into one), rounded to bf16
__device__ inline uint4 normalize8_affine(uint4 v, uint4 g, uint4 b, float mu, float rstd)
{
#pragma clang fp contract(off)
    uint32_t w[4] = {v.x, v.y, v.z, v.w}, gw[4] = {g.x, g.y, g.z, g.w}, bw[4] = {b.x, b.y, b.z, b.w}, o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float dl = bf16_lo(w[i]) - mu, dh = bf16_hi(w[i]) - mu;
        const float al = dl * rstd, ah = dh * rstd;
        const float cl = al * bf16_lo(gw[i]), ch = ah * bf16_hi(gw[i]);
        const float lo = cl + bf16_lo(bw[i]), hi = ch + bf16_hi(bw[i]);
        o[i] = pack_bf16_rne(lo, hi);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}

// 8 bf16 + 8 bf16 -> 8 bf16: one binary32 addition each, rounded to bf16
__device__ inline uint4 add8(uint4 x, uint4 r)
{
    uint32_t xw[4] = {x.x, x.y, x.z, x.w}, rw[4] = {r.x, r.y, r.z, r.w}, o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        o[i] = pack_bf16_rne(bf16_lo(xw[i]) + bf16_lo(rw[i]), bf16_hi(xw[i]) + bf16_hi(rw[i]));
    return make_uint4(o[0], o[1], o[2], o[3]);
}

// ReLU on 8 bf16: a value passes unmodified if it is greater than zero, anything else becomes +0
__device__ inline uint4 relu8(uint4 x)
{
    uint32_t w[4] = {x.x, x.y, x.z, x.w}, o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        o[i] = (bf16_lo(w[i]) > 0.0f ? (w[i] & 0xFFFFu) : 0u) | (bf16_hi(w[i]) > 0.0f ? (w[i] & 0xFFFF0000u) : 0u);
    return make_uint4(o[0], o[1], o[2], o[3]);
}

// silu(g) * u = g / (1 + exp(-g)) * u as the binary32 value whose rounding to bf16 (nearest even) equals
// that of the expression evaluated in binary64 and rounded to binary32 first.
// Fast path, binary32 throughout: for 2^-30 <= |g| <= 32 and 2^-30 <= |u| <= 2^30 every intermediate
// is a normal number (exp(-g) in 2^+-47, the quotient above 2^-77, the product in 2^-107 .. 2^35), so
// the relative error is bounded by that of expf (documented as 1 ulp, taken as 4), of the hardware
// reciprocal (1 ulp) and three roundings: 13 * 2^-24 in all, at most 13 binary32 ulps of the result.
// The bf16 rounding of the true value and of the
// binary64 evaluation (which is within half a binary32 ulp of it after its own rounding) is therefore
// the one of this value whenever its low 16 bits are more than 32 ulps away from the half-way pattern
// 0x8000.  Anything else (1 value in 1000, and inputs outside the ranges) is evaluated in binary64.
__device__ inline uint4 swiglu8(uint4 g, uint4 u)
{
    const uint32_t gw[4] = {g.x, g.y, g.z, g.w}, uw[4] = {u.x, u.y, u.z, u.w};
    float gf[8], uf[8], y[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        gf[2 * i] = bf16_lo(gw[i]); gf[2 * i + 1] = bf16_hi(gw[i]);
        uf[2 * i] = bf16_lo(uw[i]); uf[2 * i + 1] = bf16_hi(uw[i]);
    }
    uint32_t redo = 0;  // the eight fast evaluations are straight-line code; what they leave open is redone below
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float ag = fabsf(gf[i]), au = fabsf(uf[i]);
        y[i] = gf[i] * __builtin_amdgcn_rcpf(1.0f + expf(-gf[i])) * uf[i];
        const uint32_t low = __float_as_uint(y[i]) & 0xFFFFu;
        const bool safe = ag >= 0x1p-30f && ag <= 32.0f && au >= 0x1p-30f && au <= 0x1p30f &&
                          low - (0x8000u - 32u) > 64u;  // unsigned: |low - 0x8000| > 32
        redo |= safe ? 0u : 1u << i;
    }
    if (redo != 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if ((redo >> i) & 1u) {
                const double gd = (double)gf[i];
                y[i] = (float)(gd / (1.0 + exp(-gd)) * (double)uf[i]);
            }
    }
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = pack_bf16_rne(y[2 * i], y[2 * i + 1]);
    return make_uint4(o[0], o[1], o[2], o[3]);
}

__device__ inline double sum_values(double acc, uint4 v)
{
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        acc += (double)bf16_lo(w[i]);
        acc += (double)bf16_hi(w[i]);
    }
    return acc;
}

// statistics of a row from its two binary64 sums: 1 / sqrt(second moment or variance + eps) in binary32
// arithmetic (IEEE add, square root, division), and for layer normalisation the mean rounded to binary32
template <int NORM>
__device__ inline void row_statistics(double s1, double ss, int64_t K, float eps, float& mu, float& rstd)
{
#pragma clang fp contract(off)
    double second = ss / (double)K;
    mu = 0.0f;
    if constexpr (NORM == 2) {
        const double mean = s1 / (double)K;
        second = fmax(second - mean * mean, 0.0);  // variance, never negative
        mu = (float)mean;
    }
    rstd = 1.0f / sqrtf((float)second + eps);
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

// NORM (the producer fused in front): 0 plain quantizer, 1 RMS normalisation (gain), 2 layer normalisation
// (gain, bias), 3 ReLU, 4 gated SiLU (X is the gate, `other` the second operand).  With 1 and 2 a non-null
// `other` is a residual added to X first; the sum, rounded to bf16, also goes to H.  Every thread reads an
// element of `other` before it writes the same element of H, and nothing else touches it: H may be `other`.
template <int RP, int NT, int NORM>
__global__ __launch_bounds__(NT) void k_quantize_act(const uint16_t* __restrict__ X, int64_t K, int64_t ldx,
                                                         uint8_t* __restrict__ Xq, float* __restrict__ sx,
                                                         const uint16_t* __restrict__ U, int r, float* __restrict__ T,
                                                         Producer pr)
{
    const uint16_t* __restrict__ gain = pr.gain;
    const uint16_t* __restrict__ bias = pr.bias;
    const float eps = pr.eps;
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
    if constexpr (NORM != 0) {  // the whole row sits in registers (the launcher guarantees K <= 8 * kRegChunks * NT)
        if (pr.other != nullptr || NORM == 4) {
            const uint4* orow = reinterpret_cast<const uint4*>(pr.other + row * pr.ld_other);
            uint4* hrow = reinterpret_cast<uint4*>(pr.H + row * K);
#pragma unroll
            for (int c = 0; c < kRegChunks; ++c) {
                const int idx = tid + c * kThreads;
                if (idx < nchunk) {
                    if constexpr (NORM == 4) {
                        v[c] = swiglu8(v[c], orow[idx]);
                        if (pr.H != nullptr) hrow[idx] = v[c];
                    } else {
                        v[c] = add8(v[c], orow[idx]);
                        hrow[idx] = v[c];
                    }
                }
            }
        }
        if constexpr (NORM == 3) {
#pragma unroll
            for (int c = 0; c < kRegChunks; ++c) v[c] = relu8(v[c]);
        }
    }
    if constexpr (NORM == 1 || NORM == 2) {
        // the whole row sits in registers (the launcher guarantees K <= 8 * kRegChunks * NT): sum of
        // squares (and of the values, for layer normalisation) in binary64, waves meet in LDS and
        // every thread adds the partial sums in the same order; then the normalised row replaces the row
        __shared__ double s_ss[kWaves], s_s1[NORM == 2 ? kWaves : 1];
        const uint4* grow = reinterpret_cast<const uint4*>(gain);
        const uint4* brow = reinterpret_cast<const uint4*>(bias);
        uint4 g[kRegChunks], b[NORM == 2 ? kRegChunks : 1];
        double ss = 0.0, s1 = 0.0;
#pragma unroll
        for (int c = 0; c < kRegChunks; ++c) {
            int idx = tid + c * kThreads;
            g[c] = make_uint4(0, 0, 0, 0);
            if (idx < nchunk) g[c] = grow[idx];
            if constexpr (NORM == 2) {
                b[c] = make_uint4(0, 0, 0, 0);
                if (idx < nchunk) b[c] = brow[idx];
                s1 = sum_values(s1, v[c]);
            }
            ss = sum_squares(ss, v[c]);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            ss += __shfl_xor(ss, off);
            if constexpr (NORM == 2) s1 += __shfl_xor(s1, off);
        }
        if ((tid & 63) == 0) {
            s_ss[tid >> 6] = ss;
            if constexpr (NORM == 2) s_s1[tid >> 6] = s1;
        }
        __syncthreads();
        ss = s_ss[0];
        if constexpr (NORM == 2) s1 = s_s1[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) {
            ss += s_ss[w];
            if constexpr (NORM == 2) s1 += s_s1[w];
        }
        float mu, rstd;
        row_statistics<NORM>(s1, ss, K, eps, mu, rstd);
#pragma unroll
        for (int c = 0; c < kRegChunks; ++c) {
            if constexpr (NORM == 2) {
                // chunks past the row's end stay zero: the bias must not leak into the absmax
                if (tid + c * kThreads < nchunk) v[c] = normalize8_affine(v[c], g[c], b[c], mu, rstd);
            } else {
                v[c] = normalize8(v[c], g[c], rstd);
            }
        }
    }
    uint32_t am = 0;
#pragma unroll
    for (int c = 0; c < kRegChunks; ++c) am = absmax_bits(am, v[c]);
    if constexpr (NORM == 0)
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
        if constexpr (NORM == 0)
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
    if constexpr (NORM == 0)
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
// LORC: the rank-8 left factor T = y . U rides along.  The workgroup then has eight waves (eight tokens) and keeps
// the whole of U (K x 8 binary16 values, 16 bytes per row, at most 128 KB) in LDS: the loads of U are issued ahead of
// the row's own, so that they are the first to land, and the multiply-adds of a chunk start as soon as that chunk
// of the row has arrived, while the rest of the row is still on its way -- there is no barrier and no further load
// in the loop.
template <int MAXC, int NORM, bool LORC>
__global__ __launch_bounds__(LORC ? 512 : 256) void k_quantize_rows(const uint16_t* __restrict__ X, int64_t M, int64_t K, int64_t ldx,
                                                     uint8_t* __restrict__ Xq, float* __restrict__ sx,
                                                     const uint16_t* __restrict__ U, float* __restrict__ T, Producer pr)
{
    const uint16_t* __restrict__ gain = pr.gain;
    const uint16_t* __restrict__ bias = pr.bias;
    const float eps = pr.eps;
    const int lane = threadIdx.x & 63;
    constexpr int kRowsPerWg = LORC ? 8 : 4;
    int64_t row = (int64_t)blockIdx.x * kRowsPerWg + (threadIdx.x >> 6);
    bool live = true;  // LORC: the waves stage U together, so a wave past the last token stays, repeats that token and stores nothing
    if (row >= M) {
        if constexpr (!LORC) return;  // whole waves leave; nothing below synchronises across waves
        live = false;
        row = M - 1;
    }
    const uint4* xrow = reinterpret_cast<const uint4*>(X + row * ldx);
    uint2* qrow = reinterpret_cast<uint2*>(Xq + row * K);
    const int nchunk = (int)(K / 8);

    // LORC: row k of U is 8 binary16 values, one uint4.  Thread t fetches row 512 c + t of every 512-row chunk c
    // (past K: the last row; the row's elements are zero there) and stores it at slot 64 i + (l ^ 2 i) of the
    // chunk, i = t % 8, l = t / 8: lane l, which holds elements 8 l .. 8 l + 7 of the chunk, then finds the row of
    // its i-th element at slot 64 i + (l ^ 2 i) -- for a fixed i the 64 lanes read 64 consecutive slots in a
    // permuted order (conflict-free 16-byte reads, no exchange of elements), and the sixteen lanes that store
    // together (two values of l, all eight i) hit sixteen different slots of a 16-slot block (without the XOR
    // they would hit two, eight lanes each).
    // Every load of this form is unconditional (indices past the end are clamped into the row, what they fetch is
    // replaced by zeros afterwards): with loads inside branches the compiler can no longer count the outstanding ones
    // and waits for all of them at the first use of any.
    extern __shared__ __attribute__((aligned(16))) uint4 s_u[];  // LORC: MAXC * 512 slots
    uint4 ureg[LORC ? MAXC : 1];
    if constexpr (LORC) {
        const uint4* u4 = reinterpret_cast<const uint4*>(U);
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int64_t k = (int64_t)c * 512 + threadIdx.x;
            ureg[c] = u4[k < K ? k : K - 1];
        }
    }
    uint4 v[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int idx = c * 64 + lane;
        if constexpr (LORC) {
            v[c] = xrow[idx < nchunk ? idx : nchunk - 1];
        } else {
            v[c] = make_uint4(0, 0, 0, 0);
            if (idx < nchunk) v[c] = xrow[idx];
        }
    }
    if constexpr (LORC) {  // needs the loads of U only: the row's are younger
        const int slot = (threadIdx.x & 7) * 64 + ((threadIdx.x >> 3) ^ (2 * (threadIdx.x & 7)));
#pragma unroll
        for (int c = 0; c < MAXC; ++c) s_u[c * 512 + slot] = ureg[c];
        __syncthreads();
    }
    auto zero_past_end = [&](int c) {  // LORC: what the clamped loads fetched past the row's end
        if (c * 64 + lane >= nchunk) v[c] = make_uint4(0, 0, 0, 0);
    };
    if constexpr (LORC && NORM != 0) {
#pragma unroll
        for (int c = 0; c < MAXC; ++c) zero_past_end(c);
    }
    if constexpr (NORM != 0) {
        if (pr.other != nullptr || NORM == 4) {
            const uint4* orow = reinterpret_cast<const uint4*>(pr.other + row * pr.ld_other);
            uint4* hrow = reinterpret_cast<uint4*>(pr.H + row * K);
#pragma unroll
            for (int c = 0; c < MAXC; ++c) {
                const int idx = c * 64 + lane;
                if (idx < nchunk) {
                    if constexpr (NORM == 4) {
                        v[c] = swiglu8(v[c], orow[idx]);
                        if (pr.H != nullptr && live) hrow[idx] = v[c];
                    } else {
                        v[c] = add8(v[c], orow[idx]);
                        if (live) hrow[idx] = v[c];
                    }
                }
            }
        }
        if constexpr (NORM == 3) {
#pragma unroll
            for (int c = 0; c < MAXC; ++c) v[c] = relu8(v[c]);
        }
    }
    if constexpr (NORM == 1 || NORM == 2) {
        double ss = 0.0, s1 = 0.0;
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            ss = sum_squares(ss, v[c]);
            if constexpr (NORM == 2) s1 = sum_values(s1, v[c]);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {  // every lane ends with the same sums
            ss += __shfl_xor(ss, off);
            if constexpr (NORM == 2) s1 += __shfl_xor(s1, off);
        }
        float mu, rstd;
        row_statistics<NORM>(s1, ss, K, eps, mu, rstd);
        const uint4* grow = reinterpret_cast<const uint4*>(gain);
        const uint4* brow = reinterpret_cast<const uint4*>(bias);
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int idx = c * 64 + lane;
            if (idx < nchunk) {
                if constexpr (NORM == 2) v[c] = normalize8_affine(v[c], grow[idx], brow[idx], mu, rstd);
                else v[c] = normalize8(v[c], grow[idx], rstd);
            }
        }
    }
    float acc[8];
    if constexpr (LORC) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            if constexpr (NORM == 0) zero_past_end(c);  // here, so that chunk c waits for its own load only
            if (c * 64 < nchunk) {  // the same for the whole workgroup; lanes past the row's end hold zeros
                const uint32_t xw[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float x = __uint_as_float((i & 1) ? (xw[i >> 1] & 0xffff0000u) : (xw[i >> 1] << 16));
                    const uint4 u = s_u[c * 512 + 64 * i + (lane ^ (2 * i))];
                    const uint32_t uw[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        // binary16 halves of a dword, widened inside the multiply-add (mixed-precision FMA: the same
                        // exact widening and one binary32 rounding as convert-then-fma, without the conversions)
                        const half2_t p = __builtin_bit_cast(half2_t, uw[q]);
                        acc[2 * q] = fmaf(x, (float)p[0], acc[2 * q]);
                        acc[2 * q + 1] = fmaf(x, (float)p[1], acc[2 * q + 1]);
                    }
                }
            }
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
    if (lane == 0 && live) sx[row] = scale;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int idx = c * 64 + lane;
        if (idx < nchunk && live) qrow[idx] = encode8(v[c], inv);
    }
    if constexpr (LORC) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float a = acc[j];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off);
            if (lane == 0 && live) T[row * 8 + j] = a;
        }
    }
}

// The same with a helper wave per token (plain and ReLU forms, rows of at most 5120 elements): 2048 tokens are only
// eight waves per compute unit, and a lone chain of K x 8 multiply-adds per token is what the call then waits for
// (one or two waves per SIMD issue a vector instruction every 12 or 6 cycles).  Sixteen waves per workgroup: wave
// w < 8 owns token w as before but multiplies only the first H chunks of its row; wave w + 8 fetches the other
// chunks of the same row (the requests of the token wave for them, issued behind the staging barrier, then hit in
// L2), multiplies them and hands its eight partial sums over through LDS.  Both kinds issue the same number of
// loads ahead of the barrier, in the same straight-line code, so the compiler's load counts stay exact.
template <int MAXC, int NORM>
__global__ __launch_bounds__(1024) void k_quantize_rows_helped(const uint16_t* __restrict__ X, int64_t M, int64_t K, int64_t ldx,
                                                             uint8_t* __restrict__ Xq, float* __restrict__ sx,
                                                             const uint16_t* __restrict__ U, float* __restrict__ T)
{
    static_assert(NORM == 0 || NORM == 3, "element-wise producers only: a helper has half a row");
    constexpr int H = (MAXC + 1) / 2, R = MAXC - H;  // chunks multiplied by the token wave / by its helper
    extern __shared__ __attribute__((aligned(16))) uint4 s_u[];  // MAXC * 512 slots, as in k_quantize_rows
    __shared__ float s_part[8][8];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const bool helper = w >= 8;  // wave-uniform
    int64_t row = (int64_t)blockIdx.x * 8 + (w & 7);
    const bool live = row < M;
    if (!live) row = M - 1;  // stays for the barriers, repeats the last token, stores nothing
    const uint4* xrow = reinterpret_cast<const uint4*>(X + row * ldx);
    uint2* qrow = reinterpret_cast<uint2*>(Xq + row * K);
    const int nchunk = (int)(K / 8);
    const int base = helper ? H : 0;  // first chunk of this wave's share

    // U: the 512 threads of each half of the workgroup take the chunks of one parity (a chunk past the last is the
    // last again: the same rows to the same slots)
    uint4 ureg[H];
    const int st = threadIdx.x & 511, par = threadIdx.x >> 9;
    const uint4* u4 = reinterpret_cast<const uint4*>(U);
#pragma unroll
    for (int j = 0; j < H; ++j) {
        const int c = min(2 * j + par, MAXC - 1);
        const int64_t k = (int64_t)c * 512 + st;
        ureg[j] = u4[k < K ? k : K - 1];
    }
    uint4 f[H];  // this wave's share of the row (a helper with one chunk less fetches its last one twice)
#pragma unroll
    for (int c = 0; c < H; ++c) {
        const int idx = min(base + c, MAXC - 1) * 64 + lane;
        f[c] = xrow[idx < nchunk ? idx : nchunk - 1];
    }
    {
        const int slot = (st & 7) * 64 + ((st >> 3) ^ (2 * (st & 7)));
#pragma unroll
        for (int j = 0; j < H; ++j) s_u[min(2 * j + par, MAXC - 1) * 512 + slot] = ureg[j];
    }
    __syncthreads();
    // the rest of the row, which the token wave needs for the maximum and the codes (its helper asked for the same
    // lines ahead of the barrier).  Issued by both kinds of wave, so that no load sits in a branch.
    uint4 g[R > 0 ? R : 1];
#pragma unroll
    for (int c = 0; c < R; ++c) {
        const int idx = (H + c) * 64 + lane;
        g[c] = xrow[idx < nchunk ? idx : nchunk - 1];
    }
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
#pragma unroll
    for (int c = 0; c < H; ++c) {
        const int ch = base + c;  // the chunk in f[c]; a helper's repeated last chunk counts for nothing
        if (ch * 64 + lane >= nchunk || ch >= MAXC) f[c] = make_uint4(0, 0, 0, 0);
        if constexpr (NORM == 3) f[c] = relu8(f[c]);
        if (ch * 64 < nchunk && ch < MAXC) {  // wave-uniform
            const uint32_t xw[4] = {f[c].x, f[c].y, f[c].z, f[c].w};
            const uint4* su = s_u + ch * 512;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float x = __uint_as_float((i & 1) ? (xw[i >> 1] & 0xffff0000u) : (xw[i >> 1] << 16));
                const uint4 u = su[64 * i + (lane ^ (2 * i))];
                const uint32_t uw[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const half2_t p = __builtin_bit_cast(half2_t, uw[q]);  // widened inside the multiply-add, as above
                    acc[2 * q] = fmaf(x, (float)p[0], acc[2 * q]);
                    acc[2 * q + 1] = fmaf(x, (float)p[1], acc[2 * q + 1]);
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc[j] += __shfl_xor(acc[j], off);
    }
    float mine = acc[0];  // every lane holds all eight sums: lane j keeps the j-th
#pragma unroll
    for (int j = 1; j < 8; ++j) mine = lane == j ? acc[j] : mine;
    if (helper) {
        if (lane < 8) s_part[w - 8][lane] = mine;
        __syncthreads();
        return;
    }
    uint32_t am = 0;
#pragma unroll
    for (int c = 0; c < H; ++c) am = absmax_bits(am, f[c]);
#pragma unroll
    for (int c = 0; c < R; ++c) {
        if ((H + c) * 64 + lane >= nchunk) g[c] = make_uint4(0, 0, 0, 0);
        if constexpr (NORM == 3) g[c] = relu8(g[c]);
        am = absmax_bits(am, g[c]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) am = max(am, (uint32_t)__shfl_xor((int)am, off));
    float scale, inv;
    token_scale(am, scale, inv);
    if (lane == 0 && live) sx[row] = scale;
#pragma unroll
    for (int c = 0; c < H; ++c) {
        const int idx = c * 64 + lane;
        if (idx < nchunk && live) qrow[idx] = encode8(f[c], inv);
    }
#pragma unroll
    for (int c = 0; c < R; ++c) {
        const int idx = (H + c) * 64 + lane;
        if (idx < nchunk && live) qrow[idx] = encode8(g[c], inv);
    }
    __syncthreads();  // the helper's sums are in LDS
    if (lane < 8 && live) T[row * 8 + lane] = mine + s_part[w][lane];  // first half of the row plus second half: a fixed order
}

// the wave-per-token kernel with the rank-8 factor: eight tokens per workgroup, all of U in dynamic LDS
template <int MAXC, int KIND>
hipError_t launch_rows_lorc(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, float* sx, const uint16_t* U,
                            float* T, const Producer& pr, hipStream_t s)
{
    const size_t smem = (size_t)MAXC * 512 * sizeof(uint4);
    static OnceStatus attr;  // raising the dynamic LDS limit is a per-function, per-process setting
    // A helper wave per token while every compute unit gets at most one workgroup (its 16 waves leave 128 registers
    // each, hence rows of at most 5120 elements): 2048 x 5120 12.1 -> 11.0 us, 1024 x 5120 11.1 -> 9.9.  With more
    // tokens the waves of later workgroups fill the SIMDs anyway and the helpers' second fetch of half of every row
    // only costs (4096 x 4096: 16.6 -> 19.3 us), so the plain form stays.
    if constexpr ((KIND == 0 || KIND == 3) && MAXC <= 10) {
        if ((M + 7) / 8 <= compute_units()) {
            auto kern = k_quantize_rows_helped<MAXC, KIND>;
            static OnceStatus attr_helped;
            if (hipError_t e = run_once(attr_helped, [&] {
                    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
                }); e != hipSuccess)
                return e;
            hipLaunchKernelGGL(kern, dim3((unsigned)((M + 7) / 8)), dim3(1024), smem, s, X, M, K, ldx, Xq, sx, U, T);
            return hipGetLastError();
        }
    }
    auto kern = k_quantize_rows<MAXC, KIND, true>;
    if (hipError_t e = run_once(attr, [&] {
            return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        }); e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)((M + 7) / 8)), dim3(512), smem, s, X, M, K, ldx, Xq, sx, U, T, pr);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_quantize_act(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, float* sx,
                               const uint16_t* U, int r, float* T, const Producer& pr, hipStream_t s)
{
    if (M == 0) return hipSuccess;
    const int kind = pr.kind;
    // many tokens: one wave per token, without the LoRC factor or with the rank-8 one (U in LDS)
    if (M >= 1024 && K <= 8192 && (r == 0 || r == 8)) {
        const dim3 g4((unsigned)((M + 3) / 4));
#define ZQ_ROWS_N(MAXC, KIND)                                                                                               \
    do {                                                                                                                    \
        if (r == 8) {  /* every chunk's load of U and of the row is issued: a tight chunk count wastes none */                 \
            constexpr int C1 = MAXC == 16 ? 10 : MAXC == 8 ? 6 : MAXC, C2 = MAXC == 16 ? 12 : MAXC;                              \
            hipError_t e = K <= 512 * C1   ? launch_rows_lorc<C1, KIND>(X, M, K, ldx, Xq, sx, U, T, pr, s)                       \
                           : K <= 512 * C2 ? launch_rows_lorc<C2, KIND>(X, M, K, ldx, Xq, sx, U, T, pr, s)                       \
                                           : launch_rows_lorc<MAXC, KIND>(X, M, K, ldx, Xq, sx, U, T, pr, s);                   \
            if (e != hipSuccess) return e;                                                                                      \
        } else {                                                                                                                \
            hipLaunchKernelGGL((k_quantize_rows<MAXC, KIND, false>), g4, dim3(256), 0, s, X, M, K, ldx, Xq, sx, U, T, pr);        \
        }                                                                                                                       \
    } while (0)
#define ZQ_ROWS(MAXC)                          \
    do {                                       \
        switch (kind) {                        \
        case 1: ZQ_ROWS_N(MAXC, 1); break;     \
        case 2: ZQ_ROWS_N(MAXC, 2); break;     \
        case 3: ZQ_ROWS_N(MAXC, 3); break;     \
        case 4: ZQ_ROWS_N(MAXC, 4); break;     \
        default: ZQ_ROWS_N(MAXC, 0); break;    \
        }                                      \
    } while (0)
        if (K <= 2048) ZQ_ROWS(4);
        else if (K <= 4096) ZQ_ROWS(8);
        else ZQ_ROWS(16);
#undef ZQ_ROWS
#undef ZQ_ROWS_N
        return hipGetLastError();
    }
    const dim3 grid((unsigned)M);
    // 1024 threads per token for a handful of tokens, and for rows with a producer too long for 256 threads' registers
    const bool wide = (M <= 64 && K >= 2048) || (kind != 0 && K > 8 * kRegChunks * 256);
#define ZQ_QUANT_N(RP, NT, KIND) \
    hipLaunchKernelGGL((k_quantize_act<RP, NT, KIND>), grid, dim3(NT), 0, s, X, K, ldx, Xq, sx, U, r, T, pr)
#define ZQ_QUANT_K(RP, NT)                        \
    do {                                          \
        switch (kind) {                           \
        case 1: ZQ_QUANT_N(RP, NT, 1); break;     \
        case 2: ZQ_QUANT_N(RP, NT, 2); break;     \
        case 3: ZQ_QUANT_N(RP, NT, 3); break;     \
        case 4: ZQ_QUANT_N(RP, NT, 4); break;     \
        default: ZQ_QUANT_N(RP, NT, 0); break;    \
        }                                         \
    } while (0)
#define ZQ_QUANT(RP)                    \
    do {                                \
        if (wide) ZQ_QUANT_K(RP, 1024); \
        else ZQ_QUANT_K(RP, 256);       \
    } while (0)
    if (r == 0) ZQ_QUANT(0);
    else if (r <= 8) ZQ_QUANT(8);
    else if (r <= 16) ZQ_QUANT(16);
    else if (r <= 32) ZQ_QUANT(32);
    else ZQ_QUANT(64);
#undef ZQ_QUANT
#undef ZQ_QUANT_K
#undef ZQ_QUANT_N
    return hipGetLastError();
}

}  // namespace zqfp
