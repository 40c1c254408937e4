// Group-wise FP4 (E2M1) weight quantizer with power-of-two group scales
// (paper Section 3: fine-grained quantization; "Casting the FP4 to FP8",
// methods M1 and M2) and its inverse view.  Offline step: written for
// exactness and a GEMM-friendly layout, not for speed.
//
// One workgroup per strip of 16 output channels.  Phase 1 finds every group's
// absmax (exact), phase 2 turns it into the exponent byte (integer / exact
// power-of-two work only), phase 3 encodes the codes and writes them in the
// register order of the block-scaled matrix instruction.
#include "zqfp_internal.h"

namespace zqfp {
namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void k_pack_weight(const uint16_t* __restrict__ W, int64_t ldw, BlobLayout L,
                                                        int mode, uint8_t* __restrict__ blob)
{
    extern __shared__ float smem[];
    const int ng = (int)(L.K / L.G);
    float* s_gmax = smem;                                  // [ng][16]
    float* s_red = smem + (size_t)ng * 16;                 // [16][16]
    int* s_ebyte = reinterpret_cast<int*>(s_red + 256);    // [ng][16]
    float* s_col = reinterpret_cast<float*>(s_ebyte + (size_t)ng * 16);  // [16] column scale

    const int strip = blockIdx.x, tid = threadIdx.x;
    const int c = tid & 15, kl = tid >> 4;
    const int64_t n = (int64_t)strip * 16 + c;
    const bool live = n < L.N;

    // phase 1: exact absmax of every group
    for (int g = 0; g < ng; ++g) {
        float a = 0.0f;
        if (live)
            for (int64_t k = (int64_t)g * L.G + kl; k < (int64_t)(g + 1) * L.G; k += 16)
                a = fmaxf(a, fabsf(bf16_bits_to_f32(W[k * ldw + n])));
        s_red[kl * 16 + c] = a;
        __syncthreads();
        if (tid < 16) {
            float m = 0.0f;
            for (int i = 0; i < 16; ++i) m = fmaxf(m, s_red[i * 16 + tid]);
            s_gmax[g * 16 + tid] = m;
        }
        __syncthreads();
    }

    // phase 2: exponent bytes and column scale
    if (tid < 16) {
        float cs = 1.0f;
        if (mode == 1) {
            for (int g = 0; g < ng; ++g)
                s_ebyte[g * 16 + tid] = (L.wbits == 8 ? m1_exponent_e4m3(s_gmax[g * 16 + tid]) : m1_exponent(s_gmax[g * 16 + tid])) + 127;
        } else {
            float mx = 0.0f;
            for (int g = 0; g < ng; ++g) mx = fmaxf(mx, s_gmax[g * 16 + tid]);
            if (mx != 0.0f) cs = mx / (L.wbits == 8 ? 448.0f : 6.0f);  // IEEE binary32 division
            for (int g = 0; g < ng; ++g) s_ebyte[g * 16 + tid] = 127 - m2_shift(mx, s_gmax[g * 16 + tid]);
        }
        s_col[tid] = cs;
        int64_t nn = (int64_t)strip * 16 + tid;
        reinterpret_cast<float*>(blob + L.off_colscale)[nn] = (nn < L.N) ? cs : 0.0f;
    }
    __syncthreads();

    // exponent bytes, [strip][quad][column][4]
    for (int i = tid; i < L.ngq * 16; i += kThreads) {
        int q = i >> 4, cc = i & 15;
        uint32_t word = 0;
        for (int b = 0; b < 4; ++b) {
            int sg = q * 4 + b;
            uint32_t e = 127;
            if (sg < L.ngs && (int64_t)strip * 16 + cc < L.N) e = (uint32_t)s_ebyte[(int)(((int64_t)sg * L.Gs) / L.G) * 16 + cc];
            word |= e << (8 * b);
        }
        reinterpret_cast<uint32_t*>(blob + L.off_exps)[(size_t)strip * L.ngq * 16 + i] = word;
    }

    if (L.wbits == 8) {
        // phase 3, E4M3 codes: fragment = [half][64 lanes][4 dwords]; a dword holds 4 consecutive k.  Same encoder
        // as the activations': clamp to +-448, then the hardware conversion (round to nearest even, sign kept).
        uint32_t* out8 = reinterpret_cast<uint32_t*>(blob + L.off_codes) + (size_t)strip * L.nkt * 512;
        for (int64_t kt = 0; kt < L.nkt; ++kt) {
            for (int idx = tid; idx < 512; idx += kThreads) {
                const int half = idx >> 8, ln = (idx >> 2) & 63, dd = idx & 3;
                const int cc = ln & 15, lbb = ln >> 4;
                const int64_t nn = (int64_t)strip * 16 + cc;
                const int64_t k0 = kt * 128 + 64 * half + 16 * lbb + 4 * dd;
                const int e = s_ebyte[(int)(k0 / L.G) * 16 + cc] - 127;
                const float csn = s_col[cc];
                uint32_t word = 0;
                if (nn < L.N) {
                    float y[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float w = bf16_bits_to_f32(W[(k0 + i) * ldw + nn]);
                        y[i] = clamp448((mode == 1) ? ldexpf(w, -e) : ldexpf(w / csn, -e));
                    }
                    int pk = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], 0, false);
                    pk = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], pk, true);
                    word = (uint32_t)pk;
                }
                out8[kt * 512 + idx] = word;
            }
        }
        if (strip == 0 && tid == 0) {
            BlobHeader h;
            h.magic = kBlobMagic; h.version = kBlobVersion;
            h.K = L.K; h.N = L.N; h.Np = L.Np;
            h.G = L.G; h.Gs = L.Gs; h.mode = mode; h.ngs = L.ngs; h.ngq = L.ngq; h.wbits = 8;
            h.off_codes = L.off_codes; h.off_exps = L.off_exps; h.off_colscale = L.off_colscale; h.total = L.total;
            *reinterpret_cast<BlobHeader*>(blob) = h;
        }
        return;
    }

    // phase 3: codes, one dword (8 codes) per thread per fragment
    const int lane = tid >> 2, d = tid & 3;
    const int fc = lane & 15, lb = lane >> 4;
    const int64_t fn = (int64_t)strip * 16 + fc;
    const float cs = s_col[fc];
    uint32_t* out = reinterpret_cast<uint32_t*>(blob + L.off_codes) + (size_t)strip * L.nkt * 256;
    for (int64_t kt = 0; kt < L.nkt; ++kt) {
        const int64_t k0 = kt * 128 + 32 * lb + 8 * d;
        const int g = (int)(k0 / L.G);
        const int e = s_ebyte[g * 16 + fc] - 127;  // group scale = cs * 2^e
        uint32_t word = 0;
        if (fn < L.N) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float w = bf16_bits_to_f32(W[(k0 + i) * ldw + fn]);
                float y = (mode == 1) ? ldexpf(w, -e)        // exact division by 2^e
                                      : ldexpf(w / cs, -e);  // IEEE division, then exact shift
                word |= e2m1_encode(y) << (4 * i);
            }
        }
        out[kt * 256 + tid] = word;
    }

    if (strip == 0 && tid == 0) {
        BlobHeader h;
        h.magic = kBlobMagic; h.version = kBlobVersion;
        h.K = L.K; h.N = L.N; h.Np = L.Np;
        h.G = L.G; h.Gs = L.Gs; h.mode = mode; h.ngs = L.ngs; h.ngq = L.ngq; h.wbits = 4;
        h.off_codes = L.off_codes; h.off_exps = L.off_exps; h.off_colscale = L.off_colscale; h.total = L.total;
        *reinterpret_cast<BlobHeader*>(blob) = h;
    }
}

__global__ __launch_bounds__(kThreads) void k_unpack(const uint8_t* __restrict__ blob, BlobLayout L,
                                                   uint8_t* __restrict__ codes, uint8_t* __restrict__ exps,
                                                   float* __restrict__ colscale)
{
    const int64_t total = L.K * L.N;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < total) {
        const int64_t k = i / L.N, n = i % L.N;
        const int64_t strip = n >> 4, kt = k >> 7;
        const int c = (int)(n & 15), kk = (int)(k & 127), lb = kk >> 5, p = kk & 31;
        if (L.wbits == 8) {
            const int half = kk >> 6, lb8 = (kk >> 4) & 3;
            codes[i] = blob[L.off_codes + (size_t)(strip * L.nkt + kt) * 2048 + half * 1024 + (lb8 * 16 + c) * 16 + (kk & 15)];
        } else {
            const uint8_t byte = blob[L.off_codes + ((size_t)(strip * L.nkt + kt) * 64 + (lb * 16 + c)) * 16 + (p >> 1)];
            codes[i] = (p & 1) ? (byte >> 4) : (byte & 15);
        }
    }
    const int64_t ng = L.K / L.G;
    if (i < ng * L.N) {
        const int64_t g = i / L.N, n = i % L.N;
        const int64_t sg = g * L.G / L.Gs;
        exps[i] = blob[L.off_exps + ((size_t)((n >> 4) * L.ngq + (sg >> 2)) * 16 + (n & 15)) * 4 + (sg & 3)];
    }
    if (i < L.N) colscale[i] = reinterpret_cast<const float*>(blob + L.off_colscale)[i];
}

}  // namespace

hipError_t launch_pack_weight(const uint16_t* W, int64_t ldw, const BlobLayout& L, int mode, uint8_t* blob,
                              hipStream_t s)
{
    if (L.nstrips == 0) return hipSuccess;
    const int ng = (int)(L.K / L.G);
    size_t smem = ((size_t)ng * 16 + 256 + (size_t)ng * 16 + 16) * 4;
    hipLaunchKernelGGL(k_pack_weight, dim3((unsigned)L.nstrips), dim3(kThreads), smem, s, W, ldw, L, mode, blob);
    return hipGetLastError();
}

hipError_t launch_unpack(const uint8_t* blob, const BlobLayout& L, uint8_t* codes, uint8_t* exps, float* colscale,
                         hipStream_t s)
{
    int64_t total = L.K * L.N;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(k_unpack, dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, blob, L,
                       codes, exps, colscale);
    return hipGetLastError();
}

}  // namespace zqfp
