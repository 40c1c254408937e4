// GPTQ on the E2M1 grid with power-of-two group scales (the weight quantizer the paper runs: Section 3,
// Appendix A; scales as in "Casting the FP4 to FP8", methods M1 / M2).  Offline step; its output is the same
// packed blob zqfp_pack_weight_fp4 makes.
//
// Input channels (rows of the K x N weight) are quantized in order; the scaled error of channel k is pushed
// onto the channels behind it with row k of U, the upper Cholesky factor of the inverse Hessian:
//     q_k = S e2m1(w_k / S);  err = (w_k - q_k) / U[k][k];  w_j -= U[k][j] err   (j > k).
// Output channels never interact, so a lane owns one output channel.  Rows are taken in blocks of B = 128
// (256 for groups of 256, so that a group never straddles a block): inside a block the updates are applied at
// once, on the block's B x 64 slab held in LDS; the rows behind the block receive the block's B errors in
// one float32 matrix product (rows of U through the scalar cache, error rows through LDS).
#include "zqfp_internal.h"

namespace zqfp {
namespace {

// Working copy of W in float32, column absmax of the original W, and the blob's frame: header, zero codes,
// exponent bytes 127, column scales (1 under M1, absmax / 6 under M2, 0 for padding columns).
__global__ __launch_bounds__(256) void k_gptq_init(const uint16_t* __restrict__ W, int64_t ldw, BlobLayout L, int mode,
                                                   float* __restrict__ Wf, float* __restrict__ colmax, uint8_t* __restrict__ blob)
{
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x, nthreads = (int64_t)gridDim.x * 256;
    uint32_t* codes = reinterpret_cast<uint32_t*>(blob + L.off_codes);
    for (int64_t i = tid; i < (int64_t)((L.off_exps - L.off_codes) / 4); i += nthreads) codes[i] = 0u;
    uint32_t* exps = reinterpret_cast<uint32_t*>(blob + L.off_exps);
    for (int64_t i = tid; i < L.nstrips * L.ngq * 16; i += nthreads) exps[i] = 0x7F7F7F7Fu;
    float* cs = reinterpret_cast<float*>(blob + L.off_colscale);
    for (int64_t n = tid; n < L.Np; n += nthreads) {
        float mx = 0.0f;
        if (n < L.N)
            for (int64_t k = 0; k < L.K; ++k) {
                const float w = bf16_bits_to_f32(W[k * ldw + n]);
                Wf[k * L.N + n] = w;
                mx = fmaxf(mx, fabsf(w));
            }
        if (n < L.N) colmax[n] = mx;
        cs[n] = n >= L.N ? 0.0f : mode == 1 ? 1.0f : mx != 0.0f ? mx / 6.0f : 1.0f;  // IEEE binary32 division
    }
    if (tid == 0) {
        BlobHeader h;
        h.magic = kBlobMagic; h.version = kBlobVersion;
        h.K = L.K; h.N = L.N; h.Np = L.Np;
        h.G = L.G; h.Gs = L.Gs; h.mode = mode; h.ngs = L.ngs; h.ngq = L.ngq; h.wbits = 4;
        h.off_codes = L.off_codes; h.off_exps = L.off_exps; h.off_colscale = L.off_colscale; h.total = L.total;
        *reinterpret_cast<BlobHeader*>(blob) = h;
    }
}

// Rows [i0, i0 + B) of the working copy, 64 output channels per workgroup (one wave, lane = channel).
__global__ __launch_bounds__(64) void k_gptq_block(float* __restrict__ Wf, const float* __restrict__ U, BlobLayout L, int mode,
                                                  int B, int64_t i0, const float* __restrict__ colmax,
                                                  float* __restrict__ Err, uint8_t* __restrict__ blob)
{
    extern __shared__ float s_w[];  // [B][64]
    const int lane = threadIdx.x;
    const int64_t n = (int64_t)blockIdx.x * 64 + lane;
    if (n >= L.N) return;  // a lane works on its own column only: nothing below synchronises
    for (int r = 0; r < B; ++r) s_w[r * 64 + lane] = Wf[(i0 + r) * L.N + n];
    const float cs = reinterpret_cast<const float*>(blob + L.off_colscale)[n];
    const float cmax = colmax[n];
    const int64_t strip = n >> 4;
    const int c = (int)(n & 15);
    uint8_t* code_bytes = blob + L.off_codes;
    uint8_t* exp_bytes = blob + L.off_exps;
    int e = 0;
    float S = 1.0f;
    uint32_t low = 0;
    for (int j = 0; j < B; ++j) {
        const int64_t k = i0 + j;
        if (k % L.G == 0) {  // a new group: its scale from the weights as they stand now
            float amax = 0.0f;
            for (int g = 0; g < L.G; ++g) amax = fmaxf(amax, fabsf(s_w[(j + g) * 64 + lane]));
            e = mode == 1 ? m1_exponent(amax) : -m2_shift(cmax, amax);
            S = mode == 1 ? ldexpf(1.0f, e) : ldexpf(cs, e);
            const int64_t sg = k / L.Gs;  // G is 32, 64, 128 or 256 here: stored groups are the groups
            exp_bytes[((size_t)(strip * L.ngq + (sg >> 2)) * 16 + c) * 4 + (sg & 3)] = (uint8_t)(e + 127);
        }
        const float w = s_w[j * 64 + lane];
        const float y = mode == 1 ? ldexpf(w, -e) : ldexpf(w / cs, -e);
        const uint32_t code = e2m1_encode(y);
        const float q = mode == 1 ? ldexpf(e2m1_value(code), e) : ldexpf(e2m1_value(code), e) * cs;
        const float* urow = U + k * L.K + i0;  // the same for every lane
        const float err = (w - q) / urow[j];
        Err[(int64_t)j * L.N + n] = err;
        for (int jj = j + 1; jj < B; ++jj) s_w[jj * 64 + lane] = fmaf(-urow[jj], err, s_w[jj * 64 + lane]);
        if ((k & 1) == 0) {
            low = code;
        } else {
            const int kk = (int)(k & 127), lb = kk >> 5, p = kk & 31;
            code_bytes[((size_t)(strip * L.nkt + (k >> 7)) * 64 + (lb * 16 + c)) * 16 + (p >> 1)] = (uint8_t)(low | (code << 4));
        }
    }
}

// Wf[r][n] -= sum_j U[i0 + j][r] Err[j][n] for the rows r behind the block.  64 x 64 tile per workgroup,
// 4 x 4 outputs per thread, B walked in steps of 16 through LDS.
__global__ __launch_bounds__(256) void k_gptq_trail(float* __restrict__ Wf, const float* __restrict__ U, int64_t K, int64_t N,
                                                  int B, int64_t i0, const float* __restrict__ Err)
{
    __shared__ float s_u[16][64 + 4], s_e[16][64 + 4];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int64_t r0 = i0 + B + (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;
    for (int j0 = 0; j0 < B; j0 += 16) {
        for (int idx = tid; idx < 16 * 64; idx += 256) {
            const int jj = idx >> 6, cc = idx & 63;
            s_u[jj][cc] = U[(i0 + j0 + jj) * K + r0 + cc];  // r0 + 63 < K: the rows behind a block come in 128s
            s_e[jj][cc] = n0 + cc < N ? Err[(int64_t)(j0 + jj) * N + n0 + cc] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            float u[4], ev[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) u[a] = s_u[jj][ty * 4 + a];
#pragma unroll
            for (int b = 0; b < 4; ++b) ev[b] = s_e[jj][tx * 4 + b];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = fmaf(u[a], ev[b], acc[a][b]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int64_t r = r0 + ty * 4 + a, n = n0 + tx * 4 + b;
            if (n < N) Wf[r * N + n] -= acc[a][b];
        }
}

}  // namespace

// float32 working copy [K][N], the current block's errors [B][N], column absmax [N]
size_t gptq_workspace_bytes(int64_t K, int64_t N, int G)
{
    const int64_t B = G > 128 ? G : 128;
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    return up((size_t)K * N * 4) + up((size_t)B * N * 4) + up((size_t)N * 4);
}

hipError_t launch_gptq_pack(const uint16_t* W, int64_t ldw, const BlobLayout& L, int mode, const float* U, uint8_t* blob,
                            void* workspace, hipStream_t s)
{
    const int64_t K = L.K, N = L.N;
    const int B = L.G > 128 ? L.G : 128;
    uint8_t* p = static_cast<uint8_t*>(workspace);
    auto take = [&](size_t bytes) {
        uint8_t* q = p;
        p += (bytes + 255) / 256 * 256;
        return q;
    };
    float* Wf = reinterpret_cast<float*>(take((size_t)K * N * 4));
    float* Err = reinterpret_cast<float*>(take((size_t)B * N * 4));
    float* colmax = reinterpret_cast<float*>(take((size_t)N * 4));
    hipLaunchKernelGGL(k_gptq_init, dim3((unsigned)((L.Np + 255) / 256)), dim3(256), 0, s, W, ldw, L, mode, Wf, colmax, blob);
    const size_t lds = (size_t)B * 64 * 4;
    static OnceStatus attr;  // 256-row blocks need more than the default dynamic-LDS limit
    if (hipError_t e = run_once(attr, [&] {
            return hipFuncSetAttribute(reinterpret_cast<const void*>(k_gptq_block), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       256 * 64 * 4);
        }); e != hipSuccess)
        return e;
    for (int64_t i0 = 0; i0 < K; i0 += B) {
        hipLaunchKernelGGL(k_gptq_block, dim3((unsigned)((N + 63) / 64)), dim3(64), lds, s, Wf, U, L, mode, B, i0, colmax, Err, blob);
        const int64_t behind = K - (i0 + B);
        if (behind > 0)
            hipLaunchKernelGGL(k_gptq_trail, dim3((unsigned)((N + 63) / 64), (unsigned)(behind / 64)), dim3(256), 0, s, Wf, U, K,
                               N, B, i0, Err);
    }
    return hipGetLastError();
}

}  // namespace zqfp
