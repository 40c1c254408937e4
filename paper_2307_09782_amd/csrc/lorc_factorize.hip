// LoRC factorisation (paper Section 3: singular value decomposition of the error matrix
// E = W - W^, original minus quantized weight; the two low-rank matrices are made from its r
// leading singular triplets).  Offline step, once per layer.
//
// E is K x N with K, N in the thousands and r around 8 (Appendix A: 8 for LLaMA, 16..56 for OPT),
// so the leading triplets come from a subspace iteration instead of a full decomposition:
//   Y = E Omega (Omega: N x l Gaussian, l = r + 8, supplied by the caller), Y <- orth(Y);
//   q times:  Z = E^T Y, Z <- orth(Z), Y = E Z, Y <- orth(Y);
//   B^T = E^T Y (N x l);  B B^T = P L P^T (l x l symmetric eigenproblem, Jacobi rotations);
//   s_i = sqrt(L_i), left vectors Y P, right vectors B^T P / s;
//   U = (Y P)_r diag(s_r)^(1/2),  V = diag(s_r)^(-1/2) (B^T P)_r^T      (singular values shared evenly).
// Every pass over E is a plain HBM stream (E in float32: 4 K N bytes per pass, 2 + 2q passes);
// the l x l work (Gram matrices, Cholesky factors, Jacobi rotations) runs in float64.  orth() is Cholesky
// QR applied twice.
#include "zqfp_internal.h"

namespace zqfp {
namespace {

constexpr int kLMax = 72;  // r <= 64 plus 8 columns of oversampling

// E[k][n] = W[k][n] - c[n] * 2^(e - 127) * e2m1(code), one element per thread
__global__ __launch_bounds__(256) void k_lorc_error(const uint16_t* __restrict__ W, int64_t ldw,
                                                    const uint8_t* __restrict__ blob, BlobLayout L, float* __restrict__ E)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= L.K * L.N) return;
    const int64_t k = i / L.N, n = i % L.N;
    const int64_t strip = n >> 4, kt = k >> 7;
    const int c = (int)(n & 15), kk = (int)(k & 127), lb = kk >> 5, p = kk & 31;
    const uint8_t byte = blob[L.off_codes + ((size_t)(strip * L.nkt + kt) * 64 + (lb * 16 + c)) * 16 + (p >> 1)];
    const uint32_t code = (p & 1) ? (byte >> 4) : (byte & 15);
    const int64_t sg = k / L.Gs;
    const uint32_t eb = blob[L.off_exps + ((size_t)(strip * L.ngq + (sg >> 2)) * 16 + c) * 4 + (sg & 3)];
    const float cs = reinterpret_cast<const float*>(blob + L.off_colscale)[n];
    const float wq = cs * (e2m1_value(code) * __uint_as_float(eb << 23));  // eb in 1..254: 2^(eb - 127)
    E[i] = __uint_as_float((uint32_t)W[k * ldw + n] << 16) - wq;
}

// Y[k][j] = sum_n E[k][n] B[n][j], j < l.  One workgroup per RPW rows (a row of B fetched once serves them all);
// thread t walks n = t, t + 256, ...
template <int LMAX, int RPW>
__global__ __launch_bounds__(256) void k_lorc_rows(const float* __restrict__ E, int64_t K, int64_t N,
                                                   const float* __restrict__ B, int l, float* __restrict__ Y)
{
    __shared__ float s_part[4][RPW][LMAX];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t k0 = (int64_t)blockIdx.x * RPW;
    const float* e[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i) e[i] = E + (k0 + i < K ? k0 + i : K - 1) * N;  // rows past the end: repeated, never stored
    float acc[RPW][LMAX];
#pragma unroll
    for (int i = 0; i < RPW; ++i)
#pragma unroll
        for (int j = 0; j < LMAX; ++j) acc[i][j] = 0.f;
    const bool full = l == LMAX && (LMAX & 3) == 0;  // whole rows of B as 16-byte loads
    for (int64_t n = tid; n < N; n += 256) {
        float x[RPW], bj[LMAX];
#pragma unroll
        for (int i = 0; i < RPW; ++i) x[i] = e[i][n];
        const float* b = B + n * l;
        if (full) {
#pragma unroll
            for (int j = 0; j < LMAX; j += 4) {
                const float4 q = *reinterpret_cast<const float4*>(b + j);
                bj[j] = q.x; bj[j + 1] = q.y; bj[j + 2] = q.z; bj[j + 3] = q.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < LMAX; ++j) bj[j] = j < l ? b[j] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < RPW; ++i)
#pragma unroll
            for (int j = 0; j < LMAX; ++j) acc[i][j] = fmaf(x[i], bj[j], acc[i][j]);
    }
#pragma unroll
    for (int i = 0; i < RPW; ++i)
#pragma unroll
        for (int j = 0; j < LMAX; ++j) {
            float u = acc[i][j];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) u += __shfl_xor(u, off);
            if (lane == 0) s_part[wave][i][j] = u;
        }
    __syncthreads();
    for (int idx = tid; idx < RPW * l; idx += 256) {  // fixed order over the four waves
        const int row = idx / l, j = idx % l;
        if (k0 + row < K)
            Y[(k0 + row) * l + j] = (s_part[0][row][j] + s_part[1][row][j]) + (s_part[2][row][j] + s_part[3][row][j]);
    }
}

// Z[n][j] = sum_k E[k][n] A[k][j], j < l.  A workgroup owns 64 columns; its eight waves walk k = w, w + 8, ...
// (a wave reads one 256-byte run of a row of E; the row of A is the same for all its lanes and comes through
// the scalar cache) and add their sums in LDS in turn.
template <int LMAX>
__global__ __launch_bounds__(512) void k_lorc_cols(const float* __restrict__ E, int64_t K, int64_t N,
                                                   const float* __restrict__ A, int l, float* __restrict__ Z)
{
    __shared__ float s_sum[64][LMAX + 1];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t n = (int64_t)blockIdx.x * 64 + lane;
    const int64_t nc = n < N ? n : N - 1;  // clamped: never stored
    float acc[LMAX];
#pragma unroll
    for (int j = 0; j < LMAX; ++j) acc[j] = 0.f;
    for (int64_t k = wave; k < K; k += 8) {
        const float x = E[k * N + nc];
        const float* a = A + k * l;
#pragma unroll
        for (int j = 0; j < LMAX; ++j) acc[j] = fmaf(x, j < l ? a[j] : 0.f, acc[j]);
    }
    for (int w = 0; w < 8; ++w) {  // a fixed order
        if (wave == w) {
#pragma unroll
            for (int j = 0; j < LMAX; ++j) s_sum[lane][j] = w == 0 ? acc[j] : s_sum[lane][j] + acc[j];
        }
        __syncthreads();
    }
    for (int idx = tid; idx < 64 * l; idx += 512) {
        const int c = idx / l, j = idx % l;
        const int64_t nn = (int64_t)blockIdx.x * 64 + c;
        if (nn < N) Z[nn * l + j] = s_sum[c][j];
    }
}

// ---- orthonormal columns: Cholesky QR, applied twice by the launcher -----------------------------------
// Partial Gram matrices: workgroup b sums A^T A over its block of rows (float64), pair (i, j) by thread
// (i * l + j) % 256, and writes part[b][l * l].
constexpr int kGramParts = 32;
__global__ __launch_bounds__(256) void k_lorc_gram(const float* __restrict__ A, int64_t R, int l, double* __restrict__ part)
{
    __shared__ float s_rows[32][kLMax];
    const int tid = threadIdx.x;
    const int64_t per = (R + gridDim.x - 1) / gridDim.x;
    const int64_t r0 = (int64_t)blockIdx.x * per, r1 = r0 + per < R ? r0 + per : R;
    const int pairs = l * l;
    double acc[(kLMax * kLMax + 255) / 256];
#pragma unroll
    for (int q = 0; q < (kLMax * kLMax + 255) / 256; ++q) acc[q] = 0.0;
    for (int64_t base = r0; base < r1; base += 32) {
        const int nr = (int)(r1 - base < 32 ? r1 - base : 32);
        for (int idx = tid; idx < nr * l; idx += 256) s_rows[idx / l][idx % l] = A[(base + idx / l) * l + idx % l];
        __syncthreads();
#pragma unroll
        for (int q = 0; q < (kLMax * kLMax + 255) / 256; ++q) {
            const int pair = tid + 256 * q;
            if (pair < pairs) {
                const int i = pair / l, j = pair % l;
                double a = acc[q];
                for (int rr = 0; rr < nr; ++rr) a += (double)s_rows[rr][i] * (double)s_rows[rr][j];
                acc[q] = a;
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < (kLMax * kLMax + 255) / 256; ++q) {
        const int pair = tid + 256 * q;
        if (pair < pairs) part[(int64_t)blockIdx.x * pairs + pair] = acc[q];
    }
}

// G = sum of the partial Gram matrices in workgroup order (into LDS)
__device__ void sum_parts(const double* part, int nparts, int l, double* G)
{
    for (int pair = threadIdx.x; pair < l * l; pair += blockDim.x) {
        double t = 0.0;
        for (int b = 0; b < nparts; ++b) t += part[(int64_t)b * l * l + pair];
        G[pair] = t;
    }
    __syncthreads();
}

// Cholesky factor of the summed Gram matrix, G = L L^T (row i of L by thread i, one column per step)
__global__ __launch_bounds__(256) void k_lorc_chol(const double* __restrict__ part, int nparts, int l, double* __restrict__ Lout)
{
    __shared__ double G[kLMax * kLMax];
    __shared__ double s_floor;
    const int tid = threadIdx.x;
    sum_parts(part, nparts, l, G);
    if (tid == 0) {
        double mx = 0.0;
        for (int i = 0; i < l; ++i) mx = fmax(mx, G[i * l + i]);
        s_floor = fmax(mx, 1e-300) * 1e-28;  // a vanishing pivot (rank-deficient input) stays finite
    }
    __syncthreads();
    for (int j = 0; j < l; ++j) {
        if (tid == 0) {
            double d = G[j * l + j];
            for (int q = 0; q < j; ++q) d -= G[j * l + q] * G[j * l + q];
            G[j * l + j] = sqrt(fmax(d, s_floor));
        }
        __syncthreads();
        if (tid > j && tid < l) {
            double v = G[tid * l + j];
            for (int q = 0; q < j; ++q) v -= G[tid * l + q] * G[j * l + q];
            G[tid * l + j] = v / G[j * l + j];
        }
        __syncthreads();
    }
    for (int idx = tid; idx < l * l; idx += 256) Lout[idx] = G[idx];
}

// A <- A L^-T: every row solves x L^T = a by forward substitution (thread per row)
__global__ __launch_bounds__(256) void k_lorc_apply(float* __restrict__ A, int64_t R, int l, const double* __restrict__ Lin)
{
    __shared__ double Ls[kLMax * kLMax];
    for (int idx = threadIdx.x; idx < l * l; idx += 256) Ls[idx] = Lin[idx];
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= R) return;
    double x[kLMax];
    for (int j = 0; j < l; ++j) {
        double v = (double)A[r * l + j];
        for (int q = 0; q < j; ++q) v -= x[q] * Ls[j * l + q];
        x[j] = v / Ls[j * l + j];
    }
    for (int j = 0; j < l; ++j) A[r * l + j] = (float)x[j];
}

// Eigen-decomposition of M = Zb^T Zb (summed from its partial Gram matrices) by cyclic Jacobi rotations,
// descending order, and the two l x r coefficient matrices of the factors:
// CU = P_r diag(s_r)^(1/2),  CV = P_r diag(s_r)^(-1/2).  Two waves: thread t owns row / column t.
__global__ __launch_bounds__(128) void k_lorc_eig(const double* __restrict__ part, int nparts, int l, int r,
                                                  double* __restrict__ CU, double* __restrict__ CV, float* __restrict__ sigma)
{
    __shared__ double M[kLMax * kLMax], P[kLMax * kLMax];
    __shared__ double s_c, s_s, s_off;
    __shared__ int s_order[kLMax];
    const int tid = threadIdx.x;
    sum_parts(part, nparts, l, M);
    for (int idx = tid; idx < l * l; idx += 128) P[idx] = (idx / l == idx % l) ? 1.0 : 0.0;
    __syncthreads();
    for (int sweep = 0; sweep < 30; ++sweep) {
        if (tid == 0) {
            double off = 0.0, diag = 0.0;
            for (int i = 0; i < l; ++i)
                for (int j = 0; j < l; ++j) (i == j ? diag : off) += M[i * l + j] * M[i * l + j];
            s_off = off <= 1e-30 * diag ? 0.0 : 1.0;
        }
        __syncthreads();
        if (s_off == 0.0) break;  // the same for every thread: read from LDS behind a barrier
        for (int p = 0; p < l - 1; ++p)
            for (int q = p + 1; q < l; ++q) {
                if (tid == 0) {
                    const double apq = M[p * l + q];
                    double c = 1.0, s = 0.0;
                    if (apq != 0.0) {
                        const double theta = (M[q * l + q] - M[p * l + p]) / (2.0 * apq);
                        const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                        c = 1.0 / sqrt(t * t + 1.0);
                        s = t * c;
                    }
                    s_c = c;
                    s_s = s;
                }
                __syncthreads();
                const double c = s_c, s = s_s;
                if (tid < l) {  // columns p, q of M and of P (row tid)
                    const double mp = M[tid * l + p], mq = M[tid * l + q];
                    M[tid * l + p] = c * mp - s * mq;
                    M[tid * l + q] = s * mp + c * mq;
                    const double pp = P[tid * l + p], pq = P[tid * l + q];
                    P[tid * l + p] = c * pp - s * pq;
                    P[tid * l + q] = s * pp + c * pq;
                }
                __syncthreads();
                if (tid < l) {  // rows p, q of M (column tid)
                    const double mp = M[p * l + tid], mq = M[q * l + tid];
                    M[p * l + tid] = c * mp - s * mq;
                    M[q * l + tid] = s * mp + c * mq;
                }
                __syncthreads();
            }
    }
    if (tid == 0) {  // order of the eigenvalues, largest first (selection sort on indices: l is tiny)
        for (int i = 0; i < l; ++i) s_order[i] = i;
        for (int i = 0; i < l; ++i)
            for (int j = i + 1; j < l; ++j)
                if (M[s_order[j] * l + s_order[j]] > M[s_order[i] * l + s_order[i]]) {
                    const int t = s_order[i];
                    s_order[i] = s_order[j];
                    s_order[j] = t;
                }
    }
    __syncthreads();
    for (int idx = tid; idx < l * r; idx += 128) {
        const int j = idx / r, i = idx % r;
        const int col = s_order[i];
        const double sv = sqrt(fmax(M[col * l + col], 0.0));
        const double root = sqrt(sv);
        CU[idx] = P[j * l + col] * root;
        CV[idx] = root > 0.0 ? P[j * l + col] / root : 0.0;
        if (j == 0) sigma[i] = (float)sv;
    }
}

// out[row][i] = sum_j A[row][j] C[j][i]  (A: R x l float32, C: l x r float64) as binary16; `transposed` writes out[i][row]
__global__ __launch_bounds__(256) void k_lorc_emit(const float* __restrict__ A, int64_t R, int l, int r,
                                                   const double* __restrict__ C, uint16_t* __restrict__ out, int transposed)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= R * r) return;
    const int64_t row = transposed ? idx % R : idx / r;
    const int i = (int)(transposed ? idx / R : idx % r);
    double a = 0.0;
    for (int j = 0; j < l; ++j) a += (double)A[row * l + j] * C[j * r + i];
    const _Float16 h = (_Float16)(float)a;
    out[transposed ? (int64_t)i * R + row : row * r + i] = __builtin_bit_cast(uint16_t, h);
}

}  // namespace

// workspace (bytes): E [K][N] float32, Ya [K][l] float32, Za [N][l] float32, CU and CV [l][r] float64,
// partial Gram matrices [kGramParts][l][l] and a Cholesky factor [l][l] float64
size_t lorc_workspace_bytes(int64_t K, int64_t N, int r)
{
    const int64_t l = r + 8;
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    return up((size_t)K * N * 4) + up((size_t)K * l * 4) + up((size_t)N * l * 4) + 2 * up((size_t)l * r * 8) +
           up((size_t)kGramParts * l * l * 8) + up((size_t)l * l * 8);
}

hipError_t launch_lorc_factorize(const uint16_t* W, int64_t ldw, const uint8_t* blob, const BlobLayout& L, int r,
                                 const float* Omega, int power_iters, uint16_t* U, uint16_t* V, float* sigma,
                                 void* workspace, hipStream_t s)
{
    const int64_t K = L.K, N = L.N;
    const int l = r + 8;
    uint8_t* p = static_cast<uint8_t*>(workspace);
    auto take = [&](size_t bytes) {
        uint8_t* q = p;
        p += (bytes + 255) / 256 * 256;
        return q;
    };
    float* E = reinterpret_cast<float*>(take((size_t)K * N * 4));
    float* Ya = reinterpret_cast<float*>(take((size_t)K * l * 4));
    float* Za = reinterpret_cast<float*>(take((size_t)N * l * 4));
    double* CU = reinterpret_cast<double*>(take((size_t)l * r * 8));
    double* CV = reinterpret_cast<double*>(take((size_t)l * r * 8));
    double* part = reinterpret_cast<double*>(take((size_t)kGramParts * l * l * 8));
    double* Lf = reinterpret_cast<double*>(take((size_t)l * l * 8));

    hipLaunchKernelGGL(k_lorc_error, dim3((unsigned)((K * N + 255) / 256)), dim3(256), 0, s, W, ldw, blob, L, E);
    auto rows = [&](const float* B, float* Y) {
        if (l <= 16) hipLaunchKernelGGL((k_lorc_rows<16, 8>), dim3((unsigned)((K + 7) / 8)), dim3(256), 0, s, E, K, N, B, l, Y);
        else if (l <= 40) hipLaunchKernelGGL((k_lorc_rows<40, 4>), dim3((unsigned)((K + 3) / 4)), dim3(256), 0, s, E, K, N, B, l, Y);
        else hipLaunchKernelGGL((k_lorc_rows<kLMax, 2>), dim3((unsigned)((K + 1) / 2)), dim3(256), 0, s, E, K, N, B, l, Y);
    };
    auto cols = [&](const float* A, float* Z) {
        const dim3 g((unsigned)((N + 63) / 64));
        if (l <= 16) hipLaunchKernelGGL((k_lorc_cols<16>), g, dim3(512), 0, s, E, K, N, A, l, Z);
        else if (l <= 40) hipLaunchKernelGGL((k_lorc_cols<40>), g, dim3(512), 0, s, E, K, N, A, l, Z);
        else hipLaunchKernelGGL((k_lorc_cols<kLMax>), g, dim3(512), 0, s, E, K, N, A, l, Z);
    };
    auto gram = [&](const float* A, int64_t R) {
        const int parts = (int)(R < kGramParts ? R : kGramParts);
        hipLaunchKernelGGL(k_lorc_gram, dim3(parts), dim3(256), 0, s, A, R, l, part);
        return parts;
    };
    auto orth = [&](float* A, int64_t R) {
        for (int pass = 0; pass < 2; ++pass) {  // the second pass removes what rounding left of the first
            const int parts = gram(A, R);
            hipLaunchKernelGGL(k_lorc_chol, dim3(1), dim3(256), 0, s, part, parts, l, Lf);
            hipLaunchKernelGGL(k_lorc_apply, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, s, A, R, l, Lf);
        }
    };

    rows(Omega, Ya);
    orth(Ya, K);
    for (int it = 0; it < power_iters; ++it) {
        cols(Ya, Za);
        orth(Za, N);
        rows(Za, Ya);
        orth(Ya, K);
    }
    cols(Ya, Za);  // B^T = E^T Y
    const int parts = gram(Za, N);
    hipLaunchKernelGGL(k_lorc_eig, dim3(1), dim3(128), 0, s, part, parts, l, r, CU, CV, sigma);
    hipLaunchKernelGGL(k_lorc_emit, dim3((unsigned)((K * r + 255) / 256)), dim3(256), 0, s, Ya, K, l, r, CU, U, 0);
    hipLaunchKernelGGL(k_lorc_emit, dim3((unsigned)((N * r + 255) / 256)), dim3(256), 0, s, Za, N, l, r, CV, V, 1);
    return hipGetLastError();
}

}  // namespace zqfp
