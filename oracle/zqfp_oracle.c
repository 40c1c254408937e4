/*
 * zqfp_oracle.c -- plain CPU oracle for the W4A8 (FP4 weight x FP8 activation)
 * linear-layer path of ZeroQuant-FP.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is slow on purpose, shares no code,
 * header, table or helper with the HIP library, and must only be called from
 * tests, the smoke check and the benchmark's "cpu_baseline" leg.  The product
 * path never routes through it.
 *
 * What each function follows (paper = ZeroQuant-FP):
 *   formats      : Section 2 (ExMy notation: sign + x exponent bits + y
 *                  mantissa bits; FP8 = E4M3 / E5M2, FP4 = E2M1) and Section 4
 *                  (E4M3 and E2M1 are the formats used).
 *   act quantizer: Section 3 (token-wise activation quantization), Eq. (1) for
 *                  the role of the real scale S (value / S is cast to the
 *                  format, code * S is the de-quantized value), Appendix A.
 *   weight packer: Section 3 (fine-grained / group-wise quantization),
 *                  "Casting the FP4 to FP8": S = 2^n, methods (M1) and (M2).
 *   shift cast   : Section 3 "Casting the FP4 to FP8" and its footnote on E5M2.
 *   gemm         : the W4A8 linear layer the cast exists for (Sections 1, 3):
 *                  Y = Q8(X) . Q4(W), written out as the plain definition with
 *                  an fp64 sum.
 *   rmsnorm,     : the normalisations whose output Section 3 quantizes (textbook
 *   layernorm      definitions; see orc_rmsnorm_bf16, orc_layernorm_bf16).
 *   add, relu,   : the other producers of quantized activations (residual add in front
 *   swiglu         of the normalisation; the ReLU in front of fc2, Section 3 "Distribution
 *                  of Activations"; its gated counterpart in the LLaMA models of Section 4).
 *   lorc         : Section 3 (LoRC: the low-rank product U.V is added to the
 *                  quantized weight), Appendix A (rank 8 for LLaMA).
 *
 * Readings taken where the paper is silent:
 *   - S = absmax / format_max (448 for E4M3, 6 for E2M1), symmetric (Z = 0).
 *   - E4M3 is the OCP "FN" flavour: bias 7, no infinities, S.1111.111 = NaN,
 *     max finite 448.
 *   - Encoders round to the nearest representable value, ties to the code
 *     with an even last bit, saturate at the largest finite value and copy
 *     the sign bit of the input.
 *   - n in S = 2^n is any integer (negative allowed).
 *   - M2's "compute group" is one output channel (one column of the K x N W).
 *   - The LoRC branch sees the un-quantized bf16 X:  Y += (X.U).V.
 *   - Activation quantizer arithmetic is a fixed sequence of IEEE binary32
 *     operations so that "bit exact" is well defined:
 *       amax = max|x|; sx = amax/448; inv = 448/amax; y = x*inv; code = enc(y).
 *     A row with amax < 2^-96 (this covers an all-zero row) gets sx = 1 and
 *     signed-zero codes.
 *   - M1 exponent n = min{ n integer : amax_g <= 6 * 2^n }  (this is
 *     ceil(log2(amax_g / 6)) evaluated without a logarithm), clamped to
 *     [-126, 127]; a zero group gets n = 0.  The stored byte is n + 127.
 *   - M2: c[n] = fl32(amax_max / 6), k_g = min{ k >= 0 : amax_max <= amax_g *
 *     2^k } (= ceil(log2(S_max / S_g))), clamped to 15; a zero group gets 15.
 *     The stored byte is 127 - k_g.  y = fl32(w / c[n]) * 2^k_g.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 * Floating point: fp64 everywhere except where the sequence above says binary32.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* storage formats of the inputs                                       */
/* ------------------------------------------------------------------ */

/* bfloat16 bits -> binary32 (bfloat16 is the upper half of a binary32) */
static float bf16_bits_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* IEEE binary16 bits -> double */
static double fp16_bits_to_f64(uint16_t h)
{
    int s = h >> 15, e = (h >> 10) & 31, m = h & 1023;
    double v;
    if (e == 31)
        v = m ? NAN : INFINITY;
    else if (e == 0)
        v = ldexp((double)m, -24);
    else
        v = ldexp((double)(1024 + m), e - 25);
    return s ? -v : v;
}

/* ------------------------------------------------------------------ */
/* ExMy formats (Section 2)                                            */
/* ------------------------------------------------------------------ */

/* E4M3 (FN): bias 7.  E = 0: m * 2^-9.  E = 1..15: (1 + m/8) * 2^(E-7).
 * S.1111.111 is NaN; there is no infinity. */
double orc_e4m3_decode(uint8_t c)
{
    int s = c >> 7, E = (c >> 3) & 15, m = c & 7;
    double v;
    if (E == 15 && m == 7)
        return NAN;
    v = (E == 0) ? ldexp((double)m, -9) : ldexp(1.0 + m / 8.0, E - 7);
    return s ? -v : v;
}

/* E5M2: bias 15, IEEE-like (E = 31: inf / NaN). */
double orc_e5m2_decode(uint8_t c)
{
    int s = c >> 7, E = (c >> 2) & 31, m = c & 3;
    double v;
    if (E == 31)
        v = m ? NAN : INFINITY;
    else
        v = (E == 0) ? ldexp((double)m, -16) : ldexp(1.0 + m / 4.0, E - 15);
    return s ? -v : v;
}

/* E2M1: bias 1.  E = 0: m * 0.5.  E = 1..3: (1 + m/2) * 2^(E-1).  Bit 3 = sign. */
double orc_e2m1_decode(uint8_t c)
{
    int s = (c >> 3) & 1, E = (c >> 1) & 3, m = c & 1;
    double v = (E == 0) ? 0.5 * m : ldexp(1.0 + m / 2.0, E - 1);
    return s ? -v : v;
}

/* Nearest finite magnitude among the values vals[0..top] of a format whose
 * positive codes are increasing in value; a tie goes to the code whose last
 * bit is 0; anything beyond the largest value lands on it (saturation). */
static uint8_t nearest_code(double a, const double *vals, int top)
{
    int best = 0;
    double bestd = fabs(vals[0] - a);
    for (int c = 1; c <= top; ++c) {
        double d = fabs(vals[c] - a);
        if (d < bestd || (d == bestd && (c & 1) == 0)) {
            best = c;
            bestd = d;
        }
    }
    return (uint8_t)best;
}

/* binary32 -> E4M3 code: nearest, ties to even code, saturating, sign copied. */
uint8_t orc_e4m3_encode(float y)
{
    double vals[0x7F];
    for (int c = 0; c <= 0x7E; ++c)
        vals[c] = orc_e4m3_decode((uint8_t)c);
    uint8_t s = signbit(y) ? 0x80 : 0x00;
    return s | nearest_code(fabs((double)y), vals, 0x7E);
}

/* real -> E2M1 code: nearest, ties to even code, saturating, sign copied. */
uint8_t orc_e2m1_encode(double y)
{
    double vals[8];
    for (int c = 0; c <= 7; ++c)
        vals[c] = orc_e2m1_decode((uint8_t)c);
    uint8_t s = signbit(y) ? 0x8 : 0x0;
    return s | nearest_code(fabs(y), vals, 0x7);
}

/* ------------------------------------------------------------------ */
/* FP4 -> FP8 by exponent shift (Section 3, "Casting the FP4 to FP8")   */
/* ------------------------------------------------------------------ */

/* Put the E2M1 code into an FP8 container (0 = E4M3, 1 = E5M2) and apply the
 * power-of-two group scale 2^n by adding n to the exponent FIELD -- integer
 * work only, no multiply, no rounding.  Returns 0 and the FP8 code if the
 * result is a normal number of the container (or zero), -1 if the shifted
 * exponent leaves the container's normal range (the caller must then not use
 * the shift path for that n). */
int orc_fp4_to_fp8_shift(uint8_t code4, int n, int container, uint8_t *code8)
{
    int mant_bits = container ? 2 : 3;
    int bias8 = container ? 15 : 7;
    int emax_field = container ? 30 : 15; /* E4M3: E = 15 is finite (m < 7) */
    int s = (code4 >> 3) & 1, E = (code4 >> 1) & 3, m = code4 & 1;
    int E8, m8;
    if (E == 0 && m == 0) { /* zero stays zero whatever the shift */
        *code8 = (uint8_t)(s << 7);
        return 0;
    }
    if (E == 0) { /* the one E2M1 subnormal, 0.5 = 1.0 * 2^-1 */
        E8 = -1 + bias8;
        m8 = 0;
    } else { /* (1 + m/2) * 2^(E-1): re-bias, widen the mantissa */
        E8 = (E - 1) + bias8;
        m8 = m << (mant_bits - 1);
    }
    E8 += n; /* the shift */
    if (E8 < 1 || E8 > emax_field)
        return -1;
    *code8 = (uint8_t)((s << 7) | (E8 << mant_bits) | m8);
    return 0;
}

/* ------------------------------------------------------------------ */
/* token-wise activation quantizer (Section 3, Appendix A)             */
/* ------------------------------------------------------------------ */

/* X: M x K bf16 bits, row stride ldx.  Xq: M x K E4M3 codes.  sx: M scales. */
void orc_quantize_act(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                      uint8_t *Xq, float *sx)
{
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t *row = X + m * ldx;
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float a = fabsf(bf16_bits_to_f32(row[k]));
            if (a > amax)
                amax = a;
        }
        if (amax < 0x1p-96f) {
            sx[m] = 1.0f;
            for (int64_t k = 0; k < K; ++k)
                Xq[m * K + k] = (uint8_t)((row[k] >> 15) << 7);
            continue;
        }
        volatile float s = amax / 448.0f;   /* one binary32 division */
        volatile float inv = 448.0f / amax; /* one binary32 division */
        sx[m] = s;
        for (int64_t k = 0; k < K; ++k) {
            volatile float y = bf16_bits_to_f32(row[k]) * inv; /* one binary32 product */
            Xq[m * K + k] = orc_e4m3_encode(y);
        }
    }
}

/* ------------------------------------------------------------------ */
/* RMS normalisation feeding the quantizer                             */
/* ------------------------------------------------------------------ */

/* binary32 -> bfloat16 bits, round to nearest even (finite inputs) */
static uint16_t f32_to_bf16_bits_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* The activations the paper quantizes token-wise are outputs of a normalisation
 * layer (Section 3, "Distribution of Activations": the inputs of attn.q_proj and
 * fc1 "have undergone layer-normalization"); for the LLaMA models of Section 4
 * that layer is RMSNorm.  This is its textbook definition,
 *     y[k] = x[k] / sqrt(mean_k(x[k]^2) + eps) * g[k],
 * with the result rounded to bfloat16, i.e. what a stand-alone normalisation
 * kernel would hand to orc_quantize_act.  Fixed arithmetic so that the codes
 * downstream have one right answer: the sum of squares in binary64 (every
 * square of a bfloat16 is exact there), then binary32 steps
 *     ms = fl32(ss / K); t = ms + eps; s = sqrt(t); rstd = 1 / s;
 *     y = bf16_rne( (x * rstd) * g ).
 * eps must be positive (an all-zero row then gives zeros).
 * X: M x K bf16 bits, row stride ldx.  g: K bf16 bits.  Y: M x K bf16 bits, dense. */
void orc_rmsnorm_bf16(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                      const uint16_t *g, float eps, uint16_t *Y)
{
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t *row = X + m * ldx;
        double ss = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double x = (double)bf16_bits_to_f32(row[k]);
            ss += x * x;
        }
        volatile float ms = (float)(ss / (double)K);
        volatile float t = ms + eps;
        volatile float s = sqrtf(t);
        volatile float rstd = 1.0f / s;
        for (int64_t k = 0; k < K; ++k) {
            volatile float a = bf16_bits_to_f32(row[k]) * rstd;
            volatile float b = a * bf16_bits_to_f32(g[k]);
            Y[m * K + k] = f32_to_bf16_bits_rne(b);
        }
    }
}

/* Layer normalisation, the producer the paper names for the OPT models it
 * inspects (Section 3, "Distribution of Activations": attn.q_proj and fc1 inputs
 * come out of "layer-normalization").  Textbook definition,
 *     y[k] = (x[k] - mean) / sqrt(var + eps) * g[k] + b[k],
 *     mean = sum x / K,  var = sum x^2 / K - mean^2  (population variance),
 * result rounded to bfloat16.  Fixed arithmetic: both sums, the mean and the
 * variance (clamped at 0) in binary64; then binary32 steps, each rounded once,
 *     mu = fl32(mean); v = fl32(var); rstd = 1 / sqrt(v + eps);
 *     y = bf16_rne( ((x - mu) * rstd) * g + b ).
 * eps must be positive.  X: M x K bf16 bits, row stride ldx.  g, b: K bf16 bits.
 * Y: M x K bf16 bits, dense. */
void orc_layernorm_bf16(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                        const uint16_t *g, const uint16_t *b, float eps, uint16_t *Y)
{
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t *row = X + m * ldx;
        double s1 = 0.0, s2 = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double x = (double)bf16_bits_to_f32(row[k]);
            s1 += x;
            s2 += x * x;
        }
        double mean = s1 / (double)K;
        double var = s2 / (double)K - mean * mean;
        if (var < 0.0)
            var = 0.0;
        volatile float mu = (float)mean;
        volatile float v = (float)var;
        volatile float t = v + eps;
        volatile float sd = sqrtf(t);
        volatile float rstd = 1.0f / sd;
        for (int64_t k = 0; k < K; ++k) {
            volatile float d = bf16_bits_to_f32(row[k]) - mu;
            volatile float a = d * rstd;
            volatile float c = a * bf16_bits_to_f32(g[k]);
            volatile float e = c + bf16_bits_to_f32(b[k]);
            Y[m * K + k] = f32_to_bf16_bits_rne(e);
        }
    }
}

/* ------------------------------------------------------------------ */
/* other producers of the quantized activations                        */
/* ------------------------------------------------------------------ */

/* Residual stream in front of a normalisation: h = x + r, rounded to bfloat16 (what a stand-alone
 * add kernel hands on, both to the normalisation and to the next residual connection).  One
 * binary32 addition, then bfloat16 round-to-nearest-even.
 * X, R: M x K bf16 bits, row strides ldx, ldr.  H: M x K bf16 bits, dense. */
void orc_add_bf16(const uint16_t *X, const uint16_t *R, int64_t M, int64_t K,
                  int64_t ldx, int64_t ldr, uint16_t *H)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            volatile float h = bf16_bits_to_f32(X[m * ldx + k]) + bf16_bits_to_f32(R[m * ldr + k]);
            H[m * K + k] = f32_to_bf16_bits_rne(h);
        }
}

/* The input of fc2 is the output of a ReLU (Section 3, "Distribution of Activations", observation
 * (2): negative values are voided, positive values pass unmodified).  y = x if x > 0, else +0.
 * X: M x K bf16 bits, row stride ldx.  Y: M x K bf16 bits, dense. */
void orc_relu_bf16(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, uint16_t *Y)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            uint16_t x = X[m * ldx + k];
            Y[m * K + k] = bf16_bits_to_f32(x) > 0.0f ? x : 0;
        }
}

/* The LLaMA counterpart of that producer (the models of Section 4 gate their feed-forward layer):
 * the input of the down projection is silu(g) * u with silu(g) = g / (1 + exp(-g)).  Evaluated in
 * binary64 (library exp), then rounded to binary32 and from there to bfloat16:
 *     t = g / (1 + exp(-g)) * u;  y = bf16_rne(fl32(t)).
 * G, U: M x K bf16 bits, row strides ldg, ldu.  Y: M x K bf16 bits, dense. */
void orc_swiglu_bf16(const uint16_t *G, const uint16_t *U, int64_t M, int64_t K,
                     int64_t ldg, int64_t ldu, uint16_t *Y)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            double g = (double)bf16_bits_to_f32(G[m * ldg + k]);
            double u = (double)bf16_bits_to_f32(U[m * ldu + k]);
            double t = g / (1.0 + exp(-g)) * u;
            Y[m * K + k] = f32_to_bf16_bits_rne((float)t);
        }
}

/* ------------------------------------------------------------------ */
/* group-wise FP4 weight quantizer with power-of-two scales (M1, M2)   */
/* ------------------------------------------------------------------ */

/* (M1)  n = ceil(log2(amax/6)) as the least integer with amax <= 6 * 2^n. */
static int m1_exponent(double amax)
{
    int n = 0;
    if (amax == 0.0)
        return 0;
    while (amax > ldexp(6.0, n))
        ++n;
    while (amax <= ldexp(6.0, n - 1))
        --n;
    if (n < -126) n = -126;
    if (n > 127) n = 127;
    return n;
}

/* (M2)  k = ceil(log2(S_max / S_g)) as the least k >= 0 with S_max <= S_g 2^k;
 * S = amax / 6 on both sides, so the 6 cancels. */
static int m2_shift(double amax_max, double amax_g)
{
    int k = 0;
    if (amax_g == 0.0)
        return 15;
    while (k < 15 && amax_max > ldexp(amax_g, k))
        ++k;
    return k;
}

/* W: K x N bf16 bits, row stride ldw (W[k][n]: input feature k, output
 * channel n).  Groups are G consecutive k for one n.
 * mode 1 = (M1), mode 2 = (M2) with one compute group per output channel.
 * codes: K x N, one E2M1 code per byte.  exps: (K/G) x N bytes, value n + 127
 * where the group's scale is c[n] * 2^n.  colscale: N floats (1 for M1).
 * Returns the number of elements whose |w / S^| exceeded 6 (saturated). */
int64_t orc_pack_weight(const uint16_t *W, int64_t K, int64_t N, int64_t ldw,
                        int G, int mode, uint8_t *codes, uint8_t *exps,
                        float *colscale)
{
    int64_t ng = K / G, clipped = 0;
    double *amax = (double *)malloc((size_t)ng * sizeof(double));
    for (int64_t n = 0; n < N; ++n) {
        double amax_max = 0.0;
        for (int64_t g = 0; g < ng; ++g) {
            double a = 0.0;
            for (int64_t k = g * G; k < (g + 1) * G; ++k) {
                double v = fabs((double)bf16_bits_to_f32(W[k * ldw + n]));
                if (v > a)
                    a = v;
            }
            amax[g] = a;
            if (a > amax_max)
                amax_max = a;
        }
        if (mode == 1) {
            colscale[n] = 1.0f;
            for (int64_t g = 0; g < ng; ++g) {
                int e = m1_exponent(amax[g]);
                exps[g * N + n] = (uint8_t)(e + 127);
                for (int64_t k = g * G; k < (g + 1) * G; ++k) {
                    double w = (double)bf16_bits_to_f32(W[k * ldw + n]);
                    double y = ldexp(w, -e); /* exact: w / 2^e */
                    if (fabs(y) > 6.0)
                        ++clipped;
                    codes[k * N + n] = orc_e2m1_encode(y);
                }
            }
        } else {
            volatile float c = (float)amax_max / 6.0f; /* one binary32 division */
            if (amax_max == 0.0)
                c = 1.0f;
            colscale[n] = c;
            for (int64_t g = 0; g < ng; ++g) {
                int kg = m2_shift(amax_max, amax[g]);
                exps[g * N + n] = (uint8_t)(127 - kg);
                for (int64_t k = g * G; k < (g + 1) * G; ++k) {
                    volatile float q = bf16_bits_to_f32(W[k * ldw + n]) / c; /* binary32 division */
                    double y = ldexp((double)q, kg);
                    if (fabs(y) > 6.0)
                        ++clipped;
                    codes[k * N + n] = orc_e2m1_encode(y);
                }
            }
        }
    }
    free(amax);
    return clipped;
}

/* ------------------------------------------------------------------ */
/* the W4A8 linear layer, plain definition                             */
/* ------------------------------------------------------------------ */

/* acc[m][n] = sum_k dec8(Xq[m][k]) * dec4(codes[k][n]) * 2^(exps[k/G][n]-127)
 * summed in k order in fp64;
 *   Y[m][n]    = fl32( fl32(sx[m] * colscale[n]) * acc )           (no LoRC)
 *   Y[m][n]    = fl32( fl32(sx*c) * acc + sum_j T[m][j] * V[j][n] ) (LoRC, r > 0)
 *   Sabs[m][n] = fl32(sx*c) * sum_k |a*w|  (+ sum_j |T*V|)
 * T: M x r binary32, V: r x N binary16 bits.  Sabs may be NULL. */
void orc_gemm(const uint8_t *Xq, const float *sx, int64_t M, int64_t K,
              const uint8_t *codes, const uint8_t *exps, const float *colscale,
              int64_t N, int G, const float *T, const uint16_t *V, int r,
              float *Y, double *Sabs, int threads)
{
    int64_t ng = K / G;
    double dec8[256], dec4[16];
    for (int c = 0; c < 256; ++c)
        dec8[c] = orc_e4m3_decode((uint8_t)c);
    for (int c = 0; c < 16; ++c)
        dec4[c] = orc_e2m1_decode((uint8_t)c);
    double *p2 = (double *)malloc((size_t)(ng * N) * sizeof(double));
    for (int64_t i = 0; i < ng * N; ++i)
        p2[i] = ldexp(1.0, (int)exps[i] - 127);
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t m = 0; m < M; ++m) {
        double *acc = (double *)calloc((size_t)N, sizeof(double));
        double *aab = (double *)calloc((size_t)N, sizeof(double));
        for (int64_t k = 0; k < K; ++k) {
            double a = dec8[Xq[m * K + k]];
            const uint8_t *crow = codes + k * N;
            const double *prow = p2 + (k / G) * N;
            for (int64_t n = 0; n < N; ++n) {
                double p = a * (dec4[crow[n]] * prow[n]);
                acc[n] += p;
                aab[n] += fabs(p);
            }
        }
        for (int64_t n = 0; n < N; ++n) {
            volatile float sc = sx[m] * colscale[n]; /* one binary32 product */
            double y = (double)sc * acc[n], ya = fabs((double)sc) * aab[n];
            for (int j = 0; j < r; ++j) {
                double tv = (double)T[m * r + j] * fp16_bits_to_f64(V[(int64_t)j * N + n]);
                y += tv;
                ya += fabs(tv);
            }
            Y[m * N + n] = (float)y;
            if (Sabs)
                Sabs[m * N + n] = ya;
        }
        free(acc);
        free(aab);
    }
    free(p2);
}

/* The same definition for a list of sampled outputs (ms[i], ns[i]); used where
 * the full matrix is too large for the loop above to finish in seconds. */
void orc_gemm_samples(const uint8_t *Xq, const float *sx, int64_t M, int64_t K,
                      const uint8_t *codes, const uint8_t *exps,
                      const float *colscale, int64_t N, int G, const float *T,
                      const uint16_t *V, int r, const int64_t *ms,
                      const int64_t *ns, int64_t count, float *Y, double *Sabs)
{
    (void)M;
    for (int64_t i = 0; i < count; ++i) {
        int64_t m = ms[i], n = ns[i];
        double acc = 0.0, aab = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double w = orc_e2m1_decode(codes[k * N + n]) *
                       ldexp(1.0, (int)exps[(k / G) * N + n] - 127);
            double p = orc_e4m3_decode(Xq[m * K + k]) * w;
            acc += p;
            aab += fabs(p);
        }
        volatile float sc = sx[m] * colscale[n];
        double y = (double)sc * acc, ya = fabs((double)sc) * aab;
        for (int j = 0; j < r; ++j) {
            double tv = (double)T[m * r + j] * fp16_bits_to_f64(V[(int64_t)j * N + n]);
            y += tv;
            ya += fabs(tv);
        }
        Y[i] = (float)y;
        if (Sabs)
            Sabs[i] = ya;
    }
}

/* ------------------------------------------------------------------ */
/* W8A8: FP8 (E4M3) weights against FP8 activations                     */
/* ------------------------------------------------------------------ */

/* The paper's second weight format (Section 4, Table 2, rows W8A8 / FP -- FP;
 * "FP8 weights rival INT8"): group-wise E4M3 weights, fine-grained quantization
 * as for FP4 (Section 3), scale S = amax / 448 (the format's largest value in
 * place of E2M1's 6).
 *   mode 0: S_g real (what the paper's W8A8 rows use): S_g = fl32(amax_g / 448),
 *           y = fl32(w / S_g); gscale[g][n] = S_g (1 for a zero group), exps = 127,
 *           colscale = 1.
 *   mode 1: (M1) S^_g = 2^n, least n with amax_g <= 448 * 2^n; y = w * 2^-n (exact).
 *   mode 2: (M2) c[n] = fl32(amax_max / 448), S^_g = c[n] * 2^-k with the same k as
 *           for FP4 (the format's largest value cancels in S_max / S_g);
 *           y = fl32(w / c[n]) * 2^k; values beyond 448 saturate.
 * codes: K x N E4M3 codes.  exps: (K/G) x N bytes (n + 127, or 127 - k).
 * gscale: (K/G) x N floats, written in every mode (2^n, c 2^-k: the group's whole
 * scale), may be NULL.  Returns the number of saturated elements. */
static int m1_exponent_fmax(double amax, double fmax)
{
    int n = 0;
    if (amax == 0.0)
        return 0;
    while (amax > ldexp(fmax, n))
        ++n;
    while (amax <= ldexp(fmax, n - 1))
        --n;
    if (n < -126) n = -126;
    if (n > 127) n = 127;
    return n;
}

int64_t orc_pack_weight_fp8(const uint16_t *W, int64_t K, int64_t N, int64_t ldw,
                            int G, int mode, uint8_t *codes, uint8_t *exps,
                            float *colscale, float *gscale)
{
    int64_t ng = K / G, clipped = 0;
    double *amax = (double *)malloc((size_t)ng * sizeof(double));
    for (int64_t n = 0; n < N; ++n) {
        double amax_max = 0.0;
        for (int64_t g = 0; g < ng; ++g) {
            double a = 0.0;
            for (int64_t k = g * G; k < (g + 1) * G; ++k) {
                double v = fabs((double)bf16_bits_to_f32(W[k * ldw + n]));
                if (v > a)
                    a = v;
            }
            amax[g] = a;
            if (a > amax_max)
                amax_max = a;
        }
        volatile float c = 1.0f;
        if (mode == 2 && amax_max > 0.0)
            c = (float)amax_max / 448.0f; /* one binary32 division */
        colscale[n] = c;
        for (int64_t g = 0; g < ng; ++g) {
            int e = 0;        /* exponent of the power of two in the group's scale */
            volatile float s = 1.0f; /* the real part of the group's scale */
            if (mode == 0) {
                if (amax[g] > 0.0)
                    s = (float)amax[g] / 448.0f;
            } else if (mode == 1) {
                e = m1_exponent_fmax(amax[g], 448.0);
            } else {
                e = -m2_shift(amax_max, amax[g]);
                s = c;
            }
            exps[g * N + n] = (uint8_t)(e + 127);
            if (gscale)
                gscale[g * N + n] = (float)ldexp((double)s, e);
            for (int64_t k = g * G; k < (g + 1) * G; ++k) {
                float w = bf16_bits_to_f32(W[k * ldw + n]);
                volatile float q = (mode == 1) ? w : w / s; /* binary32 division (none under M1) */
                double y = ldexp((double)q, -e);               /* exact */
                if (fabs(y) > 448.0)
                    ++clipped;
                /* |y| <= 448 * 2 at most, far inside binary32: the conversion is exact */
                codes[k * N + n] = orc_e4m3_encode((float)y);
            }
        }
    }
    free(amax);
    return clipped;
}

/* acc[m][n] = sum_k dec8(Xq[m][k]) * dec8(codes[k][n]) * scale(k/G, n), in k order in fp64, where the
 * group's scale is 2^(exps-127) (modes 1, 2; gscale == NULL) or gscale[g][n] (mode 0);
 * Y = fl32( fl32(sx[m] * colscale[n]) * acc )  (+ T.V as in orc_gemm).  One output at a time: for the
 * full matrix pass every (m, n). */
void orc_gemm_w8_samples(const uint8_t *Xq, const float *sx, int64_t M, int64_t K,
                         const uint8_t *codes, const uint8_t *exps, const float *colscale,
                         const float *gscale, int64_t N, int G, const float *T,
                         const uint16_t *V, int r, const int64_t *ms, const int64_t *ns,
                         int64_t count, float *Y, double *Sabs)
{
    (void)M;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < count; ++i) {
        int64_t m = ms[i], n = ns[i];
        double acc = 0.0, aab = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double sc = gscale ? (double)gscale[(k / G) * N + n]
                               : ldexp(1.0, (int)exps[(k / G) * N + n] - 127);
            double p = orc_e4m3_decode(Xq[m * K + k]) * (orc_e4m3_decode(codes[k * N + n]) * sc);
            acc += p;
            aab += fabs(p);
        }
        volatile float sc = sx[m] * colscale[n];
        double y = (double)sc * acc, ya = fabs((double)sc) * aab;
        for (int j = 0; j < r; ++j) {
            double tv = (double)T[m * r + j] * fp16_bits_to_f64(V[(int64_t)j * N + n]);
            y += tv;
            ya += fabs(tv);
        }
        Y[i] = (float)y;
        if (Sabs)
            Sabs[i] = ya;
    }
}

/* ------------------------------------------------------------------ */
/* LoRC left factor (Section 3): T = X . U from the un-quantized X      */
/* ------------------------------------------------------------------ */

/* X: M x K bf16 bits (stride ldx); U: K x r binary16 bits.  T[m][j] is the
 * fp64 sum rounded once to binary32; Tabs[m][j] = sum_k |x*u| (may be NULL). */
void orc_lorc_left(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                   const uint16_t *U, int r, float *T, double *Tabs)
{
    for (int64_t m = 0; m < M; ++m)
        for (int j = 0; j < r; ++j) {
            double s = 0.0, sa = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = (double)bf16_bits_to_f32(X[m * ldx + k]) *
                           fp16_bits_to_f64(U[k * r + j]);
                s += p;
                sa += fabs(p);
            }
            T[m * r + j] = (float)s;
            if (Tabs)
                Tabs[m * r + j] = sa;
        }
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
