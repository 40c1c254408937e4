/*
 * zqfp.h -- C ABI of libzqfp: the W4A8 linear-layer inference path of
 * ZeroQuant-FP on AMD MI355X (gfx950).
 *
 *   Y = Q8(X) . Q4(W)  [+ (X.U).V]
 *
 * Q8: token-wise FP8 (E4M3) activation quantization.  Q4: group-wise FP4
 * (E2M1) weight quantization whose group scales are powers of two, so that
 * aligning an FP4 weight with the FP8 activation precision is an exponent
 * adjustment and never a multiply (paper Section 3, "Casting the FP4 to
 * FP8", methods M1 and M2).  The optional term is LoRC, the low-rank
 * compensation of the weight quantization error (paper Section 3).
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer owned by the caller unless a
 *     parameter is documented as host.  The library keeps no reference to any
 *     of them after the call's work has run.
 *   - Every call only enqueues work on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream); it never synchronizes the device and
 *     never allocates or frees device memory.
 *   - Matrices are row-major.  X is M x K (tokens x input features), W is
 *     K x N (input features x output channels), groups are G consecutive k of
 *     one output channel n.
 *   - Return value: 0 on success, a negative ZQFP_E_* code otherwise; nothing
 *     is enqueued when an argument check fails.  Inputs must be finite; the
 *     result for NaN / infinity inputs is unspecified.
 *   - Shape limits: K % 128 == 0, G % 32 == 0, K % G == 0, K / G <= 256,
 *     0 <= r <= 64 (else ZQFP_E_SHAPE).
 *     M and N are arbitrary (M == 0 or N == 0 is a successful no-op).
 *     X, Xq, U, Y, Omega, gain / bias / residual pointers and workspaces must be
 *     16-byte aligned, packed blobs 256-byte aligned, and ldx (and the other
 *     activation row strides) multiples of 8 elements (ZQFP_E_ALIGN).  The
 *     offline weight-side calls read W element by element: W needs only its
 *     natural 2-byte alignment and ldw >= N.
 *   - Thread safety: calls may be made from several host threads; the error
 *     text is per thread, one-time kernel set-up is serialised inside.
 */
#ifndef ZQFP_H
#define ZQFP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZQFP_OK 0
#define ZQFP_E_NULL (-1)  /* a required pointer is NULL */
#define ZQFP_E_SHAPE (-2) /* a size violates the limits above */
#define ZQFP_E_ALIGN (-3) /* pointer or leading dimension alignment */
#define ZQFP_E_MODE (-4)  /* unknown scale mode / output dtype / accumulation mode */
#define ZQFP_E_HIP (-5)   /* a HIP call failed; see zqfp_last_hip_error() */
#define ZQFP_E_WORKSPACE (-6) /* workspace given but smaller than the query says,
                                 or (static variant) larger than the built-in array */
#define ZQFP_E_BLOB (-7)  /* zqfp_packed_weight_check: not a blob of this (K, N, G) */

#define ZQFP_SCALE_M1 1 /* S^ = 2^ceil(log2 S) per group               */
#define ZQFP_SCALE_M2 2 /* S^_g = S_max / 2^ceil(log2(S_max / S_g))    */

#define ZQFP_OUT_F32 0
#define ZQFP_OUT_BF16 1

/* How the matrix cores sum the (exact) FP8 x FP4 products.  The gfx950 FP8
 * matrix instruction adds each run of 8 consecutive k in a narrow window
 * anchored at the run's largest exponent; a product more than 8 binades
 * below it loses low bits (truncation toward zero).
 *   EXACT  every activation tile is fed twice, once with only its codes of
 *          exponent field >= 8 and once with the others; inside each half no
 *          product is truncated, so the only rounding left is the float32
 *          accumulation.  Twice the matrix-core work.  Meets
 *          |err| <= 2^-18 * sum_k |a_k w_k|.
 *   FAST   one pass.  |err| < 2^-10 * sum_k |a_k w_k| in the worst case
 *          (about 2^-16 on activations with outlier channels). */
#define ZQFP_ACCUM_EXACT 0
#define ZQFP_ACCUM_FAST 1

/* Library version (major * 100 + minor). */
int zqfp_version(void);

/* Text of the last HIP error seen by this thread's calls (host string, owned
 * by the library, valid until the next failing call). */
const char *zqfp_last_hip_error(void);

/*
 * quantize_act_fp8 -- token-wise FP8 activation quantization (paper Section 3
 * and Appendix A: one scale per token; Section 2 / Section 4: format E4M3).
 *
 *   X   [M, K] bfloat16, row stride ldx elements                    (in)
 *   Xq  [M, K] uint8 E4M3 codes (bias 7, max 448, no infinities), dense (out)
 *   sx  [M]    float32 token scales: X[m,k] ~ sx[m] * value(Xq[m,k])  (out)
 *
 * Per token, in IEEE binary32: amax = max|x|, sx = amax / 448,
 * inv = 448 / amax, code = E4M3(x * inv) rounded to nearest (ties to the even
 * code), saturating, sign kept.  A token with amax < 2^-96 gets sx = 1 and
 * signed-zero codes.
 *
 * Optional LoRC left factor, computed in the same sweep over X (paper
 * Section 3, LoRC): if U != NULL,
 *   U   [K, r] binary16, dense                                      (in)
 *   T   [M, r] float32, dense:  T = X . U  (un-quantized X, fp32 sums) (out)
 * Pass U = NULL, r = 0, T = NULL to skip it.
 */
int zqfp_quantize_act_fp8(const void *X, int64_t M, int64_t K, int64_t ldx,
                          uint8_t *Xq, float *sx,
                          const void *U, int r, float *T,
                          void *stream);

/*
 * rmsnorm_quantize_act_fp8 -- the same quantizer fused behind the RMS
 * normalisation that produces the activations (paper Section 3, "Distribution
 * of Activations": the quantized inputs of attn.q_proj and fc1 are outputs of
 * a normalisation layer; RMSNorm for the LLaMA models of Section 4):
 *
 *   y[m,k] = bf16( X[m,k] / sqrt(mean_k X[m,k]^2 + eps) * gain[k] )
 *
 * followed by zqfp_quantize_act_fp8 applied to y, without y ever leaving the
 * registers.  Sum of squares in binary64; then, in IEEE binary32,
 * ms = fl(ss / K), rstd = 1 / sqrt(ms + eps), y = bf16_rne((x * rstd) * gain).
 * The codes and scales are those of the unfused sequence, bit for bit.
 *
 *   gain  [K] bfloat16 (device, 16-byte aligned)                      (in)
 *   eps   > 0
 *   K     <= 32768 (a token's row is held in registers)
 *   T     = y . U when U != NULL (the LoRC branch sees the normalised y)
 * Other arguments and errors as for zqfp_quantize_act_fp8.
 */
int zqfp_rmsnorm_quantize_act_fp8(const void *X, const void *gain, float eps,
                                  int64_t M, int64_t K, int64_t ldx,
                                  uint8_t *Xq, float *sx,
                                  const void *U, int r, float *T, void *stream);

/*
 * layernorm_quantize_act_fp8 -- the same, behind a layer normalisation with
 * gain and bias (paper Section 3, "Distribution of Activations": the inputs of
 * attn.q_proj and fc1 are layer-normalisation outputs; the form the OPT models
 * of Section 4 use):
 *
 *   y[m,k] = bf16( (X[m,k] - mean_m) / sqrt(var_m + eps) * gain[k] + bias[k] )
 *
 * with the population variance var_m = mean_k X^2 - mean_m^2 (clamped at 0).
 * Sums of x and x^2, the mean and the variance in binary64; then, in IEEE
 * binary32, mu = fl(mean), v = fl(var), rstd = 1 / sqrt(v + eps),
 * y = bf16_rne(((x - mu) * rstd) * gain + bias), each operation rounded on its
 * own.  The codes and scales are those of the unfused sequence, bit for bit.
 *
 *   gain, bias  [K] bfloat16 each (device, 16-byte aligned)            (in)
 * Other arguments, limits and errors as for zqfp_rmsnorm_quantize_act_fp8.
 */
int zqfp_layernorm_quantize_act_fp8(const void *X, const void *gain,
                                    const void *bias, float eps,
                                    int64_t M, int64_t K, int64_t ldx,
                                    uint8_t *Xq, float *sx,
                                    const void *U, int r, float *T,
                                    void *stream);

/*
 * add_rmsnorm_quantize_act_fp8, add_layernorm_quantize_act_fp8 -- the two
 * calls above with the residual connection in front of the normalisation taken
 * along:  h = bf16(X + R) (one binary32 addition, round to nearest even) is
 * written to H and is what gets normalised and quantized.
 *
 *   R    [M, K] bfloat16, row stride ldr >= K (multiple of 8), 16-byte aligned  (in)
 *   H    [M, K] bfloat16, dense, 16-byte aligned; may be R itself when
 *        ldr == K (the residual stream updated in place), must not overlap
 *        X or R otherwise                                                      (out)
 * Other arguments, limits and errors as for the calls without the residual.
 */
int zqfp_add_rmsnorm_quantize_act_fp8(const void *X, const void *R, int64_t ldr,
                                      void *H, const void *gain, float eps,
                                      int64_t M, int64_t K, int64_t ldx,
                                      uint8_t *Xq, float *sx,
                                      const void *U, int r, float *T,
                                      void *stream);
int zqfp_add_layernorm_quantize_act_fp8(const void *X, const void *R,
                                        int64_t ldr, void *H, const void *gain,
                                        const void *bias, float eps,
                                        int64_t M, int64_t K, int64_t ldx,
                                        uint8_t *Xq, float *sx,
                                        const void *U, int r, float *T,
                                        void *stream);

/*
 * relu_quantize_act_fp8 -- the quantizer behind the ReLU whose output is the
 * input of fc2 (paper Section 3, "Distribution of Activations", observation
 * (2)):  y = X where X > 0, +0 elsewhere; then zqfp_quantize_act_fp8 on y.
 * K <= 32768; other arguments and errors as for zqfp_quantize_act_fp8 (T = y.U).
 */
int zqfp_relu_quantize_act_fp8(const void *X, int64_t M, int64_t K, int64_t ldx,
                               uint8_t *Xq, float *sx,
                               const void *U, int r, float *T, void *stream);

/*
 * swiglu_quantize_act_fp8 -- the same for the gated feed-forward layer of the
 * LLaMA models of paper Section 4, whose down projection reads
 *
 *   y[m,k] = bf16( silu(G[m,k]) * Up[m,k] ),   silu(g) = g / (1 + exp(-g)),
 *
 * evaluated in binary64, rounded to binary32 and from there to bfloat16; then
 * zqfp_quantize_act_fp8 on y.
 *
 *   G    [M, K] bfloat16, row stride ldg (the gate projection's output)  (in)
 *   Up   [M, K] bfloat16, row stride ldu (the up projection's output)    (in)
 *   H    [M, K] bfloat16, dense, 16-byte aligned: y itself, for a caller
 *        that wants the unquantized activation too; may be NULL        (out)
 * K <= 32768; alignment, other arguments and errors as for
 * zqfp_quantize_act_fp8 (T = y.U).
 */
int zqfp_swiglu_quantize_act_fp8(const void *G, const void *Up, int64_t ldu,
                                 void *H, int64_t M, int64_t K, int64_t ldg,
                                 uint8_t *Xq, float *sx,
                                 const void *U, int r, float *T, void *stream);

/*
 * pack_weight_fp4 -- group-wise FP4 (E2M1) weight quantization with
 * power-of-two scales (paper Section 3: fine-grained quantization; "Casting
 * the FP4 to FP8": S = 2^n with methods M1 / M2; Appendix A: group size).
 * Offline step; its output is the only weight format the GEMM reads.
 *
 *   W       [K, N] bfloat16, row stride ldw elements                (in)
 *   G       group size along K
 *   mode    ZQFP_SCALE_M1: per group n_g = ceil(log2(amax_g / 6)), scale
 *           2^n_g, column scale 1.
 *           ZQFP_SCALE_M2: per output channel c[n] = max_g amax_g / 6 (real,
 *           float32) and per group k_g = ceil(log2(S_max / S_g)) (clamped to
 *           15), scale c[n] * 2^-k_g; codes saturate at +-6.
 *   packed  zqfp_packed_weight_bytes(K, N, G) bytes, 256-byte aligned  (out)
 *
 * The blob is opaque: a 256-byte header, the E2M1 codes two per byte in the
 * register order of the gfx950 block-scaled matrix instruction, the group
 * exponents as E8M0 bytes (n + 127), and the float32 column scales.
 * zqfp_unpack_codes gives the layout-independent view.
 */
size_t zqfp_packed_weight_bytes(int64_t K, int64_t N, int G);
int zqfp_pack_weight_fp4(const void *W, int64_t K, int64_t N, int64_t ldw,
                         int G, int mode, void *packed, void *stream);

/*
 * packed_weight_check -- does a blob belong to (K, N, G)?  The GEMM calls take
 * K, N and G as arguments because the blob's header lives in device memory
 * and reading it there would force a synchronization; a blob packed for other
 * sizes would be read with the wrong layout.  A caller that wants the check
 * copies the blob's first ZQFP_BLOB_HEADER_BYTES bytes to the host once (after
 * packing has finished) and passes them here.  Pure host logic, no GPU call.
 *
 *   header  HOST pointer to the first ZQFP_BLOB_HEADER_BYTES bytes of a blob
 * Returns ZQFP_OK; ZQFP_E_NULL; ZQFP_E_SHAPE if (K, N, G) itself is outside the
 * limits; ZQFP_E_BLOB if the magic number, the layout version, K, N, G or the
 * section offsets are not those of a blob of (K, N, G).
 */
#define ZQFP_BLOB_HEADER_BYTES 256
int zqfp_packed_weight_check(const void *header, int64_t K, int64_t N, int G);

/*
 * lorc_factorize -- the two low-rank matrices of LoRC (paper Section 3: singular
 * value decomposition of the error matrix E = W - W^, the original weight minus
 * the quantized one; Appendix A: rank 8 for LLaMA, 16..56 for OPT).  Offline
 * step.  U V is the rank-r approximation of E from its r leading singular
 * triplets, with the singular values shared evenly between the factors,
 *   U = P_r diag(s_r)^(1/2),  V = diag(s_r)^(1/2) Q_r^T   (E = P diag(s) Q^T),
 * found by a subspace iteration with r + 8 columns and `power_iters` rounds
 * (2 is enough for quantization error, whose spectrum is flat), so that the
 * residual |E - U V|_F is within a fraction of a percent of the optimum.
 *
 *   W        [K, N] bfloat16, row stride ldw                           (in)
 *   packed   the blob zqfp_pack_weight_fp4 made (of W, or of any K x N
 *            matrix: E is W minus whatever the blob de-quantizes to)     (in)
 *   r        rank, 1..64, with r + 8 <= min(K, N)
 *   Omega    [N, r + 8] float32 (16-byte aligned), independent standard
 *            normal draws; the caller supplies them so that the result is
 *            reproducible                                                (in)
 *   U        [K, r] binary16      V  [r, N] binary16                     (out)
 *   sigma    [r] float32: the r leading singular values of E, descending (out)
 *   workspace  zqfp_lorc_workspace_bytes(K, N, r) bytes of device memory,
 *            256-byte aligned (E in float32 and the iteration's blocks)
 * Returns ZQFP_E_SHAPE for a rank or iteration count outside the limits.
 */
size_t zqfp_lorc_workspace_bytes(int64_t K, int64_t N, int r);
int zqfp_lorc_factorize(const void *W, int64_t K, int64_t N, int64_t ldw,
                        const void *packed, int G, int r,
                        const float *Omega, int power_iters,
                        void *U, void *V, float *sigma,
                        void *workspace, void *stream);

/*
 * gptq_pack_weight_fp4 -- zqfp_pack_weight_fp4 with GPTQ's error feedback (the
 * weight quantizer of the paper's experiments: Section 3, Appendix A), on the
 * same E2M1 grid and with the same power-of-two scales (M1 / M2).  Offline
 * step.  Input channels k = 0, 1, ... are quantized in order; the scaled error
 * of channel k is pushed onto the channels behind it,
 *   q_k = S e2m1(w_k / S);  err = (w_k - q_k) / U[k][k];  w_j -= U[k][j] err  (j > k),
 * where U is the upper Cholesky factor of the inverse Hessian of the layer's
 * inputs, inv(H) = U^T U.  A group's scale is fixed when its first channel is
 * reached, from the weights as updated so far; under M2 the column scale is
 * the ORIGINAL column's absmax / 6.  With H = I the result is the blob of
 * zqfp_pack_weight_fp4.  Arithmetic is binary32: against a float64 evaluation
 * a code can differ where an updated weight sits within rounding error of a
 * grid midpoint.
 *
 *   W         [K, N] bfloat16, row stride ldw                          (in)
 *   Hinv_u    [K, K] float32 row-major, upper triangular               (in)
 *   G         32, 64, 128 or 256
 *   packed    zqfp_packed_weight_bytes(K, N, G) bytes, 256-byte aligned (out)
 *   workspace zqfp_gptq_workspace_bytes(K, N, G) bytes of device memory,
 *             256-byte aligned (a float32 working copy of W and one block
 *             of errors)
 */
size_t zqfp_gptq_workspace_bytes(int64_t K, int64_t N, int G);
int zqfp_gptq_pack_weight_fp4(const void *W, int64_t K, int64_t N, int64_t ldw,
                              const float *Hinv_u, int G, int mode,
                              void *packed, void *workspace, void *stream);

/*
 * unpack_codes -- canonical view of a packed blob, for bit-exact comparison
 * and inspection (same K, N, G as at packing time).
 *   codes    [K, N] uint8, one E2M1 code (0..15, bit 3 = sign) per byte  (out)
 *   exps     [K/G, N] uint8 E8M0 exponent bytes                        (out)
 *   colscale [N] float32                                               (out)
 */
int zqfp_unpack_codes(const void *packed, int64_t K, int64_t N, int G,
                      uint8_t *codes, uint8_t *exps, float *colscale,
                      void *stream);

/*
 * w4a8_gemm -- the W4A8 linear layer (paper Sections 1 and 3: FP8 activations
 * against FP4 weights brought to FP8 precision by their power-of-two scale).
 *
 *   Y[m,n] = (sx[m] * colscale[n]) * sum_k value(Xq[m,k]) * value(q[k,n]) * 2^n_g(k),n
 *
 * The sum is accumulated in float32 on the matrix cores from exact products
 * (see ZQFP_ACCUM_* for how); the power of two is applied by the hardware's
 * per-32-element block exponent, never by a multiply on the weight.
 *
 *   Xq, sx   as produced by zqfp_quantize_act_fp8                     (in)
 *   packed   as produced by zqfp_pack_weight_fp4 for (K, N, G)         (in)
 *   Y        [M, N], row stride ldy elements, float32 or bfloat16     (out)
 *   workspace  zqfp_gemm_workspace_bytes(M, K, N) bytes of device memory,
 *            16-byte aligned; contents need not be initialised and are not
 *            preserved.  It is non-zero only where few output tiles meet a long
 *            K (K is then cut into slices whose float32 partial tiles are summed
 *            in fixed order by a second kernel).  NULL is always accepted: the
 *            call then runs without the split (same result within tolerance).
 *   workspace_bytes  size of what `workspace` points to.  A non-NULL workspace
 *            smaller than the query's answer is refused (ZQFP_E_WORKSPACE) and
 *            nothing is enqueued.
 */
size_t zqfp_gemm_workspace_bytes(int64_t M, int64_t K, int64_t N);
int zqfp_w4a8_gemm(const uint8_t *Xq, const float *sx, int64_t M, int64_t K,
                   const void *packed, int64_t N, int G,
                   void *Y, int64_t ldy, int out_dtype, int accum,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * w4a8_gemm_lorc -- the same layer with the LoRC correction fused into the
 * epilogue (paper Section 3, LoRC; Appendix A: rank 8 for LLaMA):
 *
 *   Y[m,n] = w4a8_gemm(...)[m,n] + sum_{j<r} T[m,j] * V[j,n]
 *
 *   T  [M, r] float32 = X . U from zqfp_quantize_act_fp8               (in)
 *   V  [r, N] binary16, dense                                          (in)
 */
int zqfp_w4a8_gemm_lorc(const uint8_t *Xq, const float *sx, int64_t M, int64_t K,
                        const void *packed, int64_t N, int G,
                        const float *T, const void *V, int r,
                        void *Y, int64_t ldy, int out_dtype, int accum,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * W8A8: FP8 (E4M3) weights against FP8 activations (paper Section 4, Table 2,
 * rows "W8A8 ... FP -- FP"; "FP8 weights rival INT8").  Group-wise weight
 * scales as for FP4 (Section 3) with the format's largest value 448 in place
 * of 6, constrained to powers of two by the same two methods (M1: per group
 * 2^ceil(log2(amax_g / 448)); M2: c[n] * 2^-k_g), so that the matrix
 * instruction's block exponent applies them.  Real-valued group scales (what the
 * paper's W8A8 rows use) would need a multiply per group and output in the
 * accumulation loop and are not offered.
 *
 * pack_weight_fp8 / unpack_codes_fp8 / packed_weight_fp8_bytes mirror the FP4
 * calls (codes are E4M3 bytes; G must be a multiple of 128).  The blob's header
 * records the code width; zqfp_packed_weight_check accepts both kinds.
 *
 * w8a8_gemm:  Y[m,n] = (sx[m] c[n]) * sum_k v(Xq[m,k]) v(q[k,n]) 2^n_g  (+ T.V).
 * Arguments as for zqfp_w4a8_gemm_lorc (T = V = NULL, r = 0: no LoRC); no
 * workspace.  Accumulation: an FP8 x FP8 product has up to 8 significant bits, so
 * inside the matrix core's 13-bit window of a run of 8 consecutive k only
 * products within 7 binades of the run's largest are summed exactly; neither
 * mode can promise the W4A8 bound (16 passes over 4 x 4 exponent bands would).
 * Worst case for both modes: |err| <= 7 * 2^-13 * sum_k |a_k w_k| (the seven
 * smaller products of a run each lose less than 2^-13 of the largest one).
 * ZQFP_ACCUM_EXACT here means two passes over the activation's exponent bands,
 * as for W4A8: it removes the part of the truncation that comes from the
 * activations' dynamic range (outlier channels), not the part that comes from
 * the weights' own spread inside a run.  Measured on the benchmark
 * distributions: relative Frobenius error 2..3 * 10^-5 and |err| <= 10^-5 *
 * sum|a w| with two passes, 3..6 * 10^-5 and 1.6 * 10^-5 with one
 * (ZQFP_ACCUM_FAST); truncation is toward zero, so the error is a small bias
 * toward smaller magnitudes rather than noise.
 */
size_t zqfp_packed_weight_fp8_bytes(int64_t K, int64_t N, int G);
int zqfp_pack_weight_fp8(const void *W, int64_t K, int64_t N, int64_t ldw,
                         int G, int mode, void *packed, void *stream);
int zqfp_unpack_codes_fp8(const void *packed, int64_t K, int64_t N, int G,
                          uint8_t *codes, uint8_t *exps, float *colscale,
                          void *stream);
int zqfp_w8a8_gemm(const uint8_t *Xq, const float *sx, int64_t M, int64_t K,
                   const void *packed, int64_t N, int G,
                   const float *T, const void *V, int r,
                   void *Y, int64_t ldy, int out_dtype, int accum, void *stream);

/*
 * w4a8_linear -- the whole layer in one call, from bfloat16 activations:
 * zqfp_quantize_act_fp8 followed by zqfp_w4a8_gemm(_lorc) (paper Section 3:
 * token-wise activation quantization is chosen for latency; for a handful of
 * tokens the quantizer's own launch is a quarter of the step).
 *
 *   - M <= 16, K <= 4096 and r == 0: ONE kernel.  The decode GEMM reads X
 *     itself and quantizes it in its prologue, with the arithmetic of
 *     zqfp_quantize_act_fp8, so Y equals the two-call sequence bit for bit.
 *     Xq and sx are optional outputs here (NULL: not written).
 *   - otherwise: the two calls, enqueued one after the other; Xq, sx (and T
 *     when r > 0) must then be given, as the buffers between them.
 *
 *   X    [M, K] bfloat16, row stride ldx (multiple of 8), 16-byte aligned   (in)
 *   U    [K, r] binary16 or NULL with r == 0;  V  [r, N] binary16          (in)
 *   Xq   [M, K] uint8, sx [M] float32, T [M, r] float32                     (out)
 *   Y, workspace, other arguments and errors as for zqfp_w4a8_gemm_lorc.
 */
int zqfp_w4a8_linear(const void *X, int64_t ldx, int64_t M, int64_t K,
                     const void *packed, int64_t N, int G,
                     const void *U, const void *V, int r,
                     uint8_t *Xq, float *sx, float *T,
                     void *Y, int64_t ldy, int out_dtype, int accum,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * w4a8_gemm_lorc_static -- zqfp_w4a8_gemm_lorc for callers that cannot allocate
 * device memory or pass a workspace along: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments without the
 * workspace (r = 0, T = V = NULL gives zqfp_w4a8_gemm); same kernels, same
 * results bit for bit.  Where the other call would hand float32 partial
 * results through the caller's workspace (K-split of few tiles, K beyond 64
 * k-tiles at M <= 16), this one hands them through an array that is part of
 * the library's device image: ZQFP_STATIC_SCRATCH_BYTES bytes, which every GPU
 * that runs the library holds until the process ends.  The call allocates and
 * frees nothing.
 *
 *   - zqfp_gemm_workspace_bytes(M, K, N) > ZQFP_STATIC_SCRATCH_BYTES is refused
 *     with ZQFP_E_WORKSPACE (text in zqfp_last_hip_error()); nothing is enqueued.
 *   - The array's device address is looked up on the first call on a device
 *     that needs it (hipGetSymbolAddress, with that device current): make that
 *     first call, and the first call of each new shape class (one-time kernel
 *     attributes), outside graph capture.
 *   - All calls on one GPU share the array.  Nothing in it needs to start at
 *     zero (every partial result that is read has been written by the same
 *     call), but calls that overlap in time on one GPU -- different streams, or
 *     graphs replayed concurrently -- race on it: serialise them, or use the
 *     workspace form for all but one.
 */
#define ZQFP_STATIC_SCRATCH_BYTES (32u << 20)
int zqfp_w4a8_gemm_lorc_static(const uint8_t *Xq, const float *sx, int64_t M,
                               int64_t K, const void *packed, int64_t N, int G,
                               const float *T, const void *V, int r,
                               void *Y, int64_t ldy, int out_dtype, int accum,
                               void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ZQFP_H */
