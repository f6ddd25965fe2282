/*
 * svdq_oracle.h -- plain CPU oracle for the W4A4 SVDQuant-style linear layer.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may link or load this.  It shares no code with
 * the GPU library and the GPU library never calls it.
 *
 * What it computes (paper Sec. III-A eq. 3-4, Sec. III-B eq. 5-7, Sec. III-C
 * eq. 8-9 and eq. 11), one step per function, in the paper's order:
 *
 *   x^[m,k]  = x[m,k] / lambda[k]                 (eq. 5, smoothing X D^-1)
 *   a[m,g]   = max_{k in group g} |x^[m,k]|        (reference magnitude of eq. 8,
 *                                                   measured per token per 64-group)
 *   s[m,g]   = (rho * a[m,g]) / q_max, q_max = 7   (eq. 8-9; rho = clipping ratio)
 *   q[m,k]   = clip(round(x^[m,k] / s[m,g]), -8, 7) (eq. 3, zero-point 0)
 *   acc[m,n,g] = sum_{k in g} q[m,k] * qw[n,k]      (4-bit main branch of eq. 7/11)
 *   y[m,n]   = sum_g acc * s[m,g] * sw[g,n]         (dequantisation side of eq. 3)
 *            + sum_j (sum_k x^[m,k] L1[k,j]) L2[j,n] (low-rank branch of eq. 7,
 *                                                   on the UN-quantised x^)
 *            + b[n]
 *
 * Floating point: the chain that decides integer codes (x^, a, s, 1/s, round)
 * is binary32, one correctly rounded IEEE operation per step, because the
 * codes are compared bit for bit.  Everything after the integer accumulators
 * is binary64.
 *
 * All pointers are host pointers.  Layouts are row-major.  bf16 values are
 * passed as uint16_t bit patterns.  Packed int4: byte j of a row holds code
 * 2j in its low nibble and code 2j+1 in its high nibble, two's complement.
 * Every function returns 0 on success and -1 on an invalid argument.
 * nthreads <= 0 means "all hardware threads"; threads split token rows only.
 */
#ifndef SVDQ_ORACLE_H
#define SVDQ_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SVDQ_ORACLE_GROUP = 64, SVDQ_ORACLE_QMAX = 7, SVDQ_ORACLE_QMIN = -8 };

/* bf16 <-> binary32.  Widening is exact; narrowing is round-to-nearest-even. */
float    svdq_oracle_bf16_to_f32(uint16_t v);
uint16_t svdq_oracle_f32_to_bf16(float v);

/* Number of threads the row-parallel functions use for nthreads <= 0. */
int svdq_oracle_hw_threads(void);

/*
 * Eq. 5 then eq. 8-9 then eq. 3: smooth, per-token per-group absmax, clipped
 * scale, round-half-to-even int4 codes, pack.
 *   x          [M, ldx] bf16, first K columns used
 *   inv_lambda [K] binary32, the caller's RN(1/lambda[k])
 *   rho        clipping ratio in (0, 1]
 *   qx         out [M, K/2] packed codes
 *   sx         out [M, K/64] binary32 scales; a group whose scale is not a
 *              normal number (all-zero or denormal group) gets scale 0 and
 *              codes 0
 */
int svdq_oracle_quantize_act(const uint16_t* x, int64_t ldx, const float* inv_lambda,
                             float rho, int64_t M, int K,
                             uint8_t* qx, float* sx, int nthreads);

/*
 * Low-rank down-projection of eq. 7 on the un-quantised smoothed activation:
 * h[m,j] = sum_k x^[m,k] * L1[k,j], x^ the binary32 value of eq. 5, summed in
 * binary64.   L1 [K, r] bf16;   h out [M, r] binary64.
 */
int svdq_oracle_lowrank_down(const uint16_t* x, int64_t ldx, const float* inv_lambda,
                             const uint16_t* L1, int64_t M, int K, int r,
                             double* h, int nthreads);

/*
 * Integer group accumulators of the 4-bit branch:
 * acc[m,n,g] = sum_{k in g} qx[m,k] * qw[n,k]   (int32, exact).
 *   qx [M, K/2], qw [N, K/2] packed codes;  acc out [M, N, K/64].
 */
int svdq_oracle_group_acc(const uint8_t* qx, const uint8_t* qw,
                          int64_t M, int N, int K, int32_t* acc, int nthreads);

/*
 * The quantised layer of eq. 7 / eq. 11 from already-quantised activations:
 * y = sum_g acc*sx*sw + h*L2 + bias.
 *   sw [K/64, N] binary32;  h [M, r] binary64 or NULL (then r must be 0);
 *   L2 [r, N] bf16 or NULL;  bias [N] binary32 or NULL.
 * Outputs (each may be NULL): y64 [M,N] binary64, y32 = (float)y64,
 * ybf16 = RNE_bf16(y32).
 */
int svdq_oracle_linear(const uint8_t* qx, const float* sx,
                       const uint8_t* qw, const float* sw,
                       const double* h, const uint16_t* L2, const float* bias,
                       int64_t M, int N, int K, int r,
                       double* y64, float* y32, uint16_t* ybf16, int nthreads);

/*
 * Timestep -> bin -> clipping ratio (Sec. III-C: the trajectory is cut into
 * bins and inference looks the ratio up).  The paper leaves the bin edges
 * open; the reading here is uniform bins over one expert's own step range:
 * bin = floor((step - step0) * nbins / nsteps_expert).  Returns table[bin],
 * or NaN when step lies outside [step0, step0 + nsteps_expert).
 */
float svdq_oracle_alpha_lookup(const float* table, int nbins, int step, int step0, int nsteps_expert);

/*
 * Objective of the clipping-ratio search of Sec. III-C for one calibration step:
 * sum_{m,n} (Y[m,n] - Y^[m,n])^2 with both outputs given as bf16 [M, N], in binary64.
 */
double svdq_oracle_sq_error(const uint16_t* y_ref, const uint16_t* y, int64_t M, int N);

/* ------------------------------------------------------------------------
 * MXFP4 variant: the 4-bit data format the paper's tables are quoted in
 * (caption of Table I).  Same layer (eq. 5, 7, 8, 11); the uniform integer
 * grid of eq. 3 is replaced by the microscaling FP4 format: blocks of 32
 * values along K share one power-of-two scale (E8M0 byte e, value 2^(e-127)),
 * elements are E2M1 (sign, 2 exponent bits, 1 mantissa bit: magnitudes
 * 0, 0.5, 1, 1.5, 2, 3, 4, 6).  Conversion follows the published MX rule with
 * the clipped threshold of eq. 8 as the block's reference magnitude:
 *
 *   x^     = x * inv_lambda                          (eq. 5, binary32)
 *   a      = max_{k in block} |x^|
 *   alpha  = rho * a                                 (eq. 8, binary32)
 *   E      = floor(log2(alpha));  X = 2^(E - 2)      (2 = exponent of the
 *                                                     largest E2M1 binade)
 *   code   = E2M1 nearest to x^ / X, ties to the even code, |.| > 6 -> 6
 *   sign bit of the code = sign bit of x^
 *
 * A block with alpha < 2^-124 (in particular an all-zero block) is empty:
 * scale byte 0 and all codes 0.  Packed codes: byte j of a row holds code 2j
 * in its low nibble, code 2j+1 in its high nibble.
 */
enum { SVDQ_ORACLE_MX_BLOCK = 32 };

/* Value of a 4-bit E2M1 code (bit 3 = sign). */
float svdq_oracle_e2m1_value(int code);

/*   qx out [M, K/2] packed E2M1 codes;  sx out [M, K/32] E8M0 bytes.  K % 32 == 0. */
int svdq_oracle_quantize_act_mxfp4(const uint16_t* x, int64_t ldx, const float* inv_lambda,
                                   float rho, int64_t M, int K,
                                   uint8_t* qx, uint8_t* sx, int nthreads);

/*
 * y = sum_blocks (sum_{k in block} vx[m,k] vw[n,k]) 2^(sx[m,b]-127) 2^(sw[b,n]-127) + h L2 + bias
 *   qw [N, K/2] packed E2M1 codes, sw [K/32, N] E8M0 bytes; the rest as svdq_oracle_linear.
 */
int svdq_oracle_linear_mxfp4(const uint8_t* qx, const uint8_t* sx,
                             const uint8_t* qw, const uint8_t* sw,
                             const double* h, const uint16_t* L2, const float* bias,
                             int64_t M, int N, int K, int r,
                             double* y64, float* y32, uint16_t* ybf16, int nthreads);

/*
 * GELU (tanh form) of bf16 values, rounded to bf16 (nearest even): the activation between the up- and the
 * down-projection of the feed-forward block, for the quantise pass that applies it on the fly.  The paper does
 * not define it; it is the model's activation.  out[i] = bf16(x[i] / (1 + exp(-2 sqrt(2/pi) (x[i] + 0.044715 x[i]^3)))),
 * evaluated in binary32 by a fixed operation sequence (see the source).  Finite inputs.
 */
int svdq_oracle_gelu_tanh_bf16(const uint16_t* x, int64_t n, uint16_t* out);

#ifdef __cplusplus
}
#endif
#endif
