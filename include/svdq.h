/*
 * svdq.h -- C ABI of the MI355X (gfx950) W4A4 SVDQuant-style linear layer.
 *
 * The layer (paper Sec. III-B eq. 7 and Sec. III-C eq. 11, with the uniform
 * quantiser of Sec. III-A eq. 3-4 and the clipping threshold of eq. 8-9):
 *
 *   x^ = x / lambda                                   smoothing, eq. 5
 *   Q_A(x^) : per token, per 64-group: a = max|x^|, s = rho*a/7,
 *             q = clip(round_half_even(x^/s), -8, 7)   eq. 3, 8, 9
 *   y  = sum_g (sum_{k in g} q[m,k] qw[n,k]) s[m,g] sw[g,n]     4-bit branch
 *      + (x^ L1) L2                                     low-rank branch, eq. 7
 *      + b
 *
 * rho is the clipping ratio the paper looks up per (expert, layer, timestep
 * bin); lambda, L1, L2, the int4 residual codes qw and their scales sw come
 * from offline calibration (smoothing, SVD split, GPTQ) and are inputs here.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, valid on the
 *     current HIP device, 16-byte aligned, not aliasing any output.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it; nothing synchronises; the library keeps no state
 *     besides a cached device-architecture check, and allocates nothing.
 *   - Return value: SVDQ_OK or a negative svdq_status.  Arguments are checked on
 *     the host BEFORE any launch, so an error means nothing was enqueued.
 *     M == 0 is a successful no-op.  NaN/Inf inputs give unspecified outputs.
 *   - Row-major everywhere.  bf16 = upper half of an IEEE binary32.
 *   - Packed int4: within a row, byte j holds code 2j in its low nibble and code
 *     2j+1 in its high nibble, 4-bit two's complement.
 *   - Group size is 64 along K; K % 64 == 0.
 *   - Quantised ACTIVATIONS are stored group-major: codes qx[K/64][M][32 bytes]
 *     (the 32 bytes = the 64 codes of token m in group g, packed as above) and
 *     scales sx[K/64][M].  The quantise kernel produces a group of 32..64 tokens at
 *     a time and the GEMM consumes a group of 128 tokens at a time, so this order
 *     makes both sides' HBM accesses contiguous.  The token-major view is
 *     qx_tm[m][g*32 + b] = qx[g][m][b], sx_tm[m][g] = sx[g][m].
 *   - Weight codes handed to svdq_pack_weight are channel-major: qw[N][K/2].
 */
#ifndef SVDQ_H
#define SVDQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SVDQ_OK = 0,
    SVDQ_ERR_INVALID_ARG = -1,        /* NULL required pointer, negative size, rho outside (0,1], bad enum */
    SVDQ_ERR_UNSUPPORTED_SHAPE = -2,  /* K % 64, N % 128, r not in {0,16,32}, ld too small or misaligned, M > SVDQ_MAX_M */
    SVDQ_ERR_UNSUPPORTED_ARCH = -3,   /* current device is not gfx950 */
    SVDQ_ERR_HIP = -4                 /* a HIP runtime call or launch failed */
} svdq_status;

enum { SVDQ_GROUP = 64, SVDQ_N_TILE = 128, SVDQ_MAX_RANK = 32, SVDQ_MAX_K = 16384 };
/* Largest token count of any kernel entry point (the kernels keep per-lane byte offsets into one group's block of
 * the activation buffers in 32 bits); more rows are rejected with SVDQ_ERR_UNSUPPORTED_SHAPE before any launch. */
#define SVDQ_MAX_M ((int64_t)1 << 26)
enum { SVDQ_OUT_BF16 = 0, SVDQ_OUT_F32 = 1 };

const char* svdq_status_string(int status);

/* ABI version; bumped when a signature or a packed layout changes. */
int svdq_version(void);

/*
 * Host helper for Sec. III-C: map a denoising step to its timestep bin and
 * return that bin's clipping ratio.  `table` is a HOST array of nbins ratios of
 * one expert; the expert covers steps [step0, step0 + nsteps_expert); bins are
 * uniform over that range: bin = floor((step - step0) * nbins / nsteps_expert).
 * Returns NaN for a NULL table, nbins <= 0, nsteps_expert <= 0 or a step outside
 * the range.
 */
float svdq_alpha_lookup(const float* table, int nbins, int step, int step0, int nsteps_expert);

/*
 * One-time, offline: fold the smoothing vector into the low-rank down factor
 * and lay it out for the quantise kernel.  Stores rn(inv_lambda[k] * L1[k,j])
 * split into two bf16 pieces (hi + lo, 16 significant bits) in matrix-core
 * operand order, zero-padded to 32 columns.
 *   L1_bf16     [K, r] bf16, r in {16, 32}
 *   inv_lambda  [K] binary32, the caller's RN(1/lambda[k])        (eq. 5)
 *   l1_packed   out, svdq_packed_l1_bytes(K) bytes
 */
size_t svdq_packed_l1_bytes(int K);
int svdq_pack_lowrank_down(const void* L1_bf16, const float* inv_lambda, int K, int r,
                           void* l1_packed, void* stream);

/*
 * Kernel (a): ONE pass over x that smooths (eq. 5), takes the per-token
 * per-64-group absmax, derives the clipped scale (eq. 8-9), rounds and packs
 * int4 codes (eq. 3) and computes the low-rank down-projection h = x^ L1 on
 * the un-quantised x^ (eq. 7).
 *   x_bf16      [M, ldx] bf16, first K columns used; ldx >= K, ldx % 8 == 0;
 *               K <= SVDQ_MAX_K (the smoothing vector is kept in LDS)
 *   inv_lambda  [K] binary32
 *   rho         clipping ratio in (0, 1]
 *   l1_packed   from svdq_pack_lowrank_down, or NULL to skip h (then r must be 0)
 *   qx          out [K/64, M, 32] group-major packed codes (M*K/2 bytes)
 *   sx          out [K/64, M] group-major binary32 scales; a group whose scale would
 *               not be a normal number gets scale 0 and codes 0
 *   h           out [M, r] binary32 (ignored when l1_packed == NULL)
 * Bit-exact contract: x^ = x * inv_lambda, a = max|x^|, s = (rho*a)/7,
 * q = clip(rne(x^ * (1/s))), each a single IEEE binary32 operation.
 */
int svdq_quantize_act(const void* x_bf16, int64_t ldx, const float* inv_lambda, float rho,
                      const void* l1_packed, int64_t M, int K, int r,
                      uint8_t* qx, float* sx, float* h, void* stream);

/*
 * One-time, offline: canonical residual codes + scales -> kernel-private layout.
 *   qw        [N, K/2] channel-major packed int4 codes of the residual R (eq. 6)
 *   sw        [K/64, N] binary32 scales
 *   w_packed  out, svdq_packed_weight_bytes(N, K) bytes (codes stay 4-bit)
 * N % 128 == 0.
 */
size_t svdq_packed_weight_bytes(int N, int K);
int svdq_pack_weight(const uint8_t* qw, const float* sw, int N, int K, void* w_packed, void* stream);

/*
 * Kernels (b)+(c): int4 x int4 GEMM on the int8 matrix cores with one int32
 * accumulator per 64-group, binary32 dequantisation, then the fused epilogue
 * y = main + h L2 + bias with one rounding to the output type.
 *   qx, sx    as written by svdq_quantize_act
 *   w_packed  from svdq_pack_weight
 *   h         [M, r] binary32 and L2_bf16 [r, N] bf16, or both NULL with r == 0
 *   bias      [N] binary32 or NULL
 *   y         out [M, ldy]; bf16 (round-to-nearest-even) for SVDQ_OUT_BF16,
 *             binary32 for SVDQ_OUT_F32 (the value before the bf16 rounding;
 *             meant for tests); ldy >= N, ldy % 8 == 0
 */
int svdq_linear_w4a4(const uint8_t* qx, const float* sx, const void* w_packed,
                     const float* h, const void* L2_bf16, const float* bias,
                     int64_t M, int N, int K, int r,
                     void* y, int64_t ldy, int out_dtype, void* stream);

/*
 * Un-fused low-rank branch of eq. 7, for callers that run the two halves
 * separately and as a cross-check of the fused kernels.
 *   mode 0:  h[M,r] = (x * inv_lambda) L1     x_bf16 [M,ldx], L1_bf16 [K,r] raw bf16
 *            (uses x_bf16, ldx, inv_lambda, L_bf16 = L1, K, r, h as output)
 *   mode 1:  y[M,ldy] (bf16, in/out) += h L2   L_bf16 = L2 [r,N]
 *            (uses h as input, L_bf16 = L2, N, r, y_bf16, ldy)
 * Unused arguments are ignored.  r in {16, 32}.
 */
int svdq_lowrank(int mode, const void* x_bf16, int64_t ldx, const float* inv_lambda,
                 const void* L_bf16, int64_t M, int K, int N, int r,
                 float* h, void* y_bf16, int64_t ldy, void* stream);

/*
 * Test hook: the int32 group accumulators acc[m,n,g] = sum_{k in g} q[m,k] qw[n,k]
 * exactly as the GEMM kernel's matrix-core path forms them, for rows
 * [m0, m0+mt) of an M-row problem (qx group-major as above):
 * acc out [mt, N, K/64] int32.
 */
int svdq_debug_group_acc(const uint8_t* qx, const void* w_packed, int64_t M, int N, int K,
                         int64_t m0, int mt, int32_t* acc, void* stream);

/*
 * ---- E3M2-container execution of the same int4 layer (eq. 3, 5, 7, 8, 11): identical codes,
 * scales and arithmetic (one exact integer sum per 64-group, binary32 dequantisation), with each
 * 4-bit code q in [-8, 7] stored as the 6-bit floating-point field that equals q (1 sign bit,
 * 3 exponent bits of bias 3, 2 mantissa bits: 0 -> 0, +-1 -> 12, +-2 -> 16, +-3 -> 18, +-4..7 -> 20..23,
 * -8 -> 56; sign in bit 5).  gfx950 has no int4 matrix instruction; its FP6 matrix instruction
 * multiplies these fields exactly, a whole group per instruction, at twice the int8 rate and
 * without unpacking, so this is the fast way to run the layer on this chip.  It costs 6 bits per
 * code in memory instead of 4.  The canonical weight input is the same as for svdq_pack_weight.
 *
 * Activation operand buffer `act`, svdq_act_e3m2_bytes(M, K) bytes, device: for each 64-group g a
 * block of Mp = round_up(M, 4) rows, 56 bytes per row, in three planes
 *     [Mp][2][16 B]   bytes 0..15 of the 24 code bytes of (row, 32-k half); fields ascend from bit 0
 *     [2][Mp][8 B]    bytes 16..23
 *     [Mp][8 B]       token scale s[m,g] as two bf16 pieces, p = hi | lo << 16 (hi + lo ~ s, 16 bits),
 *                     stored twice: {p, p}
 * Rows M..Mp-1 are padding: never written, read only into results that are discarded.
 */
size_t svdq_act_e3m2_bytes(int64_t M, int K);

/* Kernel (a) writing `act`.  Arguments as svdq_quantize_act; sx [K/64][M] binary32 (the exact
 * scales, for inspection) may be NULL.  Codes and scales are bit-identical to svdq_quantize_act. */
int svdq_quantize_act_e3m2(const void* x_bf16, int64_t ldx, const float* inv_lambda, float rho,
                           const void* l1_packed, int64_t M, int K, int r,
                           uint8_t* act, float* sx, float* h, void* stream);

/* act -> nibble codes qx [K/64][M][32 B] in the layout of svdq_quantize_act (format conversion
 * and test hook). */
int svdq_unpack_act_e3m2(const uint8_t* act, int64_t M, int K, uint8_t* qx, void* stream);

/* Offline weight packing for svdq_linear_w4a4_e3m2: qw [N, K/2] nibbles and sw [K/64, N] binary32
 * as for svdq_pack_weight; w_packed out, svdq_packed_weight_e3m2_bytes(N, K) bytes (0 for
 * unsupported shapes), 16-byte aligned. */
size_t svdq_packed_weight_e3m2_bytes(int N, int K);
int svdq_pack_weight_e3m2(const uint8_t* qw, const float* sw, int N, int K, void* w_packed, void* stream);

/* Kernels (b)+(c) on `act`: y as svdq_linear_w4a4 (same shapes, constraints and error behaviour). */
int svdq_linear_w4a4_e3m2(const uint8_t* act, const void* w_packed,
                          const float* h, const void* L2_bf16, const float* bias,
                          int64_t M, int N, int K, int r,
                          void* y, int64_t ldy, int out_dtype, void* stream);

/* Two layers fused across their boundary (the feed-forward block: up-projection, GELU,
 * down-projection; eq. 7 and 11 of the first layer followed by eq. 5, 8, 9, 3 and the low-rank
 * down-projection of eq. 7 of the second).  svdq_linear_w4a4_e3m2 of the first layer, but y never
 * reaches memory: each 64 x 64 tile is rounded to bf16 (the value svdq_linear_w4a4_e3m2 would have
 * stored), passed through GELU if `gelu` != 0 (as svdq_quantize_act_gelu defines it), and quantised
 * for the NEXT layer, whose K axis is this layer's N.  The result is what
 *     svdq_linear_w4a4_e3m2(..., y bf16) ; svdq_quantize_act[_gelu](E3M2, y, next_*)
 * writes: next_act and next_sx bit for bit, next_h up to summation order.
 *   next_inv_lambda [N] binary32, next_rho in (0, 1]: the next layer's smoothing vector and clipping ratio.
 *   next_l1_packed  svdq_pack_lowrank_down(L1' [N, next_r], next_inv_lambda) or NULL (then next_r = 0,
 *                   next_h unused).
 *   next_act  out, svdq_act_e3m2_bytes(M, N) bytes.  next_sx out [N/64][M] binary32 or NULL.
 *   next_h    out [M, next_r] binary32.  Zeroed by the call, then every tile adds its 64-channel share
 *             with floating-point atomic adds: the summation order, hence the last bits, vary from
 *             run to run (the separate quantise kernel sums in a fixed order).
 * "Bit for bit" is against THIS library's two-call sequence.  Against an independent implementation of
 * the chain (first layer, bf16 rounding, GELU, second layer's quantiser) the operands agree exactly
 * wherever the two implementations' bf16 outputs of the first layer agree: y itself is only fixed up to
 * the layer's tolerance, and one bf16 step in any of a token's 64 activations of a group can move that
 * group's scale and codes (on the synthetic feed-forward block 81 % of the (token, group) pairs agree in
 * all 64 activations, 90 % of the 32-blocks for the MXFP4 variant; elsewhere the scale stays within
 * 2^-6 relative and the dequantised values within 1.15 scale steps).
 * Shapes, alignment and error behaviour as svdq_linear_w4a4_e3m2 and svdq_quantize_act_e3m2. */
int svdq_linear_w4a4_e3m2_next(const uint8_t* act, const void* w_packed,
                               const float* h, const void* L2_bf16, const float* bias,
                               int64_t M, int N, int K, int r, int gelu,
                               const float* next_inv_lambda, float next_rho,
                               const void* next_l1_packed, int next_r,
                               uint8_t* next_act, float* next_sx, float* next_h, void* stream);

/* Test hook: the integer group sums as the FP6 matrix-core path forms them; acc out [mt, N, K/64]
 * int32, rows [m0, m0 + mt) as for svdq_debug_group_acc. */
int svdq_debug_group_acc_e3m2(const uint8_t* act, const void* w_packed, int64_t M, int N, int K,
                              int64_t m0, int mt, int32_t* acc, void* stream);

/*
 * ---- Kernel (a) with the feed-forward activation fused.  In the DiT's feed-forward block the down-projection
 * (the module the paper calls ffn.2, one of the two most quantisation-sensitive ones, Sec. IV) reads
 * gelu(up-projection output).  This call takes the up-projection's bf16 output x itself and applies
 * GELU (tanh form: gelu(v) = v / (1 + exp(-2 sqrt(2/pi) (v + 0.044715 v^3)))) to every element on the fly, rounded
 * to bf16 as a separate element-wise kernel would have stored it; everything after that is the call selected by
 * `format` (same arguments, layouts and error behaviour; `codes` / `scales` are that call's qx / sx, act / sx or
 * qx / sx_e8m0).  The write and the read of the activated tensor disappear.  Finite inputs.
 */
enum { SVDQ_FMT_INT4 = 0, SVDQ_FMT_INT4_E3M2 = 1, SVDQ_FMT_MXFP4 = 2 };
int svdq_quantize_act_gelu(int format, const void* x_bf16, int64_t ldx, const float* inv_lambda, float rho,
                           const void* l1_packed, int64_t M, int K, int r,
                           uint8_t* codes, void* scales, float* h, void* stream);

/* Test hook: out_bf16[i] = bf16(gelu(x_bf16[i])) through the device function the fused pass uses; n elements. */
int svdq_debug_gelu(const void* x_bf16, int64_t n, void* out_bf16, void* stream);

/*
 * ---- GPTQ on the residual (Sec. III-B: the residual branch is quantised with GPTQ instead of round-to-nearest).
 * Offline calibration.  Column-sequential form of the algorithm in binary64: weights are visited in the order
 * k = 0..K-1; a visited weight is rounded to the int4 grid of its (channel, 64-group) scale (absmax of the group's
 * current weights when its first weight is visited, / 7 in binary32; code = clip(rint(binary32(w) / scale), -8, 7))
 * and its rounding error is spread over the not yet visited weights of the same channel in proportion to row k of
 * the inverse of H + damp * mean(diag H) * I, from which index k is then eliminated.  An input channel with
 * H[k,k] == 0 gets H[k,k] = 1 and zero weights.  With H = I and damp = 0 the result is round-to-nearest.
 *
 *   svdq_gptq_hessian:  H [K, K] binary64, device, += X^T X^ with X^ = x * inv_lambda (eq. 5) over the M rows of
 *                       x_bf16 [M, ldx]; the caller zeroes H before the first calibration batch.
 *   svdq_gptq_quantize: R [K, N] binary32 residual (row k = input channel), H as above (not modified),
 *                       workspace of svdq_gptq_workspace_bytes(N, K) bytes (16-byte aligned, device);
 *                       out qw [N, K/2] packed codes and sw [K/64, N] binary32 scales: the canonical weight form
 *                       that svdq_pack_weight and svdq_pack_weight_e3m2 take.  K % 64 == 0.  The pivots are taken
 *                       in panels of 64 (same rounded operations per element in the same order, so the result
 *                       does not depend on it); enqueues about 5 * K small kernels on `stream`.
 */
size_t svdq_gptq_workspace_bytes(int N, int K);
int svdq_gptq_hessian(const void* x_bf16, int64_t ldx, const float* inv_lambda, int64_t M, int K, double* H, void* stream);
int svdq_gptq_quantize(const float* R, const double* H, double damp, int N, int K, void* workspace,
                       uint8_t* qw, float* sw, void* stream);

/*
 * ---- MXFP4 variant: the 4-bit data format of the paper's Table I on the block-scaled
 * matrix instruction of gfx950.  Same layer (eq. 5, 7, 8, 11) and same calling conventions;
 * the integer grid of eq. 3 is replaced by microscaling FP4: blocks of 32 values along K share
 * one E8M0 scale byte e (value 2^(e-127)), elements are E2M1 codes (bit 3 sign, magnitudes
 * 0, 0.5, 1, 1.5, 2, 3, 4, 6).  Conversion: a = max|x^| over the block, alpha = rho * a (eq. 8),
 * shared exponent floor(log2 alpha) - 2, element = E2M1 nearest to x^ / 2^shared (ties to the even
 * code, saturating at 6, sign bit of x^); a block with alpha < 2^-124 gets byte 0 and codes 0.
 *
 *   qx   [K/64][M][32 B]: packed E2M1 codes, same container as the int4 path (the 32 bytes of a
 *        token and 64-group are two MX blocks: bytes 0..15 and 16..31)
 *   sx   [ceil(K/128)][M][2][2] bytes: for token m and pair of 64-groups (2s, 2s+1) the byte
 *        [h][j] scales MX block 2 (2s + j) + h, i.e. k in [64 (2s + j) + 32 h, +32); bytes of a
 *        group past K are 0
 *   weights at the boundary: qw [N, K/2] packed E2M1 codes, sw [K/32, N] E8M0 bytes
 * The matrix core applies the block scales and accumulates in binary32 over all of K; there is
 * no integer accumulator and no per-group step.  Codes and scale bytes are bit-exact against the
 * definition; y is compared within the layer's tolerance.
 */
int svdq_quantize_act_mxfp4(const void* x_bf16, int64_t ldx, const float* inv_lambda, float rho,
                            const void* l1_packed, int64_t M, int K, int r,
                            uint8_t* qx, uint8_t* sx_e8m0, float* h, void* stream);
size_t svdq_packed_weight_mxfp4_bytes(int N, int K);
int svdq_pack_weight_mxfp4(const uint8_t* qw, const uint8_t* sw_e8m0, int N, int K, void* w_packed, void* stream);
int svdq_linear_mxfp4(const uint8_t* qx, const uint8_t* sx_e8m0, const void* w_packed,
                      const float* h, const void* L2_bf16, const float* bias,
                      int64_t M, int N, int K, int r,
                      void* y, int64_t ldy, int out_dtype, void* stream);

/* svdq_linear_w4a4_e3m2_next for the MXFP4 layer: svdq_linear_mxfp4 whose epilogue rounds each tile to
 * bf16, applies GELU if `gelu` != 0 and writes what svdq_quantize_act_mxfp4 (svdq_quantize_act_gelu
 * with SVDQ_FMT_MXFP4) of that output would write for the next layer (K' = N): next_qx
 * [N/64][M][32 B] and next_sx_e8m0 [N/128][M][2][2] bit for bit, next_h [M, next_r] (zeroed by the
 * call, then accumulated with atomic adds: last bits vary with summation order).  next_* as for
 * svdq_linear_w4a4_e3m2_next; shapes and errors as svdq_linear_mxfp4. */
int svdq_linear_mxfp4_next(const uint8_t* qx, const uint8_t* sx_e8m0, const void* w_packed,
                           const float* h, const void* L2_bf16, const float* bias,
                           int64_t M, int N, int K, int r, int gelu,
                           const float* next_inv_lambda, float next_rho,
                           const void* next_l1_packed, int next_r,
                           uint8_t* next_qx, uint8_t* next_sx_e8m0, float* next_h, void* stream);

/*
 * Offline calibration, Sec. III-C: the clipping ratio of a (layer, timestep bin) is the candidate that
 * minimises the expected squared reconstruction error || Y - Y^(rho) ||^2 of the quantised layer over
 * the calibration steps of the bin.  The search runs the hot path (svdq_quantize_act* +
 * svdq_linear_*) once per candidate and step and needs one more kernel, this reduction:
 *   out[0] = sum_{m < M, n < N} (y_ref[m,n] - y[m,n])^2       (device binary64, deterministic)
 *   y_ref_bf16 [M, ld_ref], y_bf16 [M, ldy] bf16;  N % 8 == 0, leading dimensions % 8 == 0
 *   workspace  caller's device buffer of svdq_sq_error_workspace_bytes() bytes (partial sums)
 * M == 0 gives 0.
 *   svdq_sq_error_add   the same sum ADDED to acc[0] (device binary64): the expectation over the calibration steps
 *                       of a bin, accumulated on the device in stream order (deterministic).  The caller zeroes
 *                       the table of accumulators [nbins][ncandidates] before the first step and passes the
 *                       entry of (bin, candidate).
 *   svdq_argmin_rows    idx[b] = index of the smallest entry of table[b][0..ncols) (the first one on a tie): the
 *                       arg-min over the candidate set, per bin.  table, idx on the device; ncols >= 1.
 */
size_t svdq_sq_error_workspace_bytes(void);
int svdq_sq_error(const void* y_ref_bf16, int64_t ld_ref, const void* y_bf16, int64_t ldy,
                  int64_t M, int N, void* workspace, double* out, void* stream);
int svdq_sq_error_add(const void* y_ref_bf16, int64_t ld_ref, const void* y_bf16, int64_t ldy,
                      int64_t M, int N, void* workspace, double* acc, void* stream);
int svdq_argmin_rows(const double* table, int nrows, int ncols, int32_t* idx, void* stream);

/*
 * svdq_sq_error for callers that cannot allocate device memory or carry a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments without `workspace`, same result bit for
 * bit.  The 1024 binary64 partial sums live in a static device array of the library (8 KB per GPU, held until the
 * process ends), whose address is looked up once per device; the call allocates nothing.  The array does not grow
 * with the input; inputs of more than SVDQ_SQ_ERROR_STATIC_MAX_ELEMENTS = 2^36 elements per tensor are rejected
 * with SVDQ_ERR_UNSUPPORTED_SHAPE.  All calls on one GPU share the array: calls that overlap on one GPU (two
 * streams, two threads) race and give wrong sums; calls on one stream are safe, and nothing needs clearing between
 * them (every partial sum is rewritten by every call).
 */
#define SVDQ_SQ_ERROR_STATIC_MAX_ELEMENTS ((int64_t)1 << 36)
int svdq_sq_error_static(const void* y_ref_bf16, int64_t ld_ref, const void* y_bf16, int64_t ldy,
                         int64_t M, int N, double* out, void* stream);

/*
 * Test hook: the scalar part of kernel (a)'s chain, eq. 8-9, evaluated by the
 * kernel's own device functions on n given group magnitudes a[i] >= 0:
 *   s[i]   = (rho * a[i]) / 7, or 0 when that is not a normal number
 *   inv[i] = 1 / s[i], or 0 when s[i] == 0
 * each required to equal the single IEEE binary32 operation.  n <= 2^31.
 */
int svdq_debug_scale_chain(const float* a, float rho, int64_t n, float* s, float* inv, void* stream);

#ifdef __cplusplus
}
#endif
#endif
