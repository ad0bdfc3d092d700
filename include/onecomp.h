/*
 * onecomp.h -- C ABI of the MI355X (gfx950) layer-wise Hessian-aware quantizer.
 *
 * One linear layer is quantized in three calls that follow the paper's problem
 * statement for layer-wise PTQ (Sec. 4.3):
 *
 *   1. onecomp_hessian_accumulate  H += 2 X^T X          (Gram matrix, Sec. 2.5 / 4.3)
 *   2. onecomp_hessian_factor      U^T U = (H + lambda I)^-1, lambda = damp * mean(diag H)
 *                                                         (Sec. 4.3.1, text after Eq. (qep));
 *                                  optional activation ordering (Sec. 4.3, "actorder")
 *   3. onecomp_quantize_layer      column-by-column sweep: each column is rounded to the
 *                                  per-group asymmetric min-max grid (Eq. (1), (2), (4))
 *                                  and its residual is propagated through U to the
 *                                  columns not yet quantized (Sec. 4.3)
 *
 * Variants: onecomp_quantize_layer_grid (symmetric grid of Eq. (3)); onecomp_hessian_factor_form and
 * onecomp_quantize_layer_form (the same sweep on one Cholesky factor, without the triangular inverse);
 * onecomp_crossgram_accumulate and onecomp_qep_target (error propagation, Sec. 4.3.1);
 * onecomp_rtn_sensitivity (error metric of the bit allocation, Sec. 4.1).
 *
 * Storage convention: W is d_out x d_in row-major (rows = output channels); this
 * is the transpose of the paper's N x M weight matrix.  "Column j" is input
 * channel j; a group is `group_size` consecutive input channels of one row.
 *
 * Common rules
 *   - Every data pointer is caller-owned DEVICE memory on the current HIP device.
 *     The library never allocates or frees, and keeps no state between calls beyond cached device properties.
 *   - All work is enqueued asynchronously on `hip_stream` (a hipStream_t passed as
 *     void*; NULL = the null stream).  Device scalars (`loss`, `info`) are valid
 *     once the stream has been synchronized.
 *   - Host-checkable problems are reported through the return code and nothing is
 *     launched; a numerical failure (matrix not positive definite) is reported
 *     through the device scalar `info`.
 *   - The binary contains gfx950 code only.
 *   - Profiling: with ONECOMP_ROCTX=1 in the environment at the first call, every launching entry point pushes a
 *     ROCTx range named after itself (the ROCTx library is looked up at run time; `rocprofv3 --marker-trace` shows
 *     the ranges).  A range covers the argument checks and the enqueueing of the launches, not the kernels' run time.
 */
#ifndef ONECOMP_H
#define ONECOMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ONECOMP_OK = 0,
    ONECOMP_ERR_INVALID_ARG = 1,   /* NULL pointer, non-positive size, bad stride, bad divisibility */
    ONECOMP_ERR_UNSUPPORTED = 2,   /* dtype / bits / group / block outside the supported set */
    ONECOMP_ERR_NOT_POSDEF = 3,    /* reserved for callers that translate `info` */
    ONECOMP_ERR_WORKSPACE = 4,     /* workspace NULL or smaller than the matching *_workspace_bytes() */
    ONECOMP_ERR_HIP = 5            /* a HIP runtime call failed (launch error etc.) */
} onecomp_status;

typedef enum {
    ONECOMP_F32 = 0,
    ONECOMP_BF16 = 1
} onecomp_dtype;

/* Grid of the column sweep: per-group asymmetric min-max grid of Eq. (2), or the symmetric grid of Eq. (3).
 * The _MSE variants add the scale search of Sec. 4.3 (the sweep's "mse" option): when a group's parameters are
 * fixed, its range [lo, hi] is shrunk to p_i [lo, hi], p_i = 1 - i / 100 for i = 0 .. 79, (s, z) follow from the
 * shrunk range by the grid's own rule, and the candidate with the least sum over the group of (w - s (q - z))^2
 * (q rounded and clamped as in the sweep) is kept, the lowest i on equal sums; i = 0 is the plain grid.  The
 * candidates are compared in fp32 on the compensated values; the winner's scale is then taken in fp64. */
typedef enum {
    ONECOMP_GRID_MINMAX = 0,
    ONECOMP_GRID_SYMMETRIC = 1,
    ONECOMP_GRID_MINMAX_MSE = 2,
    ONECOMP_GRID_SYMMETRIC_MSE = 3
} onecomp_grid;

/* What the factor call hands to the sweep.
 *   ONECOMP_FACTOR_INVERSE  the inverse factor U of Sec. 4.3.1, U^T U = (H + lambda I)^-1 (one Cholesky plus one
 *                           triangular inverse, 2 d_in^3 / 3 flops).
 *   ONECOMP_FACTOR_BLOCK    one Cholesky only (d_in^3 / 3 flops).  With R = U^-1 (upper, R R^T = H + lambda I) the
 *                           matrix written is F = U on the 128 x 128 diagonal blocks and
 *                           F_jk = -U_jj R_jk / R_kk where j and k lie in different blocks.  The sweep's errors
 *                           satisfy e = (w - w^) R (w the original weights), so the compensated values on entering a
 *                           block are  w_b + c (R_bb)^-1  with  c = sum over finished columns i of (w_i - w^_i) R_ib:
 *                           the same codes, scales, zeros and loss as with U, up to rounding. */
typedef enum {
    ONECOMP_FACTOR_INVERSE = 0,
    ONECOMP_FACTOR_BLOCK = 1
} onecomp_factor_form;

/*
 * H += 2 * X^T X  over the n_tokens rows of X (Gram matrix of Sec. 2.5 / Sec. 4.3; the
 * factor 2 makes it the Hessian of ||X (W^ - W)||^2, cf. Sec. 2.4).
 *
 *   X        [n_tokens x d_in], row-major, row stride `ldx` elements (ldx >= d_in), dtype x_dtype.
 *            Read only.  Must be 16-byte aligned with ldx * sizeof(elem) a multiple of 16.
 *   H        [d_in x d_in] fp32, row-major, full symmetric storage; read-modify-write.
 *            The caller zero-fills it before the first chunk; calls are additive, so
 *            any split of the token axis into chunks gives the same sum up to fp32
 *            rounding order.  The result is bit-wise symmetric and, for a fixed
 *            chunking, bit-wise reproducible (no floating-point atomics).
 *   d_in     must be a multiple of 16.  n_tokens == 0 is a no-op returning ONECOMP_OK.
 * Products of bf16 inputs are exact; accumulation is fp32.  fp32 inputs are multiplied in fp32.
 */
onecomp_status onecomp_hessian_accumulate(const void* X, onecomp_dtype x_dtype,
                                          int64_t n_tokens, int64_t d_in, int64_t ldx,
                                          float* H, void* hip_stream);

/*
 * onecomp_hessian_accumulate with an optional scratch buffer (onecomp_hessian_accumulate is this call with
 * workspace = NULL).  The kernel computes H in tiles (256 x 256 without a workspace), one per compute unit at a
 * time; when the number of tiles does not fill the last round of compute units (or there are fewer tiles than
 * units), a workspace lets it cut tiles into 2 to 16 pieces along the token axis, park the partial sums there and
 * add them in a fixed order: same result up to fp32 rounding order, still bit-wise symmetric and reproducible, and
 * faster for such widths (d_in 4096, 262144 tokens: 6.0 -> 3.9 ms; d_in 8192, 131072 tokens: 9.1 -> 8.0 ms).  With
 * a workspace the call may also take 384 x 256 tiles (fewer cache and LDS bytes per flop; their last round always
 * needs the workspace): d_in 14336, 262144 tokens: 46-49 -> 43-46 ms.  Without a workspace only the mirror positions
 * of H can hold a second partial sum, which covers a short last round of wide matrices.  The tile shape is chosen by
 * estimated cost; ONECOMP_GRAM_SHAPE=wide|big|mid in the environment forces 384 x 256, 256 x 256 or 128 x 256 tiles
 * for d_in >= 1024 (testing and tuning; onecomp_accumulate_describe reports the choice).
 * A call of fewer than 49152 tokens is one launch, a longer one a launch per round of tiles (one tile per compute unit);
 * ONECOMP_GRAM_ROUND_LAUNCHES=0|1 forces either (tuning).  None of these choices changes what the call computes.
 *   workspace        device scratch or NULL, 256-byte aligned; any size is accepted, the kernel uses what fits
 *                    (onecomp_accumulate_workspace_bytes(x_dtype, d_in) is what it can use at most; 0 for fp32
 *                    inputs and for widths that gain nothing).  Contents on entry and exit are meaningless.
 * Other arguments and errors as for onecomp_hessian_accumulate; a misaligned workspace is ONECOMP_ERR_WORKSPACE.
 */
onecomp_status onecomp_hessian_accumulate_ws(const void* X, onecomp_dtype x_dtype,
                                             int64_t n_tokens, int64_t d_in, int64_t ldx,
                                             float* H, void* workspace, size_t workspace_bytes, void* hip_stream);
size_t onecomp_accumulate_workspace_bytes(onecomp_dtype x_dtype, int64_t d_in);
/*
 * Profiling aid: how onecomp_hessian_accumulate_ws would run a call of this size on the current device (Sec. 2.5 /
 * 4.3, the same Gram accumulation; nothing is launched).  out3 is a HOST pointer to three int32: rows and columns of
 * the output tile one workgroup of the call's main kernel owns, and the number of launches of that kernel in the
 * call (a wide layer is launched one round of tiles at a time).  workspace_bytes: size of the workspace the call
 * would be given (0: none).  Errors as for the call itself.
 */
onecomp_status onecomp_accumulate_describe(onecomp_dtype x_dtype, int64_t n_tokens, int64_t d_in, int64_t ldx,
                                           size_t workspace_bytes, int32_t* out3);

/*
 * Damping, optional activation ordering, and the Cholesky-based inverse factor
 * (Sec. 4.3.1: lambda = damp * mean(diag H), Cholesky of H + lambda I; Sec. 4.3 "actorder").
 *
 *   H         [d_in x d_in] fp32 symmetric, read only (only diagonal and one triangle need be valid;
 *             the upper triangle is read).
 *   damp      eta >= 0.  A zero diagonal entry of H (dead input channel) is replaced by 1
 *             before lambda is computed.
 *   act_order 0: natural column order.  non-zero: perm = indices of diag(H) in decreasing
 *             order (equal keys: lower index first) and the matrix factored is
 *             (H + lambda I)[perm][:, perm].
 *   perm_out  int32[d_in]; the order used (identity when act_order == 0).  May be NULL when
 *             act_order == 0.
 *   U         [d_in x d_in] fp32 row-major, out: upper triangular with positive diagonal and
 *             U^T U = (H_d)^-1 for the (permuted) damped matrix H_d; the strict lower
 *             triangle is written as zeros.  Computed in fp64, rounded once to fp32.
 *   info      device int32, out: 0 on success, k > 0 if the matrix is not positive definite
 *             (k is in 1..d_in and names the pivot, counted from the END of the
 *             permuted order, at which the factorization first met a non-positive value);
 *             U is then unspecified but every kernel still terminates normally.
 *   workspace device scratch of at least onecomp_factor_workspace_bytes(d_in) bytes, 256-byte aligned.
 *   d_in      must be a multiple of 16.
 */
onecomp_status onecomp_hessian_factor(const float* H, int64_t d_in, float damp, int act_order,
                                      int32_t* perm_out, float* U, int32_t* info,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * onecomp_hessian_factor with the form of the result chosen by the caller (onecomp_hessian_factor is this call
 * with ONECOMP_FACTOR_INVERSE).  ONECOMP_FACTOR_BLOCK writes the matrix F described at onecomp_factor_form into
 * `F_out` (same shape and layout as U, strict lower triangle zero); it needs d_in % 128 == 0 and is meant for
 * onecomp_quantize_layer_form only (onecomp_qep_target needs the inverse form).  Same workspace, same `info`.
 * An unknown form, or a d_in the form does not support, is ONECOMP_ERR_UNSUPPORTED.
 */
onecomp_status onecomp_hessian_factor_form(const float* H, int64_t d_in, float damp, int act_order,
                                           onecomp_factor_form form, int32_t* perm_out, float* F_out, int32_t* info,
                                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The column sweep (Sec. 4.3) on the per-group asymmetric grid (Eq. (1), (2), (4)).
 * For every output row independently, for columns j in sweep order:
 *   at the first column of a group: s = (max - min) / (2^bits - 1) over the CURRENT
 *     (already compensated) values of the group (s = 1 if max == min),
 *     z = clamp(rne(-min / s), 0, 2^bits - 1)
 *   q_j = clamp(rne(w_j / s) + z, 0, 2^bits - 1),  w^_j = s (q_j - z)
 *   e_j = (w_j - w^_j) / U_jj,   w_k -= e_j U_jk  for all later columns k
 * rne = round half to even.  Arithmetic: the value that is rounded has to match exact arithmetic to a small
 * fraction of a grid step over thousands of columns (one wrong rounding at a near-tie changes the rest of its row),
 * so the compensated weight is never held in fp32: the original weight (exact) and the feedback sum
 * c_j = -sum_{i<j} e_i U_ij (a fraction of a grid step) are kept apart, c in fp32; inside a 32-column inner block
 * w = w0 + c, the scale (fp64 division; returned rounded to fp32), the decision rne(w / s) (the correctly rounded
 * quotient, from the reciprocal and one correction by the FMA residual) and the feedback run in fp64.  Feedback that crosses an inner block is accumulated from zero (fp32 MFMA inside a 128-column block;
 * across blocks as (w_j - w^_j) * (U_jk / U_jj) with both factors rounded to 22 significant bits: two fp16 halves
 * after an exact power-of-two scaling taken from max |W| and max |U_jk / U_jj|, fp32 accumulation) and added to c
 * once.  A residual above 8 max|W|, which no sweep of a sane layer produces, would saturate on its way into the fp16
 * halves: `loss` then comes back as +infinity.
 *
 *   W          [d_out x d_in] row-major (dense, stride d_in), dtype w_dtype, ORIGINAL column order. Read only.
 *   U          [d_in x d_in] fp32, as written by onecomp_hessian_factor. Read only.
 *   perm       NULL (natural order) or the int32[d_in] order returned by the factor call;
 *              sweep position p handles original column perm[p].
 *   bits       2, 3, 4 or 8.
 *   group_size G: multiple of 16, divides d_in; groups are contiguous in SWEEP order.
 *   block_size B: lazy-batch width; 128 (the only supported value); d_in % B == 0 and either
 *              G divides B or B divides G.
 *   Q_codes    uint8 [d_out x d_in], one code per byte, ORIGINAL column order.  Out.
 *   scales     fp32 [d_out x d_in/G], indexed by group number in sweep order.  Out.
 *   zeros      fp32 [d_out x d_in/G], integer valued.  Out.
 *   W_hat      fp32 [d_out x d_in] = scales * (Q_codes - zeros) bit for bit, ORIGINAL column order;
 *              may be NULL.  Out.
 *   loss       device fp32 scalar, out: sum of e^2 over the layer, which equals
 *              tr((W - W^) H_d (W - W^)^T) for the damped (permuted) matrix behind U (Eq. (layerwise)).
 *              Reduced in a fixed order (bit-wise reproducible).
 *   workspace  device scratch, >= onecomp_quantize_workspace_bytes(d_out, d_in, block_size), 256-byte aligned
 *              (about 9 d_out d_in + 4 d_in^2 bytes: the fp32 feedback sums, an fp32 copy of W gathered into sweep
 *              order, codes staged in sweep order, two fp16 halves of the scaled U).
 *   d_in       at most 65535, d_out at most 2^24.
 *   W, U and W_hat must be 16-byte aligned, Q_codes 4-byte aligned (ONECOMP_ERR_INVALID_ARG otherwise).
 */
onecomp_status onecomp_quantize_layer(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                      const float* U, const int32_t* perm,
                                      int bits, int group_size, int block_size,
                                      uint8_t* Q_codes, float* scales, float* zeros,
                                      float* W_hat, float* loss,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * onecomp_quantize_layer with the grid chosen by the caller (onecomp_quantize_layer is this call with
 * ONECOMP_GRID_MINMAX).  ONECOMP_GRID_SYMMETRIC is the symmetric grid of Sec. 2.3.2, Eq. (3): at the first column
 * of a group  s = max(|min|, |max|) / (2^(bits-1) - 1)  over the current values of the group (s = 1 if all are
 * zero), signed codes q in {-(2^(bits-1) - 1), ..., 2^(bits-1) - 1}, w^ = s q.  Outputs keep the format of the
 * min-max grid: Q_codes holds the unsigned code q + (2^(bits-1) - 1), zeros holds the constant 2^(bits-1) - 1, so
 * W_hat = scales * (Q_codes - zeros) bit for bit; the highest unsigned code 2^bits - 1 is never produced.
 * Everything else (arguments, arithmetic, workspace, errors) as for onecomp_quantize_layer; an unknown grid is
 * ONECOMP_ERR_UNSUPPORTED.
 */
onecomp_status onecomp_quantize_layer_grid(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                           const float* U, const int32_t* perm,
                                           int bits, int group_size, int block_size, onecomp_grid grid,
                                           uint8_t* Q_codes, float* scales, float* zeros,
                                           float* W_hat, float* loss,
                                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * onecomp_quantize_layer_grid for a factor in either form (onecomp_quantize_layer_grid is this call with
 * ONECOMP_FACTOR_INVERSE).  With ONECOMP_FACTOR_BLOCK, `F` is the output of onecomp_hessian_factor_form in that
 * form: inside a 128-column block the steps are those of onecomp_quantize_layer (F holds U there); between blocks
 * the workspace accumulates c_k = sum_i (w_i - w^_i) R_ik / R_kk over the finished columns i of earlier blocks
 * (deviations from the ORIGINAL weights; 22-bit operands, fp32 sum, as described at onecomp_quantize_layer) and a
 * block starts from  w_b + c (U_bb rows divided by their diagonal), the product in fp32 from zero, the sum in fp64.  Outputs and their meaning are
 * unchanged; results agree with the inverse form up to rounding.  ONECOMP_FACTOR_BLOCK needs group_size <= 128 or
 * group_size == d_in (one group per row, whose grid comes from the original weights); other wide groups take their
 * grid from columns of later blocks, whose compensated values this form does not hold: ONECOMP_ERR_UNSUPPORTED.
 */
onecomp_status onecomp_quantize_layer_form(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                           const float* F, onecomp_factor_form form, const int32_t* perm,
                                           int bits, int group_size, int block_size, onecomp_grid grid,
                                           uint8_t* Q_codes, float* scales, float* zeros,
                                           float* W_hat, float* loss,
                                           void* workspace, size_t workspace_bytes, void* hip_stream);

/* Scratch sizes for the factor and sweep calls above (0 if the arguments are invalid). */
size_t onecomp_factor_workspace_bytes(int64_t d_in);
size_t onecomp_quantize_workspace_bytes(int64_t d_out, int64_t d_in, int block_size);

/*
 * Error propagation (QEP, Sec. 4.3.1): cross-Gram of the activations X_hat that reach this layer in the partly
 * quantized model and the activations X of the full-precision model,
 *     G += 2 X_hat^T X        (the factor 2 of onecomp_hessian_accumulate),
 * so that with H = 2 X_hat^T X_hat (onecomp_hessian_accumulate on X_hat) the error-propagation matrix of the
 * paper is C = X_hat^T (X - X_hat) = (G - H) / 2.  The caller zero-fills G before the first chunk.
 *   X_hat, X  [n_tokens x d_in] row-major, row strides ldxh / ldx elements, ONECOMP_BF16 only; read only.
 *             bf16 products are exact in fp32; accumulation is fp32.
 *   G         [d_in x d_in] fp32, row-major, not symmetric: G[i][k] pairs channel i of X_hat with channel k of X.
 *   d_in      multiple of 16; a step of 16 token rows must be addressable with 32-bit byte offsets
 *             (row stride below 2^25 elements), else ONECOMP_ERR_UNSUPPORTED.
 */
onecomp_status onecomp_crossgram_accumulate(const void* X_hat, const void* X, onecomp_dtype x_dtype,
                                            int64_t n_tokens, int64_t d_in, int64_t ldxh, int64_t ldx,
                                            float* G, void* hip_stream);

/*
 * Corrected quantization target of Eq. (qep), Sec. 4.3.1 (paper: W* = (I + alpha (H^ + lambda I)^-1 C) W for
 * the d_in x d_out weight).  In this library's d_out x d_in storage and scaling:
 *     W* = W + alpha W (G - H)^T (H + lambda I)^-1,   lambda = damp * mean(diag H),
 * where the regularized inverse is taken from the factor of onecomp_hessian_factor(H, damp, ...):
 * (H + lambda I)^-1 = P U^T U P^T with P the column order `perm` of that call.  W* is then passed to
 * onecomp_quantize_layer (as ONECOMP_F32) together with the same U and perm.
 *   W        [d_out x d_in] row-major, dtype w_dtype, original column order; read only.
 *   G, H     [d_in x d_in] fp32 as accumulated by the two accumulate calls on the same tokens; read only.
 *   U, perm  outputs of onecomp_hessian_factor for this H (perm NULL = natural order); read only.
 *   alpha    propagation strength in [0, 1].
 *   W_star   [d_out x d_in] fp32, original column order, out; must not alias W.
 *   workspace device scratch, >= onecomp_qep_workspace_bytes(d_out, d_in), 256-byte aligned.
 * Arithmetic: three products accumulated in fp32 from operands split into fp16 hi + lo halves (22 significant bits
 * each; every factor in the scaling of the correlation matrix, H_kj / sqrt(H_kk H_jj), so that fp16's range
 * suffices).  G - H cancels the leading digits of two Gram matrices, so the correction W* - W carries a relative
 * error of about 1e-6 |X| / |X - X_hat|.
 */
onecomp_status onecomp_qep_target(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                  const float* G, const float* H, const float* U, const int32_t* perm,
                                  float alpha, float* W_star,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* Scratch size for onecomp_qep_target (0 if the arguments are invalid): about 8 d_in^2 + 16 d_out d_in bytes. */
size_t onecomp_qep_workspace_bytes(int64_t d_out, int64_t d_in);

/*
 * Activation-aware sensitivity of the layer under one candidate configuration (bit-width allocation, Sec. 4.1:
 * err(l, c) ~ 1/2 tr(B dW A dW^T) with only the diagonals of A and B, dW = W^ - W from a fast round-to-nearest
 * proxy).  In this library's d_out x d_in storage:
 *     err = 1/2 sum_r sum_c b_r a_c (W^_rc - W_rc)^2,
 * where W^ rounds every group of group_size consecutive input channels of a row to its own grid (min-max grid of
 * Eq. (2) or symmetric grid of Eq. (3), no error feedback).  With a = b = 1 this is half the squared Frobenius
 * norm of the perturbation.
 *   W        [d_out x d_in] row-major, dtype w_dtype, 16-byte aligned; read only.
 *   a_diag   fp32 [d_in], 16-byte aligned: diagonal of the input Gram matrix A (e.g. diag H of onecomp_hessian_accumulate, which
 *            carries that call's factor 2); read only.
 *   b_diag   fp32 [d_out]: diagonal of the output curvature B, or NULL for all ones; read only.
 *   bits, group_size, grid: the candidate; group_size a multiple of 16 that divides d_in (no block restriction).
 *   err      device fp32 scalar, out.  fp32 arithmetic, partial sums combined in a fixed order (reproducible).
 *   workspace device scratch, >= onecomp_sensitivity_workspace_bytes(), 256-byte aligned.
 */
onecomp_status onecomp_rtn_sensitivity(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                       const float* a_diag, const float* b_diag,
                                       int bits, int group_size, onecomp_grid grid, float* err,
                                       void* workspace, size_t workspace_bytes, void* hip_stream);
size_t onecomp_sensitivity_workspace_bytes(void);

/*
 * onecomp_rtn_sensitivity for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight planning loops over many (bits, group size) candidates, harnesses that forbid hipMalloc.  Same
 * arguments, kernels, result (bit for bit) and errors as onecomp_rtn_sensitivity, without the workspace: the
 * per-workgroup partial sums (2048 floats, 8 KB) go to a fixed array in the library's device data segment, one per
 * GPU, held until the process ends.  The call allocates and frees nothing and never synchronizes; its first use on
 * a device looks the array's address up (no allocation, no stream operation).
 *   - Limits: d_out and d_in up to 2^24 as for onecomp_rtn_sensitivity (the scratch is sized for the largest launch,
 *     so no smaller limit applies); beyond them ONECOMP_ERR_INVALID_ARG, nothing is launched.
 *   - Every call on a GPU uses that GPU's one array, which keeps the last call's contents; each call overwrites the
 *     part it reads, so nothing has to be cleared.  Calls that overlap on one GPU (different streams or host
 *     threads) race on it: serialize them, or use onecomp_rtn_sensitivity with separate workspaces.
 */
onecomp_status onecomp_rtn_sensitivity_static(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                              const float* a_diag, const float* b_diag,
                                              int bits, int group_size, onecomp_grid grid, float* err,
                                              void* hip_stream);

/*
 * JointQ refinement of a quantized layer (Sec. 4.3.2, Eq. (jointq); with lam > 0 Eq. (jointq_reg)): local search over
 * the integer codes, the scale of the touched group refit in the same move, started from a solution in the format
 * onecomp_quantize_layer returns.  Per output row the objective is
 * f = (w - w^) (H + lam I) (w - w^)^T, w^ = s_g (q - z_g).
 *
 * Moves, order and stopping (the paper fixes only "one code changes a little, the group's scale is refit in the same
 * step, the move is kept iff the objective falls"): codes change by +-1 inside 0 .. 2^bits - 1 (0 .. 2 (2^(bits-1) - 1)
 * for the symmetric grids); zero-points stay; the groups are visited in order, n_pass times; on entering a visit the
 * group's scale is refit to its codes (s = u.p / u.A_tt u with u = q - z, p the gradient of the row's residual with
 * the group taken out); the group's columns are then scanned in order, +1 is tried before -1, the first of the two
 * that lowers f is taken at once; a visit ends with the first scan that takes nothing, or after max_scans scans.  A
 * group whose codes all equal its zero-point is left alone, and no move brings a group there (the refit scale is
 * undefined at u = 0 and the objective cannot fall by such a move; it is excluded on the codes, not by rounding).
 *
 *   W         device, d_out x d_in, row-major, fp32 or bf16: the weights the objective measures against.
 *   H         device fp32, d_in x d_in, symmetric (as onecomp_hessian_accumulate leaves it), read only.
 *             W, H and W_hat must be 16-byte aligned, Q_codes 4-byte aligned (ONECOMP_ERR_INVALID_ARG otherwise).
 *   perm      device int32[d_in] or NULL: the column order the start was quantized in (perm_out of
 *             onecomp_hessian_factor).  As in onecomp_quantize_layer, groups are group_size consecutive columns of
 *             that order, scales / zeros are indexed by group in that order, W, H, Q_codes and W_hat stay in the
 *             original column order; "in order" below means that order.
 *   lam       >= 0, added to the diagonal of H (in the paper's terms 2 n lambda, since H = 2 X^T X).
 *   group_size  divides d_in; a multiple of 16 up to 128, or a multiple of 128 (up to d_in: one group per row).
 *   Q_codes, scales  device, in and out (d_out x d_in uint8, d_out x d_in/group_size fp32).
 *   zeros     device fp32, d_out x d_in/group_size, read only.
 *   W_hat     device fp32 d_out x d_in or NULL, out: s (q - z) of the result.
 *   objective device fp32[2], out: sum over rows of f before and after.
 *   n_moves   device int32, out: number of moves taken.
 *   workspace device scratch, >= onecomp_jointq_workspace_bytes() (about 9 d_out d_in + 4 d_in^2 bytes, 17 d_out d_in
 *             + 4 d_in^2 for groups wider than 128), 256-byte aligned.
 * Arithmetic: fp32; the gradient R (H + lam I) and its rank-group_size updates are fp16 MFMA products of operands
 * split into hi + lo halves (22 significant bits each, H taken as the correlation matrix H_kj / sqrt(H_kk H_jj)),
 * accumulated in fp32.  A decision whose gain is within rounding of zero may fall either way; results are
 * reproducible run to run.
 * Errors: INVALID_ARG (null pointer, bad size, lam < 0, n_pass < 0, max_scans < 1), UNSUPPORTED (dtype, bits, grid,
 * group_size not a multiple of 16, or above 128 and not a multiple of 128), WORKSPACE.
 */
onecomp_status onecomp_jointq_refine(const void* W, onecomp_dtype w_dtype, int64_t d_out, int64_t d_in,
                                     const float* H, const int32_t* perm, float lam, int bits, int group_size,
                                     onecomp_grid grid,
                                     int n_pass, int max_scans, uint8_t* Q_codes, float* scales, const float* zeros,
                                     float* W_hat, float* objective, int32_t* n_moves,
                                     void* workspace, size_t workspace_bytes, void* hip_stream);
size_t onecomp_jointq_workspace_bytes(int64_t d_out, int64_t d_in, int group_size);

/* Static, NUL-terminated description of a status code. */
/*
 * Measurement aid, no part of the method: launches a register-only loop of independent MFMAs (no LDS, no memory
 * traffic) on every compute unit, so that a caller can time what the matrix pipes of this device sustain and quote
 * the Gram accumulation (Sec. 2.5 / 4.3) and the factor (Sec. 4.3.1) against that rate as well as against the
 * published peak, which assumes the boost clock.
 *   kind            0: v_mfma_f32_32x32x16_bf16 (the Gram kernel's instruction), 1: v_mfma_f64_16x16x4_f64 (the factor's)
 *   waves_per_simd  1 or 2 (workgroups of four waves per compute unit)
 *   random_operands 0: the same small constant in every lane; 1: pseudo-random values per lane and per MFMA (the
 *                   pipes draw more power on data that toggles, and the sustained clock follows)
 *   iters           loop trips per wave, 1 .. 2^24; each trip issues 8 MFMAs
 *   sink            device float, at least one element; never written in practice (it keeps the loop alive)
 *   flops_out       HOST double, out: floating-point operations of the launch (2 M N K per MFMA)
 * Asynchronous on hip_stream like every other call; the caller times it with events.
 */
onecomp_status onecomp_mfma_rate_probe(int kind, int waves_per_simd, int random_operands, int64_t iters, float* sink,
                                       double* flops_out, void* hip_stream);

const char* onecomp_status_string(onecomp_status status);

/* Library version as major * 10000 + minor * 100 + patch. */
int onecomp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ONECOMP_H */
