/*
 * tao.h -- C ABI of the MI355X (gfx950) per-operator tolerance engine.
 *
 * For one traced FP32 operator the engine computes the element-wise worst-case
 * IEEE-754 acceptance bound tau (same shape as the operator's output) and
 * checks a claimed output against a locally re-executed one, element by
 * element, also producing a relative-error percentile profile.  The method is
 * that of "TAO: Tolerance-Aware Optimistic Verification for Floating-Point
 * Neural Networks": bound templates of Sec. 3.1 with the constants of
 * App. A.1-A.2, the error profile of Sec. 3.2 Eq. (2) / Sec. 5.3, the leaf
 * check of Sec. 5.4.
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers to binary32 data owned by the
 *    caller; row-major; leading dimensions are in elements.  `tau` buffers are
 *    written, everything else is read only.  Nothing is retained after return.
 *  - `stream` is the caller's hipStream_t passed as void* (NULL = the null
 *    stream).  All work is enqueued asynchronously on it; no entry point
 *    allocates device memory and none synchronises, except the two device self
 *    tests, which copy their findings back to the host.
 *  - `model` is a HOST pointer (NULL selects tao_default_model()).
 *  - Return value: TAO_OK or a negative TAO_ERR_* code; on error nothing has
 *    been enqueued.  Data-dependent failures (a row for which a template has
 *    no finite bound, NaN/+inf inputs) are not status codes: the affected tau
 *    elements are written as NaN, which the check counts as violations.
 *  - Every bound is evaluated so that it never falls below the real-number
 *    value of its formula: sums are inflated by a proven bound on their own
 *    rounding error and the final binary64 value is rounded up to binary32.
 */
#ifndef TAO_H
#define TAO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TAO_NBINS 2048

enum {
    TAO_OK = 0,
    TAO_ERR_NULL = -1,      /* a required pointer is NULL */
    TAO_ERR_SHAPE = -2,     /* negative size, leading dimension smaller than the row, bad stride */
    TAO_ERR_ALIGN = -3,     /* pointer not aligned to 4 bytes (8 for tao_profile) */
    TAO_ERR_K_RANGE = -4,   /* reduction depth k with k*u >= 1: gamma_k undefined (App. A.1) */
    TAO_ERR_MODEL = -5,     /* tao_fp_model field out of range */
    TAO_ERR_KIND = -6,      /* unknown operator kind */
    TAO_ERR_LAUNCH = -7,    /* HIP reported an error; see tao_last_hip_error() */
    TAO_ERR_WORKSPACE = -8  /* workspace missing, misaligned (256 bytes) or too small */
};

/* Floating-point model (App. A.1) and intrinsic accuracies (Sec. 3.1 uses the
 * math library's documented maximum errors; the printed softmax template has
 * 2u for exp).  c_* are relative errors in units of u. */
typedef struct tao_fp_model {
    double u;        /* unit roundoff; 2^-24 for binary32 */
    int mode;        /* TAO_MODE_DETERMINISTIC: gamma_k; TAO_MODE_PROBABILISTIC: gamma~_k(lambda) */
    double lambda;   /* confidence parameter of the probabilistic constant (4 in Sec. 3.1) */
    double c_exp;    /* exp   (default 2) */
    double c_erf;    /* erf   (default 2) */
    double c_rsqrt;  /* rsqrt, or sqrt followed by a division (default 2) */
    double c_div;    /* division by n, or multiplication by a rounded 1/n (default 2) */
    unsigned flags;  /* TAO_FLAG_* */
    double c_log;    /* log   (default 2) */
    double c_sin;    /* sin   (default 4) */
    double c_cos;    /* cos   (default 4) */
    double c_tanh;   /* tanh  (default 4) */
    double c_pow;    /* pow   (default 8) */
} tao_fp_model;

enum { TAO_MODE_DETERMINISTIC = 0, TAO_MODE_PROBABILISTIC = 1 };
enum {
    TAO_FLAG_UNDERFLOW_TERMS = 1u,  /* linear, conv, rope: add K'*2^-149 for gradual underflow in the operator
                                       (App. A.1 excludes it); a product sum that comes out as exactly zero is
                                       then no longer taken for an exact zero (see tao_bound_linear); the
                                       result is the reference value or the next binary32 value above it */
    TAO_FLAG_FAST_ACCUM = 2u,       /* linear: one FP32 accumulation chain over K; still an upper
                                       bound, but looser than the default by about 2*K*u relative */
    TAO_FLAG_CHECK_IN_EPILOGUE = 4u /* tao_bound_check_linear: check in the matrix kernel's epilogue for
                                       every reduction length (no stored bound, its workspace unused);
                                       same result, slower for short reductions */
};

/* Result of tao_check_and_profile (lives in DEVICE memory, 8-byte aligned). */
typedef struct tao_profile {
    uint64_t n;            /* elements examined */
    uint64_t violations;   /* elements with !(|c - r| <= alpha*tau) */
    uint64_t nan_count;    /* elements whose relative error is NaN */
    float max_rel;         /* largest non-NaN relative error (binary32), 0 if none */
    uint32_t accept;       /* 1 iff violations == 0 (Sec. 5.4: any element outside rejects) */
    uint32_t p50_bin, p99_bin, p999_bin;   /* histogram bin holding the nearest-rank percentile */
    float p50, p99, p999;  /* upper edge of that bin (+inf / NaN for the inf / NaN bins) */
    uint32_t pad_;
    uint64_t hist[TAO_NBINS];   /* bin b counts errors e with bits(e) >> 20 == b; NaN -> 2047 */
} tao_profile;

/* Operator kinds of tao_bound_norm and tao_bound_act (operator list of App. A.3). */
enum { TAO_NORM_LAYERNORM = 0, TAO_NORM_RMSNORM = 1, TAO_NORM_BN_AFFINE = 2,
       TAO_NORM_SUM = 3, TAO_NORM_MEAN = 4 };
enum { TAO_ACT_GELU_ERF = 0, TAO_ACT_SILU = 1, TAO_ACT_MUL = 2, TAO_ACT_ADD = 3, TAO_ACT_RELU = 4,
       TAO_ACT_SUB = 5, TAO_ACT_DIV = 6, TAO_ACT_EXACT = 7, TAO_ACT_SQRT = 8, TAO_ACT_RSQRT = 9,
       TAO_ACT_EXP = 10, TAO_ACT_LOG = 11, TAO_ACT_SIN = 12, TAO_ACT_COS = 13, TAO_ACT_TANH = 14,
       TAO_ACT_POW = 15, TAO_ACT_SIGMOID = 16, TAO_ACT_GELU_TANH = 17 };

/* Fills *m with u = 2^-24, deterministic mode, lambda = 4, c_exp = c_erf =
 * c_rsqrt = c_div = c_log = 2, c_sin = c_cos = c_tanh = 4, c_pow = 8, flags = 0. */
void tao_default_model(tao_fp_model *m);

/* Gamma(k) on the host, rounded up in binary64: gamma_k = k u/(1 - k u)
 * (App. A.1 Eq. gamma-def) or gamma~_k(lambda) = exp(lambda sqrt(k) u + k u^2/(1-u)) - 1
 * (Sec. 3.1).  Returns NaN when undefined (k u >= 1); 0 for k <= 0. */
double tao_gamma(long k, const tao_fp_model *model);

/* Linear / matmul / bmm / convolution-as-GEMM bound (Sec. 3.1: reductions use
 * gamma_k with the k of the output element; App. A.2 Eq. det-sum):
 *     tau[b][i][j] = Gamma(K') * ( sum_k |A[b][i][k]| |W[b][j][k]| + |bias[j]| ),
 *     K' = K, or K + 1 when bias != NULL.
 * A: [batch][M][K] with row stride lda and batch stride strideA.
 * W: trans_w == 0: [batch][N][K] (row j = weights of output j, the layout of a
 *    Linear layer); trans_w != 0: [batch][K][N].  Row stride ldw, batch stride
 *    strideW (0 shares one W across the batch).
 * bias: [N] or NULL, shared across the batch.  tau: [batch][M][N], ldt, strideT.
 * The product |A||W| runs on the FP32 matrix cores in chains of 4 k-steps from
 * a zero accumulator; eight chain results are added as a binary32 tree and the
 * root is folded into a binary64 accumulator (at most 7 binary32 roundings per
 * term); the result is inflated by the proven rounding error of that scheme, so
 * exact <= tau <= exact * (1 + 1e-6).  M, N or batch equal to 0 is a no-op;
 * K == 0 gives tau = Gamma(K') |bias| (0 without bias).
 * Gradual underflow inside the bound's own evaluation: partial sums that fall
 * below 2^-126 are rounded absolutely (2^-150 per rounding), so a positive sum
 * also receives (1.25 K + 40) 2^-150 before the inflation ((K + 63) 2^-149 on the
 * BF16 path); the upper tolerance then reads exact (1 + 1e-6) + Gamma(K') times
 * that term, which only matters for bounds that are themselves about 2^-126 or
 * smaller.  A sum that comes out as exactly 0 is reported as the exact zero of
 * zero operands or padding; operands whose every product lies below 2^-150
 * (which binary32 arithmetic cannot represent either: App. A.1 excludes
 * underflow) need TAO_FLAG_UNDERFLOW_TERMS to stay covered. */
int tao_bound_linear(const float *A, const float *W, const float *bias, float *tau,
                     long M, long N, long K, long lda, long ldw, long ldt, int trans_w,
                     long batch, long strideA, long strideW, long strideT,
                     const tao_fp_model *model, void *stream);

/* The same bound on the BF16 matrix cores (16 x the FP32 MFMA rate): every magnitude is cut
 * exactly into three BF16 pieces by a pre-pass into ws, and eight BF16 products per operand pair
 * are accumulated with a binary64 fold per 16 k-steps; the rounding behaviour of the instruction,
 * characterised on the device and re-checked by tao_selftest_matrix_core_bf16, bounds the computed sum
 * within [S(1 - 11.5u), S(1 + 2.5u)], so again exact <= tau <= exact * (1 + 1e-6).  Arguments as
 * tao_bound_linear, plus ws: device scratch, 256-byte aligned, at least
 * tao_linear_split_workspace_bytes(M, N, K, batch, shared_w) bytes (shared_w != 0 when
 * strideW == 0 or batch == 1); contents irrelevant before and garbage after; calls sharing ws
 * must be ordered on one stream.  Operands below 2^-110 in magnitude keep the bound sound but may
 * push it beyond 1e-6.  TAO_FLAG_FAST_ACCUM is ignored.  TAO_ERR_WORKSPACE when ws is missing,
 * misaligned or too small. */
int tao_bound_linear_split(const float *A, const float *W, const float *bias, float *tau,
                           long M, long N, long K, long lda, long ldw, long ldt, int trans_w,
                           long batch, long strideA, long strideW, long strideT,
                           const tao_fp_model *model, void *ws, size_t ws_bytes, void *stream);
size_t tao_linear_split_workspace_bytes(long M, long N, long K, long batch, int shared_w);
/* 1 when the BF16 path is expected to be the faster one for this shape on the current device (its
 * 128 x 128 tiles, times the parts a long reduction is cut into when they are few, fill the device;
 * at least 256 rows; 256 columns, or 128 with a long reduction of whole 32-step groups, or 64 where
 * the tiles are few enough for four parts), else 0.  Measured rule of thumb.  Host only. */
int tao_linear_split_preferred(long M, long N, long K, long batch);
/* The bound of tao_bound_linear_split checked on the spot (Sec. 5.4 leaf check, Sec. 5.3 profile):
 * *out receives exactly what tao_check_and_profile(claimed, y_ref, tau, ...) would return for the
 * tau that tao_bound_linear_split computes from the same operands, but tau is compared in registers
 * in the matrix kernel's epilogue and only stored when `tau` is not NULL (layout ldy / strideY, like
 * y_ref and claimed: M x N per batch entry, ldy >= N).  Where the epilogue would cost more than it
 * saves -- reductions up to 1024 long with contiguous outputs that are not cut into parts -- the bound is stored instead (into
 * `tau`, else into the workspace) and the streaming check reads it: the same result, sooner.
 * y_ref: the verifier's re-executed output, claimed: the proposer's.  out: DEVICE, fully overwritten,
 * valid once the stream has drained.  ws / ws_bytes: DEVICE scratch of at least
 * tao_bound_check_linear_workspace_bytes(...), 256-byte aligned.  Runs the BF16-split kernel for every
 * shape (tao_linear_split_preferred tells where that is the faster one).  Errors as for
 * tao_bound_linear_split and tao_check_and_profile; TAO_ERR_SHAPE also for M N batch >= 2^36. */
int tao_bound_check_linear(const float *A, const float *W, const float *bias, const float *y_ref,
                           const float *claimed, float *tau,
                           long M, long N, long K, long lda, long ldw, long ldy, int trans_w,
                           long batch, long strideA, long strideW, long strideY,
                           double alpha, double eps_rel, const tao_fp_model *model, tao_profile *out,
                           void *ws, size_t ws_bytes, void *stream);
size_t tao_bound_check_linear_workspace_bytes(long M, long N, long K, long batch, int shared_w);
/* Prepared operands.  The pre-pass of the BF16 path turns an operand into its three-piece image; an
 * operand that takes part in many products -- the committed weights of a layer, which never change
 * (Sec. 5.2), or an activation that feeds several projections -- can be split once and reused:
 *   tao_split_operand          writes the image of src: [batch][rows][K] with row stride ld and batch
 *                              stride `stride` (trans == 0), or [batch][K][rows] (trans != 0: a weight
 *                              stored K x N); rows = M for the A side, N for the W side.  image: DEVICE,
 *                              256-byte aligned, at least tao_split_image_bytes(rows, K, batch) bytes
 *                              (about 6 bytes per element, rows and K padded to 128 and 32).  An image
 *                              depends on (rows, K, batch) only and may be used on either side.
 *   tao_bound_linear_images    tao_bound_linear_split on two images: the same tau, bit for bit.
 *                              shared_w != 0: one W image for every batch entry.  ws: DEVICE scratch of
 *                              tao_linear_images_workspace_bytes(M, N, K, batch) bytes (0 unless the
 *                              launch has fewer tiles than compute units and cuts the reduction into
 *                              parts; ws may then be NULL), 256-byte aligned.
 *   tao_bound_check_linear_images  tao_bound_check_linear on two images (same result, field for field);
 *                              ws of tao_check_linear_images_workspace_bytes(M, N, K, batch) bytes.
 * Images are read only by the products; products that share an image may run concurrently.  Errors
 * as for the calls they mirror; TAO_ERR_ALIGN for an image that is not 256-byte aligned. */
size_t tao_split_image_bytes(long rows, long K, long batch);
int tao_split_operand(const float *src, long rows, long K, long ld, int trans, long batch, long stride,
                      void *image, size_t image_bytes, void *stream);
int tao_bound_linear_images(const void *A_image, const void *W_image, const float *bias, float *tau,
                            long M, long N, long K, long ldt, long batch, long strideT, int shared_w,
                            const tao_fp_model *model, void *ws, size_t ws_bytes, void *stream);
size_t tao_linear_images_workspace_bytes(long M, long N, long K, long batch);
int tao_bound_check_linear_images(const void *A_image, const void *W_image, const float *bias, const float *y_ref,
                                  const float *claimed, float *tau, long M, long N, long K, long ldy, long batch,
                                  long strideY, int shared_w, double alpha, double eps_rel, const tao_fp_model *model,
                                  tao_profile *out, void *ws, size_t ws_bytes, void *stream);
size_t tao_check_linear_images_workspace_bytes(long M, long N, long K, long batch);

/* 1 if tao_bound_check_linear checks a product of this shape (contiguous outputs) without storing the
 * bound -- in the matrix kernel's epilogue, or in the pass that adds the parts of a reduction cut into
 * parts --, 0 if it stores the bound and runs the streaming check.  Host only: for callers that time or
 * schedule the two kernels separately. */
int tao_bound_check_linear_in_epilogue(long M, long N, long K, long batch);
/* Probes v_mfma_f32_32x32x16_bf16 with `cases` seeded non-negative cases (0 = 3072; the model was
 * fitted on 280 000 of the same generator's kind, which a caller may ask for) and compares every
 * result with the exact integer model the inflation of tao_bound_linear_split rests on.  *report
 * (HOST): bit 0 every case of the three normal-range families reproduced bit for bit; bit 1 every
 * result from a zero accumulator within [S(1 - 10u), S(1 + 2u)] of the exact sum S; bit 2 every result
 * of the fourth family (products and sums between 2^-150 and 2^-124: the subnormal range) within two
 * steps of 2^-149 of the exact sum, the absolute term the bound carries for that range.
 * ws / ws_bytes: DEVICE scratch of tao_selftest_workspace_bytes(cases) bytes, 256-byte aligned (the
 * self tests allocate nothing on the device).  Synchronises the stream. */
int tao_selftest_matrix_core_bf16(unsigned *report, long cases, void *ws, size_t ws_bytes, void *stream);
size_t tao_selftest_workspace_bytes(long cases);

/* 2-D convolution bound without a stored patch matrix (Sec. 3.1: conv is a
 * reduction with gamma_k of the output element; Conv2D of the operator list,
 * App. A.3):
 *     tau[n][oh][ow][co] = Gamma(K') * ( sum_{r,s,c} |x[n][oh*stride_h - pad_h + r*dil_h]
 *                                        [ow*stride_w - pad_w + s*dil_w][c]| |w[co][r][s][c]| + |bias[co]| ),
 *     K = R*S*C for every output element, K' = K or K + 1 with a bias.
 * Taps that fall into the zero padding add nothing and keep their place in K.
 * x: [batch][H][W][C] channels last, contiguous (device).  w: [Cout][R][S][C]
 * contiguous.  bias: [Cout] or NULL.  tau: [batch][OH][OW][Cout] contiguous,
 * OH = (H + 2 pad_h - dil_h (R-1) - 1)/stride_h + 1, OW likewise; groups = 1.
 * Same accumulation scheme and guarantee as tao_bound_linear, applied to the
 * implicit patch matrix [batch*OH*OW][R*S*C]: its 32-wide k slabs are gathered
 * from x while loading (16-byte gathers when C is a multiple of 32, x is
 * 16-byte aligned and at most 2^31 bytes; element by element otherwise).
 * Errors: TAO_ERR_SHAPE for a non-positive filter size, stride or dilation, a
 * negative padding, a filter larger than the padded input, any extent >= 2^28,
 * batch*OH*OW or R*S*C >= 2^31; TAO_ERR_K_RANGE as for tao_bound_linear.
 * batch*OH*OW == 0 or Cout == 0 is a no-op. */
int tao_bound_conv2d(const float *x, const float *w, const float *bias, float *tau,
                     long batch, long H, long W, long C, long Cout, long R, long S,
                     long stride_h, long stride_w, long pad_h, long pad_w, long dil_h, long dil_w,
                     const tao_fp_model *model, void *stream);

/* The same convolution bound on the BF16 matrix cores (the scheme of tao_bound_linear_split: three
 * exact BF16 pieces per operand, same guarantee): the filters' image is written into ws by a small
 * pre-pass, the implicit patch matrix is gathered from x and cut into its pieces while the product
 * loads it, so no patch matrix and no image of it is ever stored.  Arguments as tao_bound_conv2d.
 * Served when C is a multiple of 32, x is 16-byte aligned and the launch has enough 128 x 128 output
 * tiles to keep the reduction in one part (tao_conv2d_split_supported returns 1; host only):
 * TAO_ERR_SHAPE otherwise -- tao_bound_conv2d serves every shape.
 * tao_bound_check_conv2d: the bound checked on the spot like tao_bound_check_linear (y_ref, claimed and
 * the optional tau: [batch][OH][OW][Cout] contiguous; the result of tao_check_and_profile on the stored
 * bound, field for field).  ws / ws_bytes: DEVICE scratch of tao_conv2d_split_workspace_bytes(...,
 * with_check) bytes, 256-byte aligned. */
int tao_conv2d_split_supported(long batch, long H, long W, long C, long Cout, long R, long S,
                               long stride_h, long stride_w, long pad_h, long pad_w, long dil_h, long dil_w);
size_t tao_conv2d_split_workspace_bytes(long batch, long H, long W, long C, long Cout, long R, long S,
                                        long stride_h, long stride_w, long pad_h, long pad_w, long dil_h, long dil_w,
                                        int with_check);
int tao_bound_conv2d_split(const float *x, const float *w, const float *bias, float *tau,
                           long batch, long H, long W, long C, long Cout, long R, long S,
                           long stride_h, long stride_w, long pad_h, long pad_w, long dil_h, long dil_w,
                           const tao_fp_model *model, void *ws, size_t ws_bytes, void *stream);
int tao_bound_check_conv2d(const float *x, const float *w, const float *bias, const float *y_ref, const float *claimed,
                           float *tau, long batch, long H, long W, long C, long Cout, long R, long S,
                           long stride_h, long stride_w, long pad_h, long pad_w, long dil_h, long dil_w,
                           double alpha, double eps_rel, const tao_fp_model *model, tao_profile *out,
                           void *ws, size_t ws_bytes, void *stream);

/* Softmax over the last dimension (Sec. 3.1 "Minimal example: softmax", closed
 * to second order).  x, y_ref, tau: [rows][cols] with row stride ld; y_ref is
 * the verifier's own binary32 softmax output.  Per row, with n = cols:
 *     a_j = u(|x_j| + |max x|), rho_j = (a_j(1+a_j) + c_exp u)/(1 - c_exp u), q_j = y_j/(1-u),
 *     sigma = Gamma(n-1) sum q + (1 + Gamma(n-1)) sum rho q,
 *     tau_i = q_i rho_i + q_i (1 + rho_i) sigma/(1 - sigma) + u y_i.
 * Entries with x = -inf are masked: tau = 0 and they are left out of the sums.
 * A row that is fully masked, contains NaN or +inf, or has sigma >= 1 gets NaN. */
int tao_bound_softmax(const float *x, const float *y_ref, float *tau, long rows, long cols, long ld,
                      const tao_fp_model *model, void *stream);

/* Row-wise normalisations and reductions over the last dimension (operators of
 * App. A.3; templates follow the primitive rule of Sec. 3.1).  x: [rows][cols],
 * row stride ld.  y_ref: the verifier's binary32 output ([rows][cols] with row
 * stride ld; [rows] for MEAN; unused for SUM), or NULL: the fresh-rounding term
 * u|y| of the primitive rule is then taken at an upper bound Y of |y| over every
 * canonical execution, formed from the inputs (a bound that knows y is never larger):
 *   LAYERNORM (|x - mean| r |g| + E_p + |b|)(1+u), E_p the bound before that term;  RMSNORM |x g| R (1+u)^2;
 *   BN_AFFINE (|x s|(1+u) + |t|)(1+u);  MEAN (sum|x| / cols)(1 + Gamma(cols-1))(1 + c_div u).
 *  LAYERNORM  y = (x - mean) rsqrt(var + eps) g + b; g = gamma_or_scale[cols] or NULL (= 1),
 *             b = beta_or_shift[cols] or NULL (= 0; enters a bound only through Y); two-pass algorithm.
 *  RMSNORM    y = g (x rsqrt(mean(x^2) + eps)); g as above.
 *  BN_AFFINE  y = x s_c + t_c per column c; s = gamma_or_scale (required), t = beta_or_shift.
 *  SUM, MEAN  tau: [rows];  Gamma(cols-1) sum|x|  (/cols + |y| c_div u/(1 - c_div u) for MEAN).
 * eps is rounded to binary32 first, as the operator does.  A row whose bound is
 * not finite (lower end of var + eps not positive) gets NaN.
 * TAO_ERR_K_RANGE when Gamma(cols - 1) is undefined (cols u >= 1) and, for LAYERNORM and
 * RMSNORM (also in tao_bound_groupnorm and tao_bound_check_norm), when it exceeds 1/2
 * (cols above about 5.59 million with the default model): the template subtracts the
 * variance's own error bound from the variance, and nothing useful is left of it there. */
int tao_bound_norm(int kind, const float *x, const float *y_ref,
                   const float *gamma_or_scale, const float *beta_or_shift, double eps,
                   float *tau, long rows, long cols, long ld,
                   const tao_fp_model *model, void *stream);

/* GroupNorm (operator list of App. A.3) of a channel-major tensor x[batch][channels][positions]
 * (contiguous; positions = product of the spatial extents): every (sample, group) is a
 * LayerNorm over its channels/groups channels times all positions, with gamma[c], beta[c]
 * of a channel applied at all its positions; the bound is tao_bound_norm's LAYERNORM
 * formula on those rows (n = channels/groups * positions).  gamma, beta: [channels] or
 * NULL.  y_ref, tau: like x.  groups == channels gives instance normalisation.
 * Rows of more than 8192 elements, when there are fewer than 512 of them, are cut
 * into chunks that exchange partial sums through ws: device memory, 8-byte
 * aligned, at least tao_groupnorm_workspace_bytes(...) bytes (0 otherwise; ws
 * may then be NULL), contents irrelevant before and after; calls that share ws must be
 * ordered on one stream.
 * TAO_ERR_SHAPE when channels is not a multiple of groups or a row reaches 2^31
 * elements; TAO_ERR_K_RANGE when n u >= 1; TAO_ERR_WORKSPACE when ws is too small. */
int tao_bound_groupnorm(const float *x, const float *y_ref, const float *gamma, const float *beta,
                        double eps, float *tau, long batch, long channels, long positions, long groups,
                        const tao_fp_model *model, void *ws, size_t ws_bytes, void *stream);
size_t tao_groupnorm_workspace_bytes(long batch, long channels, long positions, long groups);

/* Element-wise operators (App. A.3), flat length n.  y_ref is the verifier's
 * binary32 output and is always required.
 *  GELU_ERF  y = 0.5 x (1 + erf(x/sqrt 2)); needs x.
 *            tau = |x|/2 ((2/sqrt pi) e^{-t_lo^2} E_t + c_erf u min(1, (2/sqrt pi)|t|(1+4u)))
 *                  + u |y| (1 + 1/(1-u)),  t = x/sqrt 2, E_t = (2u+u^2)|t|, t_lo = max(0,|t|-E_t).
 *  SILU      y = x/(1 + exp(-x)): tau = |y| (w/(1-u) + u), w = (c_exp u/(1-c_exp u) + u)/(1-u).
 *  GELU_TANH y = 0.5 x (1 + tanh(p)), p = sqrt(2/pi)(x + 0.044715 x^3); needs x.
 *            tau = |x|/2 (sech^2(p_lo) E_p + c_tanh u min(1, |p|(1+Gamma(7)))) + u |y| (1 + 1/(1-u)),
 *            E_p = Gamma(7)|p| (seven roundings at most in either association of p,
 *            constants included), p_lo = max(0, |p| - E_p).
 *  SILU, SIGMOID  y = x/(1 + exp(-x)), 1/(1 + exp(-x)):
 *            tau = |y| (w/(1-u) + u), w = (c_exp u/(1-c_exp u) + u)/(1-u).
 *  MUL, ADD, SUB, SQRT  one correctly rounded operation: tau = u |y|.
 *  RELU, EXACT  (Neg, Abs, Max, Min, max-pooling, masked fill, data movement): tau = 0.
 *  DIV, RSQRT, EXP, LOG, SIN, COS, TANH, POW  a library function accurate to c u
 *            relatively (c = c_div, c_rsqrt, c_exp, c_log, c_sin, c_cos, c_tanh, c_pow):
 *            tau = |y| c u/(1 - c u).
 * x and x2 (the operands) are ignored except by the two GELU kinds and may be NULL otherwise. */
int tao_bound_act(int kind, const float *x, const float *x2, const float *y_ref, float *tau, long n,
                  const tao_fp_model *model, void *stream);

/* Rotary position embedding (App. A.3: Sin/Cos tables applied to activations;
 * each output is a two-term dot product of exact inputs, Sec. 3.1 reductions):
 *     y_a = x_a cos - x_b sin,  y_b = x_b cos + x_a sin,
 *     tau_a = Gamma(2)(|x_a cos| + |x_b sin|),  tau_b = Gamma(2)(|x_b cos| + |x_a sin|).
 * x, tau: [rows][d] contiguous, d even; cos, sin: [npos][d/2] contiguous; row r
 * uses table row (r / inner) % npos (inner = heads for a [token][head][d]
 * layout, 1 for [head][token][d]).  Pairs (a, b) = (j, j + d/2), or (2j, 2j+1)
 * when interleaved != 0.  TAO_ERR_SHAPE for odd d, inner < 1 or npos < 1. */
int tao_bound_rope(const float *x, const float *cos_table, const float *sin_table, float *tau,
                   long rows, long d, long inner, long npos, int interleaved,
                   const tao_fp_model *model, void *stream);

/* tao_bound_norm checked on the spot, for kind TAO_NORM_LAYERNORM and TAO_NORM_RMSNORM (TAO_ERR_KIND
 * otherwise): *out receives exactly what tao_check_and_profile(claimed, y_ref, tau, ...) returns for the
 * tau of tao_bound_norm(kind, x, y_ref, gamma, beta, eps, ...), never stored.  claimed: DEVICE, laid out
 * like x and y_ref (rows x cols, leading dimension ld).  ws / ws_bytes: DEVICE scratch of at least
 * tao_check_workspace_bytes(rows * cols), 256-byte aligned. */
int tao_bound_check_norm(int kind, const float *x, const float *y_ref, const float *gamma, const float *beta,
                         double eps, const float *claimed, long rows, long cols, long ld,
                         double alpha, double eps_rel, const tao_fp_model *model, tao_profile *out,
                         void *ws, size_t ws_bytes, void *stream);

/* tao_bound_rope checked on the spot: *out receives exactly what tao_check_and_profile(claimed,
 * y_ref, tau, ...) returns for the tau of tao_bound_rope(x, cos_table, sin_table, ...), never stored.
 * y_ref, claimed: DEVICE, rows x d contiguous like x.  ws / ws_bytes: DEVICE scratch of at least
 * tao_check_workspace_bytes(rows * d), 256-byte aligned. */
int tao_bound_check_rope(const float *x, const float *cos_table, const float *sin_table, const float *y_ref,
                         const float *claimed, long rows, long d, long inner, long npos, int interleaved,
                         double alpha, double eps_rel, const tao_fp_model *model, tao_profile *out,
                         void *ws, size_t ws_bytes, void *stream);

/* Leaf check (Sec. 5.4) and relative-error profile (Sec. 5.3; Sec. 3.2 Eq. 2)
 * of n elements, in IEEE binary64 per element:
 *     d = |claimed - ref|;  violation iff !(d <= alpha * tau);
 *     e = d / (|ref| + eps_rel), cast to binary32;  bin = NaN ? 2047 : bits(e) >> 20.
 * Percentiles p50, p99, p99.9 by nearest rank, rank = max(1, ceil(n p)), on the
 * histogram; alpha is the bound scale factor of Sec. 4.5 (1 = the paper's check).
 * eps_rel must be >= 0 (TAO_ERR_SHAPE for a negative or NaN value, here and in every entry point
 * that takes it).
 * out: DEVICE pointer, fully overwritten; valid once the stream has drained.
 * ws / ws_bytes: DEVICE scratch of at least tao_check_workspace_bytes(n). */
int tao_check_and_profile(const float *claimed, const float *ref, const float *tau, long n,
                          double alpha, double eps_rel, tao_profile *out,
                          void *ws, size_t ws_bytes, void *stream);

/* tao_check_and_profile for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels and, field for field, the same result, with the partial histograms and counters in a
 * fixed array inside the library (about 2.1 MB of device memory per GPU the call has run on, held
 * until the process ends) instead of `ws`.  Allocates nothing and calls no allocating routine; the
 * first call on a device looks up the array's address there.  n may be at most
 * TAO_STATIC_CHECK_MAX_N (TAO_ERR_SHAPE beyond it: the per-workgroup counters are 32 bits wide);
 * other errors as for tao_check_and_profile.  All calls on one GPU share the one array: calls that
 * may overlap there (different streams, different threads) race and must be ordered by the caller;
 * calls on one stream are ordered by the stream.  Nothing has to be cleared between calls. */
#define TAO_STATIC_CHECK_MAX_N ((1L << 36) - 1)
int tao_check_and_profile_static(const float *claimed, const float *ref, const float *tau, long n,
                                 double alpha, double eps_rel, tao_profile *out, void *stream);

/* Bytes of DEVICE workspace tao_check_and_profile needs for n elements (per-
 * workgroup partial histograms and counters).  The workspace must be 256-byte
 * aligned; its contents on entry do not matter and are garbage afterwards.
 * Calls that share a workspace must be ordered on one stream. */
size_t tao_check_workspace_bytes(long n);

/* tao_bound_act checked on the spot: *out receives exactly what tao_check_and_profile(claimed,
 * y_ref, tau, ...) returns for the tau of tao_bound_act(kind, x, x2, y_ref, ...), formed in
 * registers and never stored (Sec. 5.4 leaf check, Sec. 5.3 profile; 8 - 12 bytes per element
 * instead of 20 - 24).  Arguments as for the two calls; ws / ws_bytes: DEVICE scratch of at least
 * tao_check_workspace_bytes(n), 256-byte aligned. */
int tao_bound_check_act(int kind, const float *x, const float *x2, const float *y_ref, const float *claimed,
                        long n, double alpha, double eps_rel, const tao_fp_model *model, tao_profile *out,
                        void *ws, size_t ws_bytes, void *stream);

/* Softmax bound and leaf check in one pass (Sec. 3.1 softmax template, Sec. 5.4
 * check, Sec. 5.3 profile): the result is, field by field, that of
 *     tao_bound_softmax(x, y_ref, tau, ...); tao_check_and_profile(claimed, y_ref, tau, ...)
 * but tau lives only in registers (rounded to binary32 as it would have been
 * stored): the pass reads x, y_ref and claimed once and writes nothing but the
 * profile.  x, y_ref, claimed: [rows][cols], row stride ld (n = rows * cols).
 * alpha, eps_rel, out, ws, ws_bytes: as for tao_check_and_profile (workspace of
 * tao_check_workspace_bytes(n)).  Errors as for the two calls. */
int tao_bound_check_softmax(const float *x, const float *y_ref, const float *claimed,
                            long rows, long cols, long ld, double alpha, double eps_rel,
                            const tao_fp_model *model, tao_profile *out,
                            void *ws, size_t ws_bytes, void *stream);

/* Error profile of tao_profile_errors (lives in DEVICE memory, 8-byte aligned). */
#define TAO_NGRID 22   /* percentile grid P = {1, 5, 10, ..., 95, 99, 100} of Sec. 3.2 / Sec. 5.3 */
typedef struct tao_error_profile {
    uint64_t n;                 /* elements examined */
    uint64_t nan_count;         /* elements whose relative error is NaN */
    float max_abs, max_rel;     /* largest non-NaN absolute / relative error (binary32), 0 if none */
    float abs_p[TAO_NGRID];     /* percentile values on the grid: upper edge of the bin holding the */
    float rel_p[TAO_NGRID];     /*   nearest-rank element, capped by the exact maximum               */
    uint32_t abs_bin[TAO_NGRID], rel_bin[TAO_NGRID];   /* that bin */
    double p_max;               /* selection statistic; NaN without thresholds */
    uint32_t offending;         /* 1 iff p_max > 1 */
    uint32_t pad_;
    uint64_t hist_abs[TAO_NBINS], hist_rel[TAO_NBINS];  /* bin = bits(error) >> 20; NaN -> 2047 */
} tao_error_profile;

/* Empirical error profile of two outputs of one operator, as used for calibration (Sec. 3.2
 * Eq. 1-2) and for child selection in the dispute game (Sec. 5.3): per element, in IEEE binary64,
 *     abs = |claimed - ref|,   rel = abs / (|ref| + eps_rel),   both cast to binary32;
 * two histograms with the bin key of tao_check_and_profile; for each p of the 22-point grid the
 * nearest-rank percentile (rank = max(1, ceil(n p / 100))) reported as its bin and that bin's
 * upper edge, capped by the exact maximum, so p = 100 is the maximum itself; and, when the
 * committed threshold tables thr_abs[22], thr_rel[22] (DEVICE pointers, both or neither) are
 * given, the selection statistic
 *     p_max = max over the grid of { abs_p / thr_abs, rel_p / thr_rel }  (binary64 quotients,
 *     NaN quotients skipped),   offending = (p_max > 1).
 * out: DEVICE pointer, fully overwritten; valid once the stream has drained.
 * ws / ws_bytes: DEVICE scratch of at least tao_profile_workspace_bytes(n), 256-byte aligned;
 * contents on entry do not matter; calls sharing a workspace must be ordered on one stream. */
int tao_profile_errors(const float *claimed, const float *ref, long n, double eps_rel,
                       const float *thr_abs, const float *thr_rel, tao_error_profile *out,
                       void *ws, size_t ws_bytes, void *stream);
size_t tao_profile_workspace_bytes(long n);

/* Offline calibration of an operator's thresholds (Sec. 3.2): `profiles` is a DEVICE array of
 * `count` >= 1 results of tao_profile_errors (one per device pair and input).  Per grid point
 *     env_abs(p) = max over the runs of abs_p(p),   env_rel(p) likewise (NaN entries are skipped;
 *                  NaN only if every run is NaN there),
 *     thr_abs(p) = alpha * env_abs(p),  thr_rel(p) = alpha * env_rel(p)   (alpha = 3 in the paper),
 * the product being one binary64 multiplication rounded UP to binary32, so that a threshold is never
 * below alpha times the envelope.  env_abs / env_rel (DEVICE, 22 values, may be NULL) receive the
 * envelope, thr_abs / thr_rel (DEVICE, 22 values) the thresholds, in the form tao_profile_errors
 * takes them.  alpha must be finite and >= 0. */
int tao_calibrate_thresholds(const tao_error_profile *profiles, long count, double alpha,
                             float *env_abs, float *env_rel, float *thr_abs, float *thr_rel, void *stream);

/* Projection of a tentative perturbation onto the admissible set of the theoretical bound
 * (Sec. 4.4 (i)): out = clip(delta, -alpha tau, alpha tau) element by element.  The cap alpha*tau is
 * one binary64 product; an element beyond it takes the largest binary32 value not above the cap
 * (the result never leaves the set through rounding), its sign kept; NaN elements stay NaN.
 * delta, tau, out: DEVICE, n values each; out may be delta.  alpha finite and >= 0
 * (TAO_ERR_SHAPE otherwise, as for n < 0). */
int tao_project_clip(const float *delta, const float *tau, double alpha, float *out, long n, void *stream);

/* Projection onto the admissible set of the empirical thresholds (Sec. 4.4 (ii), cap curve of
 * Sec. 4.2): with a = |delta| sorted increasingly (equal values in index order) and ranks
 * k = 1..n,
 *     r_k = ((k - 0.5) / n) * 100,
 *     C(r) = c_{j-1} + (c_j - c_{j-1}) * ((r - p_{j-1}) / (p_j - p_{j-1})),   j the first grid
 *            point with r <= p_j,  c_j = alpha * thr_abs[j],  (p_0, c_0) = (0, 0)     (binary64),
 *     cap_k = max over k' <= k of C(r_k'),
 *     out[sigma(k)] = sign(delta[sigma(k)]) * min(a_sigma(k), cap_k),
 * a capped element taking the largest binary32 value not above its cap.  NaN elements rank last
 * and stay NaN.  The result is bit-identical to a stable sort followed by those steps.
 * delta, out: DEVICE, n values (out may be delta itself, no other overlap); thr_abs: DEVICE, the operator's 22 absolute
 * thresholds on the grid of Sec. 3.2 (as tao_calibrate_thresholds writes them), which must be
 * finite and >= 0 (not checked: device data; other values cannot fault, the result is then
 * unspecified).  ws / ws_bytes: DEVICE scratch of at least tao_project_workspace_bytes(n)
 * (about 16 n bytes), 256-byte aligned, contents on entry irrelevant.
 * TAO_ERR_SHAPE for n < 0, n >= 2^31 or alpha not finite and >= 0; TAO_ERR_WORKSPACE. */
int tao_project_empirical(const float *delta, const float *thr_abs, double alpha, float *out, long n,
                          void *ws, size_t ws_bytes, void *stream);
size_t tao_project_workspace_bytes(long n);   /* 0 for n <= 0 or n >= 2^31 */

/* Runs crafted inputs through the FP32 matrix-core instruction and reports, as
 * a bit mask in *report (HOST pointer), which modelling assumptions of the
 * linear bound's inflation hold on this device: bit 0 accumulation rounds to
 * nearest-even; bit 1 subnormal products are kept (no flush); bit 2 a 6-step
 * chain on random non-negative data stays within gamma_6 of the exact sum.
 * ws / ws_bytes: DEVICE scratch of tao_selftest_workspace_bytes(0) bytes, 256-byte aligned.
 * Synchronises the stream.  For callers that want to verify the device once. */
int tao_selftest_matrix_core(unsigned *report, void *ws, size_t ws_bytes, void *stream);

/* hipError_t of the most recent TAO_ERR_LAUNCH on this thread (0 if none). */
int tao_last_hip_error(void);
const char *tao_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* TAO_H */
