/*
 * quest.h - C ABI of the QuEST quantized-linear hot path for AMD MI355X (gfx950).
 *
 * The operations are those of the QuEST linear layer (arXiv 2502.05003):
 *   forward  (Algorithm 1): x_h = HT(x), xhat_h = proj(x_h) for activations and weights,
 *                           y = xhat_h what_h^T, plus the two trust masks;
 *   backward (Algorithm 2): dL/dxhat_h = dL/dy what_h, dL/dx = IHT(M_x (.) dL/dxhat_h),
 *                           dL/dwhat_h = (dL/dy)^T xhat_h, dL/dw = IHT(M_w (.) dL/dwhat_h).
 *
 * Notation.  K: row length (the matmul dimension).  n: Hadamard block (power of two, n | K).
 * b: bits, L = 2^b levels.  Per row: rms = sqrt(mean_j x_h[j]^2), grid spacing in RMS units
 * D = 2 alpha / (L - 1), cell index k = clamp(floor(x_h / (D rms)), -L/2, L/2 - 1), stored code
 * c = k + L/2 in [0, L - 1], odd integer u = 2k + 1 = 2c - (L - 1), scale s = alpha rms / (L - 1);
 * the quantized value is xhat_h = s * u (Eq. 1 with the RMS normalisation of Sec. 3.1).
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer unless the comment says "host".  The caller owns
 *     all buffers, scratch included; the library allocates nothing, frees nothing and never
 *     synchronises: a call validates its arguments on the host and enqueues kernels on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream).  Every enqueue call may be
 *     captured into a HIP graph (call quest_init first, so that no kernel attribute has to change
 *     during capture); calls on different streams may overlap as long as they share no output or
 *     workspace.
 *   - Scratch memory: an entry point that needs it takes `workspace` / `workspace_bytes`; the host
 *     function <entry point>_workspace_bytes(...) gives the size for a shape (0: none needed, -1:
 *     the shape is not supported).  The workspace must be 16-byte aligned and must not be used by
 *     anything else until the call's kernels have finished; its contents afterwards are undefined.
 *   - Errors are return codes.  A validation error (every code but QUEST_ERR_LAUNCH) means nothing
 *     was launched.  QUEST_ERR_LAUNCH means the HIP runtime refused a launch; an entry point that
 *     enqueues several kernels may have enqueued the earlier ones, and its outputs are undefined.
 *   - Outputs must not alias inputs.
 *   - "bf16" is the upper half of an IEEE binary32, stored as uint16_t.
 *   - Code container width cb(b): 1 -> 1, 2 -> 2, 3 -> 4, 4 -> 4, 8 -> 8 bits.  Element j of a row
 *     occupies bits [(j*cb) mod 8, +cb) of byte floor(j*cb/8) (little-endian: at b = 4 the even
 *     element is the low nibble).  Mask bitmaps use the same order with one bit per element
 *     (element j = bit j mod 8 of byte j/8); 1 = trusted.
 */
#ifndef QUEST_H
#define QUEST_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QUEST_OK = 0,
    QUEST_ERR_NULL = 1,    /* a required pointer is NULL */
    QUEST_ERR_SHAPE = 2,   /* rows/cols/M/N/K/ld out of the supported range */
    QUEST_ERR_BITS = 3,    /* bits not in {1,2,3,4,8} (quantizer) or not supported by the GEMM */
    QUEST_ERR_BLOCK = 4,   /* had_block not a power of two, or does not divide cols */
    QUEST_ERR_ALIGN = 5,   /* pointer or leading dimension not 16-byte aligned */
    QUEST_ERR_DTYPE = 6,   /* unknown quest_dtype */
    QUEST_ERR_LAUNCH = 7,  /* the HIP runtime refused the launch */
    QUEST_ERR_ARG = 8,     /* any other invalid argument (non-finite alpha, workspace missing or too small) */
    QUEST_ERR_SCRATCH = 9  /* quest_lowbit_gemm_static: the shape needs more than QUEST_STATIC_SCRATCH_BYTES */
} quest_status;

typedef enum { QUEST_F32 = 0, QUEST_BF16 = 1 } quest_dtype;

/* Limits checked by the entry points. */
#define QUEST_MAX_COLS 16384      /* longest row the quantizer / trust backward accept */
#define QUEST_MAX_HAD_BLOCK 16384 /* largest Hadamard block */
#define QUEST_STATIC_SCRATCH_BYTES (32 << 20) /* built-in scratch of quest_lowbit_gemm_static, per GPU */

/*
 * Algorithm 1, one operand (call once for x, once for w):
 *   x_h = HT(x) (Sec. 3.1, Eq. 3: block-diagonal normalised Sylvester transform along the row),
 *   xhat_h = proj_alpha(x_h) (Sec. 3.1 "Gaussian Fitting": RMS-normalise, clip at alpha, round to
 *   the zero-free 2^b-level grid of Eq. 1), and the trust mask M = 1[|xhat_h - x_h| <= T],
 *   T = alpha / (2^b - 1) in RMS units (Sec. 3.2).
 *
 *   x           [rows, ld] row-major, dtype f32 or bf16; ld >= cols is the row stride in elements
 *   rows        >= 0 (0 is a no-op);  cols: multiple of 8, 8 <= cols <= QUEST_MAX_COLS
 *   had_block   n: power of two dividing cols; 1 = no transform (the paper's Hadamard ablation)
 *   bits        b in {1,2,3,4,8}
 *   alpha       clip in RMS units; <= 0 selects the built-in Gaussian-optimal alpha*(b)
 *   outer_trust width of the trust region beyond the clip point in units of T; < 0 selects 1,
 *               which is the paper's mask for every b (Sec. 3.3 "The 1-bit Case" shrinks it at b = 1).
 *               An element is trusted iff |x_h| <= alpha (1 + outer_trust / (L - 1)) rms.
 *   codes       out [rows, cols*cb/8] packed codes c
 *   scales      out [rows] fp32, s = alpha rms / (L - 1)
 *   mask        out [rows, cols/8] bitmap, or NULL when no backward pass will follow
 *   xh_out      out [rows, cols] fp32 Hadamard-domain values x_h, or NULL (NULL in production)
 * Rows whose entries are all zero give s = 0, c = L/2 everywhere and an all-ones mask.  A row that
 * holds an infinity or a NaN gets a non-finite scale and unspecified codes and mask bits; other
 * rows are not affected (the paper defines the projection for finite inputs only; the row's sum of
 * squares is formed in fp32, so a row whose sum of squares exceeds the fp32 range counts as such).
 * x, codes, mask, xh_out must be 16-byte aligned and ld * sizeof(element) a multiple of 16.
 */
quest_status quest_hadamard_quantize(const void *x, quest_dtype dtype, int64_t rows, int64_t cols,
                                     int64_t ld, int32_t had_block, int32_t bits, float alpha,
                                     float outer_trust, uint8_t *codes, float *scales,
                                     uint8_t *mask, float *xh_out, void *stream);

/*
 * Algorithm 1 for both operands of one layer in one call: steps 2 and 3 for the activations x, steps
 * 4 and 5 for the weights w (the same transform, projection and trust mask as
 * quest_hadamard_quantize; x and w share the row length, which is the layer's contraction dimension,
 * the Hadamard block, the bit width and the clip).  Where one kernel covers the shape the two row
 * sets are quantized by a single launch, which is what a QAT step wants: the weights are quantized
 * anew in every step, and their launch, 5632 rows at the 1.6B model's width, is too small to fill
 * the chip by itself.
 *
 *   x, w                [rows_x, ld_x] and [rows_w, ld_w] row-major, both of `dtype`
 *   codes_*, scales_*   outputs as in quest_hadamard_quantize, one set per operand
 *   mask_x, mask_w      trust bitmaps; give both or neither (QUEST_ERR_ARG otherwise)
 *   dtype .. outer_trust as in quest_hadamard_quantize
 * rows_x or rows_w may be 0 (that operand's pointers may then be NULL).  The outputs are identical,
 * bit for bit, to those of two calls of quest_hadamard_quantize.  Same limits, alignment rules and
 * errors; no xh_out.
 */
quest_status quest_hadamard_quantize_pair(const void *x, int64_t rows_x, int64_t ld_x, uint8_t *codes_x,
                                          float *scales_x, uint8_t *mask_x, const void *w, int64_t rows_w,
                                          int64_t ld_w, uint8_t *codes_w, float *scales_w, uint8_t *mask_w,
                                          quest_dtype dtype, int64_t cols, int32_t had_block, int32_t bits,
                                          float alpha, float outer_trust, void *stream);

/*
 * The comparison quantizer of Sec. 4.1 (scale taken from the row's largest magnitude instead of
 * a fit to the value distribution), and with had_block = 1 the no-transform ablation of Sec. 4.3: everything as in
 * quest_hadamard_quantize, except that the grid spans the row's largest magnitude,
 *   a = max_j |x_h[j]|,  k = clamp(floor(x_h (L - 1) / (2 a)), -L/2, L/2 - 1),  scales[r] = a / (L - 1).
 * Nothing is clipped, so every mask bit is 1 (the mask is still written when given).  A zero row
 * gives c = L/2, scale 0.  Same arguments, layouts, limits and errors as quest_hadamard_quantize.
 */
quest_status quest_hadamard_quantize_absmax(const void *x, quest_dtype dtype, int64_t rows,
                                            int64_t cols, int64_t ld, int32_t had_block, int32_t bits,
                                            uint8_t *codes, float *scales, uint8_t *mask,
                                            float *xh_out, void *stream);

/*
 * FP4 variant of the quantizer (Sec. 4.4 "The FP4 Format"): the rounding of Eq. 1 is replaced by
 * rounding to the value set of the 4-bit floating-point format E2M1, {0, .5, 1, 1.5, 2, 3, 4, 6}
 * with a sign, scaled so that 6 sits on the clip alpha * rms:
 *   t = 6 x_h / (alpha rms) clipped to [-6, 6];  code = E2M1(t), nearest value, ties to the even
 *   code, bit 3 = sign of x_h (kept when the magnitude rounds to zero);  scales[r] = alpha rms / 6,
 *   so that xhat_h = scales[r] * value(code);  mask bit = 1 iff |x_h| <= alpha (1 + 1/6) rms
 *   (T = alpha / 6 is the largest half-interval of the grid).
 * alpha <= 0 selects the built-in alpha*_FP4.  Codes are packed two per byte, low nibble first:
 * the operand layout of the FP4 matrix instructions.  A zero row gives code 0, scale 0, mask 1.
 * Other arguments, layouts, limits and errors as quest_hadamard_quantize.
 */
quest_status quest_hadamard_quantize_fp4(const void *x, quest_dtype dtype, int64_t rows, int64_t cols,
                                         int64_t ld, int32_t had_block, float alpha, uint8_t *codes,
                                         float *scales, uint8_t *mask, float *xh_out, void *stream);

/*
 * quest_hadamard_quantize_fp4 for both operands of one layer in one call (Sec. 4.4 on Algorithm 1,
 * steps 2-5): arguments, single launch, bit-identical outputs and errors as
 * quest_hadamard_quantize_pair, with the E2M1 grid, codes and scales of quest_hadamard_quantize_fp4.
 */
quest_status quest_hadamard_quantize_fp4_pair(const void *x, int64_t rows_x, int64_t ld_x, uint8_t *codes_x,
                                              float *scales_x, uint8_t *mask_x, const void *w,
                                              int64_t rows_w, int64_t ld_w, uint8_t *codes_w,
                                              float *scales_w, uint8_t *mask_w, quest_dtype dtype,
                                              int64_t cols, int32_t had_block, float alpha, void *stream);

/* Host: the built-in Gaussian-MSE-optimal clip for the scaled E2M1 grid (Sec. 4.4). */
float quest_alpha_star_fp4(void);

/*
 * Algorithm 1, the matmul y = xhat_h what_h^T, run on the integer codes (Sec. 5 "Kernel
 * Overview", stage 3): acc[m, n] = sum_k u_a[m, k] u_b[n, k] exactly in int32, then
 * y[m, n] = bf16(float(acc[m, n]) * a_scales[m] * b_scales[n]).
 *
 *   a_codes  [M, K*cb/8] activation codes, a_scales [M];  b_codes [N, K*cb/8] weight codes,
 *            b_scales [N]; both operands K-contiguous (row-major weight), produced by
 *            quest_hadamard_quantize with the same had_block and the same bits
 *   bits     1, 2, 3 or 4 (u fits a signed byte); K: multiple of 64, 64 <= K <= 65536;
 *            M, N <= 2^22 and max(M, N) * K / 2 < 2^32 (QUEST_ERR_SHAPE otherwise)
 *   y        out bf16 [M, ld_y], ld_y >= N (row stride in elements);  may be NULL if acc_out is given
 *   acc_out  out int32 [M, N] raw accumulators, or NULL (NULL in production)
 *   workspace, workspace_bytes   scratch for bits = 1 or 2 with M, N >= 128 and K a multiple of 128:
 *            both operands are first re-coded as 4-bit codes of the same odd integers
 *            ((M + N) * K / 2 bytes, see quest_lowbit_gemm_workspace_bytes) and multiplied by the
 *            4-bit kernels.  NULL is allowed: the narrow containers are then multiplied directly by
 *            a slower kernel, with the same result.  Given but too small: QUEST_ERR_ARG.  Unused
 *            (may be NULL, 0) for bits = 3 or 4.
 * M = 0 or N = 0 is a no-op.  Code pointers must be 16-byte aligned.
 */
quest_status quest_lowbit_gemm(const uint8_t *a_codes, const float *a_scales, int64_t M,
                               const uint8_t *b_codes, const float *b_scales, int64_t N, int64_t K,
                               int32_t bits, void *y, int64_t ld_y, int32_t *acc_out, void *workspace,
                               int64_t workspace_bytes, void *stream);

/* Host: scratch bytes the fast path of quest_lowbit_gemm uses for this shape (0: none; -1: the
 * shape or bit width is not accepted). */
int64_t quest_lowbit_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int32_t bits);

/*
 * quest_lowbit_gemm for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and errors as quest_lowbit_gemm; the scratch of the 1- and 2-bit fast path is a buffer of
 * QUEST_STATIC_SCRATCH_BYTES built into the library (one per GPU, held until the process ends), so
 * the call allocates and frees nothing.  A shape whose scratch
 * (quest_lowbit_gemm_workspace_bytes: (M + N) * K / 2 bytes) exceeds that size is rejected with
 * QUEST_ERR_SCRATCH and nothing is launched; bits = 3 or 4 need no scratch and are never rejected
 * for it.  All calls on one GPU share the buffer: calls that overlap in time on one GPU (two
 * streams, or two host threads) race and must be serialised by the caller; calls on one stream are
 * ordered.  The buffer keeps the last call's contents; every byte a call reads it has written before,
 * so nothing needs clearing.  The buffer's address is looked up on the first call on a device (or
 * by quest_init).
 */
quest_status quest_lowbit_gemm_static(const uint8_t *a_codes, const float *a_scales, int64_t M,
                                      const uint8_t *b_codes, const float *b_scales, int64_t N, int64_t K,
                                      int32_t bits, void *y, int64_t ld_y, int32_t *acc_out, void *stream);

/*
 * The matmul of Algorithm 1 for the FP4 variant (Sec. 4.4), run on the E2M1 codes by the FP4 matrix
 * instructions:  acc[m, n] = sum_k v_a[m, k] v_b[n, k] (v = signed E2M1 value of a code; the sum is
 * a multiple of 1/4 and exact in fp32 for K <= 65536),  y = bf16((acc * a_scales[m]) * b_scales[n]).
 *   a_codes [M, K/2], b_codes [N, K/2], scales from quest_hadamard_quantize_fp4
 *   y        out bf16 [M, ld_y], ld_y >= N;  may be NULL if acc_out is given
 *   acc_out  out fp32 [M, N] raw accumulators, or NULL (NULL in production)
 * K a multiple of 128, 128 <= K <= 65536; M = 0 or N = 0 is a no-op; code pointers 16-byte aligned.
 */
quest_status quest_lowbit_gemm_fp4(const uint8_t *a_codes, const float *a_scales, int64_t M,
                                   const uint8_t *b_codes, const float *b_scales, int64_t N, int64_t K,
                                   void *y, int64_t ld_y, float *acc_out, void *stream);

/*
 * Algorithm 2, the two masked inverse transforms: out = IHT(M (.) g) (Sec. 3.2 "Trust Estimators
 * for the Hadamard Projection").  The normalised Sylvester transform is its own inverse.
 *
 *   g        [rows, cols] gradient w.r.t. the quantized tensor in the Hadamard domain
 *   mask     [rows, cols/8] bitmap from quest_hadamard_quantize; NULL = all trusted (plain STE)
 *   out      [rows, cols]; g_dtype / out_dtype: f32 or bf16 (bf16 rounds to nearest even)
 * Same shape limits and alignment rules as quest_hadamard_quantize (ld = cols).
 */
quest_status quest_trust_backward(const void *g, quest_dtype g_dtype, const uint8_t *mask,
                                  int64_t rows, int64_t cols, int32_t had_block, void *out,
                                  quest_dtype out_dtype, void *stream);

/*
 * Both masked inverse transforms that end Algorithm 2 (the last two steps of its backward pass: the
 * input gradient from G_x and M_x, the weight gradient from G_w and M_w) in one call.  The two
 * Hadamard-domain gradients share the row length (the layer's contraction dimension), the block and
 * the dtypes; where one kernel covers the shape a single launch transforms both row sets (the
 * weight gradient's rows alone do not fill the chip).
 *
 *   g_x, mask_x, out_x   [rows_x, cols], [rows_x, cols/8] or NULL, [rows_x, cols]
 *   g_w, mask_w, out_w   [rows_w, cols], [rows_w, cols/8] or NULL, [rows_w, cols]
 *   g_dtype .. out_dtype as in quest_trust_backward
 * Give both masks or neither (QUEST_ERR_ARG otherwise).  rows_x or rows_w may be 0 (that gradient's
 * pointers may then be NULL).  The outputs are identical, bit for bit, to those of two calls of
 * quest_trust_backward; same limits, alignment rules and errors.
 */
quest_status quest_trust_backward_pair(const void *g_x, const uint8_t *mask_x, int64_t rows_x, void *out_x,
                                       const void *g_w, const uint8_t *mask_w, int64_t rows_w, void *out_w,
                                       quest_dtype g_dtype, int64_t cols, int32_t had_block,
                                       quest_dtype out_dtype, void *stream);

/*
 * Algorithm 2, the two 16-bit matmuls against a code-packed operand whose value is
 * bf16(s * u) (the paper runs the backward multiplications in 16-bit precision, Sec. 3.3):
 *   which = 0:  out[M, K] = dy[M, N] * what_h[N, K]      (q = weight codes [N, K*cb/8], scales [N])
 *   which = 1:  out[N, K] = dy[M, N]^T * xhat_h[M, K]    (q = activation codes [M, K*cb/8], scales [M])
 *   dy bf16 [M, N] row-major, out bf16, fp32 accumulation.  bits in {1,2,3,4}.
 *   M, N, K multiples of 64, each at most 2^22.
 *   workspace, workspace_bytes   scratch of quest_grad_gemm_workspace_bytes(which, M, N, K) bytes:
 *            when the output is at least 128 x 128 the call first expands the packed operand to bf16
 *            and, if the tiles do not fill the GPU's compute units evenly, leaves partial tiles there
 *            that a second pass sums in a fixed order.  Missing or too small: QUEST_ERR_ARG.  Smaller
 *            outputs need none (the query returns 0).
 */
quest_status quest_grad_gemm(int32_t which, const void *dy, const uint8_t *q_codes,
                             const float *q_scales, int32_t bits, int64_t M, int64_t N, int64_t K,
                             void *out, void *workspace, int64_t workspace_bytes, void *stream);

/* Host: scratch bytes quest_grad_gemm needs for this shape on the current device (it depends on the
 * device's number of compute units; 256 are assumed when no device is available).  -1: shape not
 * accepted. */
int64_t quest_grad_gemm_workspace_bytes(int32_t which, int64_t M, int64_t N, int64_t K);

/*
 * quest_grad_gemm for operands quantized by quest_hadamard_quantize_fp4: the code-packed operand's
 * value is bf16(s * v), v the signed E2M1 value of its code (the backward pass of the FP4 variant,
 * Sec. 4.4, is Algorithm 2 unchanged).  which = 0 or 1 as there.  M, N, K multiples of 64 and the
 * output at least 128 x 128 (QUEST_ERR_SHAPE otherwise).  Workspace as for quest_grad_gemm, sized by
 * quest_grad_gemm_fp4_workspace_bytes.
 */
quest_status quest_grad_gemm_fp4(int32_t which, const void *dy, const uint8_t *q_codes,
                                 const float *q_scales, int64_t M, int64_t N, int64_t K, void *out,
                                 void *workspace, int64_t workspace_bytes, void *stream);

int64_t quest_grad_gemm_fp4_workspace_bytes(int32_t which, int64_t M, int64_t N, int64_t K);

/*
 * Weight-only forward product (Sec. 4.4 "Weight-only quantization": 16-bit activations against
 * 1..4-bit weights):  y[M, N] = x[M, K] * what_h^T,  what_h[n, k] = bf16(s_w[n] * u_w[n, k]).
 *   x        bf16 [M, K] row-major (the activations in the domain the weights were quantized in:
 *            for Hadamard-domain weight codes, x_h = HT(x), which quest_trust_backward computes
 *            when called without a mask)
 *   w_codes  [N, K*cb/8], w_scales [N] from either quantizer entry point;  bits in {1,2,3,4}
 *   y        out bf16 [M, N] row-major, fp32 accumulation on the bf16 matrix cores
 * M, N, K multiples of 64, M and N at least 128, M*N < 2^31 (QUEST_ERR_SHAPE otherwise).
 * Workspace as for quest_grad_gemm, sized by quest_weight_only_gemm_workspace_bytes.
 */
quest_status quest_weight_only_gemm(const void *x, const uint8_t *w_codes, const float *w_scales,
                                    int32_t bits, int64_t M, int64_t N, int64_t K, void *y,
                                    void *workspace, int64_t workspace_bytes, void *stream);

int64_t quest_weight_only_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);

/*
 * Host: optional set-up for the current device (call once per device, from any thread, before
 * capturing graphs): raises the dynamic-LDS limit of every kernel that needs it, which the enqueue
 * calls otherwise do on first use.  Allocates nothing.  QUEST_ERR_LAUNCH if the runtime refuses.
 */
quest_status quest_init(void);

/* Host: the built-in Gaussian-MSE-optimal clip alpha*(bits) (Sec. 3.1); 0 for unsupported bits. */
float quest_alpha_star(int32_t bits);

/* Host: container width in bits for a b-bit code; 0 for unsupported bits. */
int32_t quest_container_bits(int32_t bits);

/* Host: static description of a status code. */
const char *quest_status_string(quest_status status);

#ifdef __cplusplus
}
#endif
#endif /* QUEST_H */
