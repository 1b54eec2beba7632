/*
 * librtn -- the inference hot path of RTN (Reparameterized Ternary Network,
 * arxiv 1912.02057) for AMD MI355X (gfx950), behind a plain C ABI.
 *
 *   fp32 tensor --ternarize+pack--> ternary codes (+ side sums)
 *   codes x codes --ternary contraction--> int32 accumulators D
 *   D, side sums, scale/offset --four-term reparameterization--> fp32 output
 *
 * Notation.  t_a, t_w in {-1,0,+1} are the paper's fixed ternary activation
 * A^t and weight W^t; the reparameterized values are alpha_a*t_a + beta_a
 * (Eq.4: gamma, beta) and alpha_w*t_w + beta_w (the paper has alpha only; a
 * NULL beta_w means 0 and gives Eq.9 verbatim).  K = c*k*k is the length of
 * one dot product (Section "Methodology").
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The
 *     library never allocates, frees or keeps them.  Scratch memory, where an
 *     entry point needs it, is a caller buffer sized by the matching
 *     *_workspace_bytes() query.
 *   - Parameters with a granularity switch (thresholds, alpha, beta): with
 *     RTN_SCALAR the pointer is a HOST pointer to one float (read during the
 *     call); with RTN_VECTOR it is a DEVICE pointer to one float per row /
 *     column / channel as stated.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued asynchronously on it; nothing synchronizes.
 *   - Return value: RTN_OK or a negative rtn_status.  All argument checks run
 *     before anything is launched, so a rejected call has no side effects and
 *     needs no GPU.  RTN_ERR_HIP means a launch failed; rtn_last_hip_error()
 *     then returns the hipError_t as an int.
 *   - Code tensors must be 16-byte aligned; fp32/int32 tensors 4-byte aligned.
 *   - Sizes: every dimension and the products noted per function must be
 *     below 2^31; K (padded) must be at most 2^22, so D is exact in int32 and fp32.
 */
#ifndef RTN_H
#define RTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RTN_OK = 0,
    RTN_ERR_NULL = -1,        /* a required pointer is NULL */
    RTN_ERR_SHAPE = -2,       /* non-positive or too large dimension, lo > hi ... */
    RTN_ERR_ALIGN = -3,       /* pointer alignment */
    RTN_ERR_UNSUPPORTED = -4, /* format/path/granularity/kernel size outside the list */
    RTN_ERR_WORKSPACE = -5,   /* workspace NULL or too small */
    RTN_ERR_HIP = -6          /* kernel launch failed */
} rtn_status;

/* Storage of ternary codes.
 * RTN_CODE_I8: one signed byte per element holding t itself.
 * RTN_CODE_BITPLANE: the 2-bit encoding of Table 1 split into its two bit
 *   planes (W_1/A_1 = "non-zero" bits, W_2/A_2 = sign bits, 1 <=> +1; Section
 *   "Efficient Computation Pattern").  Zero is always written as 00.  A plane
 *   is uint64 words; bit j (LSB = 0) of word w of a row is element 64*w + j.
 *   The buffer holds the whole mask plane [rows][Kpad/64] followed by the
 *   whole sign plane [rows][Kpad/64].
 * In both formats a row holds Kpad = rtn_padded_k(K) elements (K rounded up
 * to a multiple of 64); the padding is code 0.
 * RTN_CODE_FP4: one 4-bit float (E2M1: sign, 2 exponent bits, 1 mantissa bit)
 *   per element, holding t itself: 0 -> 0x0, +1 -> 0x2, -1 -> 0xA; two elements
 *   per byte, element 2j in the low nibble of byte j of the row.  This is the
 *   storage of the primary path on MI355X: -1, 0, +1 are exact in E2M1, so the
 *   FP4 matrix cores (twice the int8 rate, half the operand bytes) form the
 *   ternary dot product exactly.  A row holds rtn_padded_k_format(RTN_CODE_FP4,
 *   K) elements (K rounded up to a multiple of 128, i.e. whole 64-byte steps);
 *   the padding is code 0.  The same ternary values as the paper's 2-bit code
 *   of Table 1, in the 4-bit form this hardware multiplies natively.        */
typedef enum { RTN_CODE_I8 = 0, RTN_CODE_BITPLANE = 1, RTN_CODE_FP4 = 2 } rtn_code_format;
typedef enum { RTN_SCALAR = 0, RTN_VECTOR = 1 } rtn_gran;
typedef enum { RTN_ROWS_K_CONTIG = 0, RTN_NCHW = 1 } rtn_layout;

/* What the padded border of a convolution holds (the paper does not discuss
 * padding).  RTN_PAD_TRUE_ZERO: the reparameterized activation alpha_a*t+beta_a
 * is padded with the value 0, as a framework convolution of it would be; a
 * padded tap then contributes nothing, so the sum of t_w and the count K of
 * Eq.9's constant run over in-bounds taps only and differ per border pixel.
 * RTN_PAD_CODE_ZERO: the code tensor is padded with code 0, i.e. the value
 * beta_a; Eq.9's C is then one constant per filter.                          */
typedef enum { RTN_PAD_TRUE_ZERO = 0, RTN_PAD_CODE_ZERO = 1 } rtn_pad_mode;

/* Contraction strategy.  MFMA_I8: int8 matrix cores on RTN_CODE_I8 codes.
 * POPC: Eq.8 (AND / XOR / popcount) on RTN_CODE_BITPLANE codes.
 * MFMA_FP4: FP4 matrix cores with fp32 accumulation on RTN_CODE_FP4 codes (every
 * product is exact and the sums are integers below 2^24, so D is the same integer).
 * AUTO picks the one that matches the code format.                           */
typedef enum { RTN_PATH_AUTO = 0, RTN_PATH_MFMA_I8 = 1, RTN_PATH_POPC = 2, RTN_PATH_MFMA_FP4 = 3 } rtn_path;

/* Four-term reparameterization applied to an accumulator D (Eq.9 with a weight
 * offset added; phi = ReLU; the BN affine follows ReLU in RTN's layer order):
 *   y = alpha_a*alpha_w*D + alpha_a*beta_w*Sa + beta_a*alpha_w*Sw + Kv*beta_a*beta_w
 *   if relu:      y = max(y, 0)
 *   if bn_scale:  y = bn_scale[n]*y + bn_shift[n]
 * evaluated in fp64 and rounded once to fp32.
 * GEMM:  gran_a SCALAR or VECTOR over the M rows; gran_w SCALAR or VECTOR over
 *        the N columns; sum_ta[M] = row sums of t_a, sum_tw[N] = row sums of
 *        t_w; Kv = K.
 * conv:  gran_a must be SCALAR (the paper's factors are layer-wise; a factor
 *        per input channel cannot leave the integer sum); gran_w SCALAR or
 *        VECTOR over the O filters; sum_ta[Nb][H][W] = channel sums of the
 *        input codes at each input pixel; sum_tw[O][KH][KW] = channel sums of
 *        the weight codes at each tap (both as written by rtn_ternarize_pack
 *        with RTN_NCHW).  The library forms Sa, Sw and Kv per output pixel
 *        from them according to the pad mode.
 * beta_w, bn_scale, bn_shift may be NULL (0, 1, 0); bn_* are DEVICE pointers
 * with one entry per output column / channel.                                */
typedef struct {
    const float *alpha_a, *beta_a;
    rtn_gran gran_a;
    const float *alpha_w, *beta_w;
    rtn_gran gran_w;
    const int32_t *sum_ta, *sum_tw;
    int relu;
    const float *bn_scale, *bn_shift;
} rtn_epilogue;

const char *rtn_status_string(int status);
int rtn_last_hip_error(void);

/* Tuning and testing aid for the matrix-core kernels.  The output tile a
 * 256-thread block owns is BP x BQ (BP along M for the GEMM and along O for the
 * conv; BQ along N resp. along output pixels).  Index: 0 = 64x64, 1 = 128x128,
 * 2 = 256x256, 3 = 64x256, 4 = 128x256, 5 = 256x128, 6 = 64x128, 7 = 64x256
 * with a two-stage operand ring; 8 .. 13 repeat 128x128, 64x256, 64x128, 64x64,
 * 128x128 and 128x256 with other ring depths and register budgets; 14 .. 19 are
 * conv variants that keep a tile's run of input pixels in LDS (stride 1, centred
 * window, 64 or 128 padded channels: 64x256 twice, 64x128 twice, 128x128,
 * 128x256; any other problem runs the plain tile of that size); -1 (default)
 * lets the library choose from the problem shape.  Every configuration computes the same
 * result.  The setting is process-wide and not thread-safe.
 * Returns RTN_ERR_UNSUPPORTED for an index outside -1 .. rtn_num_tile_configs()-1. */
int rtn_num_tile_configs(void);
int rtn_set_tile_config(int index);

/* K rounded up to the row length of a code tensor (a multiple of 64). */
int64_t rtn_padded_k(int64_t K);
/* The same per format: 128 for RTN_CODE_FP4, 64 otherwise (0 on invalid arguments). */
int64_t rtn_padded_k_format(rtn_code_format fmt, int64_t K);
/* Bytes of a code tensor of `rows` rows of K elements in format `fmt`
 * (0 on invalid arguments). */
size_t rtn_codes_bytes(rtn_code_format fmt, int64_t rows, int64_t K);

/* Ternarize + pack (Eq.1 / Eq.3, Table 1).
 *   t = (x > hi) - (x < lo), compared on the stored fp32 value with strict
 *   inequalities (x == threshold gives 0, NaN gives 0).  Eq.1 is lo = -Delta,
 *   hi = +Delta; Eq.3's BN-folded form is lo = -(0.5+b)/k, hi = (0.5-b)/k,
 *   computed by the caller.  lo <= hi is required for RTN_SCALAR thresholds.
 * layout RTN_ROWS_K_CONTIG: x is [d0 = rows][d1 = K] row-major (d2 = d3 = 1).
 *   codes: [rows][Kpad]; sum_t[rows] = sum of t over the row.
 *   RTN_VECTOR thresholds: one (lo, hi) per row.
 * layout RTN_NCHW: x is [d0 = N][d1 = C][d2 = H][d3 = W] (activations), or
 *   [O][I][KH][KW] (weights).  codes are written channel-innermost,
 *   [N][H][W][Cpad]; sum_t[N][H][W] = sum of t over the channels of a pixel
 *   (for weights: per filter and tap).  RTN_VECTOR thresholds: one (lo, hi)
 *   per d0 index (per filter).  RTN_CODE_I8 and RTN_CODE_FP4 need C <= 2048 in
 *   this layout; with RTN_CODE_FP4 a row / pixel is Kpad / 2 bytes.
 * sum_t may be NULL.  d0*d2*d3 and d0*d1*d2*d3 must be below 2^31 resp. 2^40. */
int rtn_ternarize_pack(const float *x, rtn_layout layout, int64_t d0, int64_t d1, int64_t d2,
                       int64_t d3, const float *thr_lo, const float *thr_hi, rtn_gran thr_gran,
                       rtn_code_format fmt, void *codes, int32_t *sum_t, void *stream);

/* Ternary contraction D[m][n] = sum_k t_a[m][k]*t_w[n][k] (the dot product
 * W^t (x) A^t of Eq.8/Eq.9), optionally followed by the fused epilogue.
 *   a_codes: [M][Kpad], w_codes: [N][Kpad] in format `fmt` (Kpad per format).
 *   acc_out: int32 [M][N] row-major, or NULL.
 *   ep + y_out: fp32 [M][N] row-major through the four-term formula, or both
 *   NULL.  At least one of acc_out / (ep, y_out) must be given.
 *   workspace: unused by the current kernels (pass NULL, 0).                 */
int rtn_ternary_gemm(rtn_code_format fmt, rtn_path path, const void *a_codes, const void *w_codes,
                     int64_t M, int64_t N, int64_t K, int32_t *acc_out, const rtn_epilogue *ep,
                     float *y_out, void *workspace, size_t workspace_bytes, void *stream);

/* Ternary 2-D convolution as an implicit GEMM (im2col view of the footnote in
 * Section "Methodology"; the patch matrix is never materialised):
 *   M = Nb*OH*OW, N = O, K = KH*KW*C, cross-correlation,
 *   ih = oh*stride - pad + kh, iw = ow*stride - pad + kw,
 *   OH = (H + 2*pad - KH)/stride + 1; a tap outside the image adds 0 to D.
 *   a_codes: [Nb][H][W][Cpad]; w_codes: [O][KH][KW][Cpad], RTN_CODE_I8 or
 *   RTN_CODE_FP4 (Cpad = rtn_padded_k_format(fmt, C), both tensors in `fmt`).
 *   acc_out: int32 [Nb][O][OH][OW] or NULL; y_out: fp32 [Nb][O][OH][OW] (NCHW).
 *   KH, KW in 1..7, stride in 1..64, 0 <= pad < min(KH, KW), pad <= 2.
 *   workspace (needed when an epilogue is given): the table written by
 *   rtn_conv2d_prepare_constants() for the same filters, pad and epilogue
 *   parameters (alpha, beta and the BN affine of `ep` are taken from the
 *   table; of `ep` itself the call reads only relu -- the sum of t_a over a
 *   pixel's window is formed from the codes inside the kernel, so ep->sum_ta
 *   may be NULL here); it is only read here, so one prepared table
 *   serves any number of calls, batch sizes and image sizes.  16-byte aligned.
 *   Nb*H*W and Nb*OH*OW must be below 2^31.                                  */
size_t rtn_conv2d_workspace_bytes(int64_t O, int KH, int KW, int pad);
/* Weight-side preparation of the conv epilogue (offline, once per layer): fills
 * `workspace` (>= rtn_conv2d_workspace_bytes(O, KH, KW, pad) bytes, 16-byte
 * aligned) with the per-filter factors of the epilogue (alpha_a*alpha_w,
 * alpha_a*beta_w, BN scale and shift) and Eq.9's pre-stored constant
 * C = beta_a*alpha_w*Sw + Kv*beta_a*beta_w for every filter and every border
 * class of output pixels (the in-bounds tap rectangle decides which taps enter
 * Sw and Kv).  Reads ep->sum_tw (the per-tap sums [O][KH][KW]) and every
 * scale, offset and BN parameter of `ep`; ep->sum_ta may be NULL.  C is the
 * number of input channels.                                                  */
int rtn_conv2d_prepare_constants(int64_t C, int64_t O, int KH, int KW, int pad, const rtn_epilogue *ep,
                                 void *workspace, size_t workspace_bytes, void *stream);
int rtn_ternary_conv2d_implicit_gemm(rtn_code_format fmt, rtn_path path, const void *a_codes,
                                     const void *w_codes, int64_t Nb, int64_t C, int64_t H,
                                     int64_t W, int64_t O, int KH, int KW, int stride, int pad,
                                     rtn_pad_mode pad_mode, int32_t *acc_out,
                                     const rtn_epilogue *ep, float *y_out, void *workspace,
                                     size_t workspace_bytes, void *stream);

/* The same convolution with a ternarizing epilogue: the activation of Eq.9 is
 * handed to the next ternary layer as codes, never as fp32.  RTN's layer order
 * is conv -> ReLU -> BN -> ternarize, so with z the fp32 value the epilogue of
 * rtn_ternary_conv2d_implicit_gemm would have stored for output channel o,
 *   t = (z > thr_hi[o]) - (z < thr_lo[o])            (Eq.1, strict, NaN -> 0)
 * is written channel-innermost as the next layer's input, in the format `fmt` of
 * the inputs (RTN_CODE_I8 or RTN_CODE_FP4):
 *   codes_out: [Nb][OH][OW][rtn_padded_k_format(fmt, O)] codes (one byte each, or
 *   two per byte), 16-byte aligned; the padding channels are written as code 0.
 * Thresholds: RTN_SCALAR (host pointers, lo <= hi) or RTN_VECTOR (device, one
 * pair per output channel).  The per-channel form is Eq.3: a BN affine k*z + b
 * with k > 0 need not be applied (leave ep->bn_scale NULL) when the caller
 * passes hi = (0.5-b)/k, lo = -(0.5+b)/k; with ReLU and a positive scale the
 * comparison is Eq.10's thresholded ReLU on the integer sum.  Pixel sums of
 * the written codes are not produced: the conv entry points form them from the
 * codes.
 * Block-tail form (the last conv of a residual block, whose output meets the
 * shortcut before the next block ternarizes it): with `residual` (fp32
 * [Nb][O][OH][OW], nullable) and `relu_out`,
 *   s = z + residual   (one fp32 add on the rounded z, as a separate add kernel
 *                       would compute it),     s = max(s, 0) if relu_out,
 * and s takes the place of z in the comparison.  y_out (fp32 [Nb][O][OH][OW],
 * nullable) receives the value that was ternarized (z, or s), for the next
 * block's shortcut.  residual and y_out may be the same buffer.
 * ep, workspace and every other argument as for
 * rtn_ternary_conv2d_implicit_gemm (ep->sum_ta may be NULL); Nb*OH*OW*
 * rtn_padded_k(O) must be below 2^40.                                        */
int rtn_ternary_conv2d_ternarize(rtn_code_format fmt, rtn_path path, const void *a_codes,
                                 const void *w_codes, int64_t Nb, int64_t C, int64_t H, int64_t W,
                                 int64_t O, int KH, int KW, int stride, int pad,
                                 rtn_pad_mode pad_mode, const rtn_epilogue *ep,
                                 const float *residual, int relu_out, const float *thr_lo,
                                 const float *thr_hi, rtn_gran thr_gran, float *y_out,
                                 void *codes_out, void *workspace, size_t workspace_bytes,
                                 void *stream);

/* Weight-only ternary layer (the 2-bit-weight / 32-bit-activation rows of the
 * paper's ImageNet table): ternary weights alpha_w * t_w as everywhere else
 * (Section "Weight Ternarization": a scale, no offset), activations left in fp32:
 *   y[m][n] = alpha_w[n] * sum_k x[m][k] * t_w[n][k];  then ReLU if relu; then
 *   bn_scale[n]*y + bn_shift[n] if bn_scale (both nullable, DEVICE vectors).
 *   x: fp32 [M][K] row-major; w_codes: RTN_CODE_I8 [N][rtn_padded_k(K)] as written
 *   by rtn_ternarize_pack; alpha_w: RTN_SCALAR (host) or RTN_VECTOR over N (device);
 *   y_out: fp32 [M][N].
 * On the matrix cores each fp32 activation is split exactly into three bf16 terms
 * (x = hi + mid + lo); the products with -1, 0, +1 are exact and are accumulated in
 * fp32, so the result differs from the exactly rounded one only by the fp32
 * accumulation of 3K terms: |y - y_exact| <= 3K * 2^-24 * alpha_w * sum_k |x[m][k]| in
 * the worst case, about sqrt(3K) * 2^-24 of that sum typically.  x must be finite.
 * workspace: rtn_weight_gemm_workspace_bytes(M, N, K) bytes, 16-byte aligned (holds
 * the split activations and the weights as bf16; overwritten by every call).    */
size_t rtn_weight_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
int rtn_ternary_weight_gemm(const float *x, const void *w_codes, int64_t M, int64_t N, int64_t K,
                            const float *alpha_w, rtn_gran gran_w, int relu, const float *bn_scale,
                            const float *bn_shift, float *y_out, void *workspace,
                            size_t workspace_bytes, void *stream);

/* conv form of the weight-only ternary layer: x fp32 [Nb][C][H][W], w_codes
 * RTN_CODE_I8 [O][KH][KW][rtn_padded_k(C)] as written by rtn_ternarize_pack with
 * RTN_NCHW, zero padding (a padded tap adds nothing), geometry limits as for
 * rtn_ternary_conv2d_implicit_gemm:
 *   y[n][o][oh][ow] = alpha_w[o] * sum over in-bounds (c, kh, kw) of x * t_w,
 * then ReLU / BN affine as above; y_out fp32 [Nb][O][OH][OW].  Same exact split of
 * the activations and the same error bound with K = C*KH*KW.  workspace:
 * rtn_weight_conv2d_workspace_bytes(...) bytes, 16-byte aligned, overwritten by
 * every call.                                                                  */
size_t rtn_weight_conv2d_workspace_bytes(int64_t Nb, int64_t C, int64_t H, int64_t W, int64_t O, int KH,
                                         int KW, int pad);
int rtn_ternary_weight_conv2d(const float *x, const void *w_codes, int64_t Nb, int64_t C, int64_t H,
                              int64_t W, int64_t O, int KH, int KW, int stride, int pad,
                              const float *alpha_w, rtn_gran gran_w, int relu, const float *bn_scale,
                              const float *bn_shift, float *y_out, void *workspace,
                              size_t workspace_bytes, void *stream);

/* Weight side of the weight-only layer, done once per layer and off the timed path
 * (the offline preparation of the weights the paper's "Inference" paragraph describes:
 * everything that depends only on the trained filters is stored ahead of time).
 *   rtn_weight_gemm_prepare: the codes [N][rtn_padded_k(K)] as bf16 values.
 *   rtn_weight_conv2d_prepare: the codes [O][KH][KW][rtn_padded_k(C)] as bf16 values,
 *   then the per-filter epilogue table (alpha_w and the BN affine; nullable BN as above).
 * prepared: DEVICE, 16-byte aligned, at least rtn_weight_*_prepared_bytes(...) bytes;
 * it is only read by the *_prepared calls below, so one buffer serves any number of
 * calls, batch sizes and image sizes.  Those calls compute exactly what
 * rtn_ternary_weight_gemm / rtn_ternary_weight_conv2d compute (same kernels, same
 * bits); their workspace (same size functions as above) then holds only the split
 * activations.  The conv takes alpha_w and the BN affine from the prepared table. */
size_t rtn_weight_gemm_prepared_bytes(int64_t N, int64_t K);
int rtn_weight_gemm_prepare(const void *w_codes, int64_t N, int64_t K, void *prepared,
                            size_t prepared_bytes, void *stream);
int rtn_ternary_weight_gemm_prepared(const float *x, const void *prepared, int64_t M, int64_t N,
                                     int64_t K, const float *alpha_w, rtn_gran gran_w, int relu,
                                     const float *bn_scale, const float *bn_shift, float *y_out,
                                     void *workspace, size_t workspace_bytes, void *stream);
size_t rtn_weight_conv2d_prepared_bytes(int64_t C, int64_t O, int KH, int KW, int pad);
int rtn_weight_conv2d_prepare(const void *w_codes, int64_t C, int64_t O, int KH, int KW, int pad,
                              const float *alpha_w, rtn_gran gran_w, const float *bn_scale,
                              const float *bn_shift, void *prepared, size_t prepared_bytes,
                              void *stream);
int rtn_ternary_weight_conv2d_prepared(const float *x, const void *prepared, int64_t Nb, int64_t C,
                                       int64_t H, int64_t W, int64_t O, int KH, int KW, int stride,
                                       int pad, int relu, float *y_out, void *workspace,
                                       size_t workspace_bytes, void *stream);

/* Backward of the reparameterized ternary activation Abar^t = gamma*Q(Abar) + beta
 * (Section "Backward Update in Reparameterized Ternarization"), for n elements:
 *   grad_gamma_beta[0] = sum_i t_i * g_i,  grad_gamma_beta[1] = sum_i g_i      (Eq.6)
 *   grad_in[i] = gamma * g_i if |a_i| <= 1, else 0                            (Eq.7)
 * with t = (a > thr_hi) - (a < thr_lo) as in rtn_ternarize_pack and g = grad_out.
 * a, grad_out, grad_in (nullable): DEVICE fp32 [n]; thr_lo, thr_hi, gamma: HOST
 * floats; grad_gamma_beta: DEVICE double[2], overwritten.  The sums are formed in
 * double, per 16384-element block and then in block order, so they are reproducible
 * run to run; gamma*g is one fp32 product.  workspace:
 * rtn_activation_backward_workspace_bytes(n) bytes, 8-byte aligned.             */
size_t rtn_activation_backward_workspace_bytes(int64_t n);
int rtn_activation_backward(const float *a, const float *grad_out, int64_t n, const float *thr_lo,
                            const float *thr_hi, const float *gamma, float *grad_in,
                            double *grad_gamma_beta, void *workspace, size_t workspace_bytes,
                            void *stream);

/* rtn_activation_backward for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels, results and argument rules, but the per-block partial sums go to a fixed
 * 1 MiB array inside the library (one copy per GPU, held until the process ends) instead
 * of a caller workspace.  The call allocates and frees nothing.
 * n must be at most rtn_activation_backward_static_max_n() (2^30 elements), else
 * RTN_ERR_SHAPE.  Every call on a GPU uses that GPU's one array: calls that overlap
 * in time on the same GPU (different streams, different threads) race; calls ordered
 * on one stream do not.  Nothing needs clearing between calls -- each call writes
 * every partial sum it later reads.                                              */
int64_t rtn_activation_backward_static_max_n(void);
int rtn_activation_backward_static(const float *a, const float *grad_out, int64_t n,
                                   const float *thr_lo, const float *thr_hi, const float *gamma,
                                   float *grad_in, double *grad_gamma_beta, void *stream);

/* Backward of the reparameterized ternary weights (Section "Weight Ternarization":
 * Wbar = k_W*W + b_W, W^t = Q(Wbar), Wbar^t = alpha*W^t, the three parameters per
 * filter), for O filters of K weights each.  The paper prints the derivatives for the
 * activation (Eq.6, Eq.7); these are the same rules taken through the weight
 * transform by the chain rule.  With g = grad_out = dL/dWbar^t and
 * d[k] = alpha[o]*g[o][k] if |Wbar[o][k]| <= 1, else 0:
 *   grad_params[3*o + 0] = sum_k t[o][k]*g[o][k]        (dL/dalpha)
 *   grad_params[3*o + 1] = sum_k W[o][k]*d[k]           (dL/dk_W)
 *   grad_params[3*o + 2] = sum_k d[k]                   (dL/db_W)
 *   grad_w[o][k] = k_W[o]*d[k]                          (dL/dW)
 * Wbar is one fp32 fused multiply-add, t = (Wbar > thr_hi) - (Wbar < thr_lo); alpha*g
 * and k_W*d are one fp32 product each; the sums are formed in double in a fixed
 * order (reproducible run to run); a weight outside the clip, a NaN included, adds
 * nothing to the second and third sum.
 * w, grad_out, grad_w (nullable): DEVICE fp32 [O][K] row-major; k_w, b_w, alpha: DEVICE
 * fp32 [O]; thr_lo <= thr_hi: HOST floats; grad_params: DEVICE double [O][3],
 * overwritten.  Needs no workspace.                                            */
int rtn_weight_backward(const float *w, const float *grad_out, int64_t O, int64_t K,
                        const float *thr_lo, const float *thr_hi, const float *k_w, const float *b_w,
                        const float *alpha, float *grad_w, double *grad_params, void *stream);

/* Depthwise ternary convolution (the 3x3 layers of MobileNet, one of the networks of
 * the paper's ImageNet table): channel c of the input is convolved with its own KH x KW
 * ternary filter, so a dot product has K = KH*KW terms, and the four-term formula of
 * rtn_epilogue holds per channel with Sa, Sw, Kv taken over the taps of that channel's
 * window (in-bounds taps only for RTN_PAD_TRUE_ZERO).
 *   a_codes: RTN_CODE_I8 [Nb][H][W][rtn_padded_k(C)], as rtn_ternarize_pack(RTN_NCHW) writes.
 *   w_codes: RTN_CODE_I8 [C][rtn_padded_k(KH*KW)], one row of tap codes (kh*KW + kw) per
 *     channel: rtn_ternarize_pack(RTN_ROWS_K_CONTIG) of the filters [C][KH*KW], which
 *     allows one threshold pair per filter.
 *   acc_out: int32 [Nb][C][OH][OW] or NULL; ep + y_out: fp32 [Nb][C][OH][OW] or both NULL.
 *   ep: alpha_a, beta_a RTN_SCALAR; alpha_w, beta_w (nullable) RTN_SCALAR or RTN_VECTOR
 *   over the C channels; relu, bn_scale, bn_shift as everywhere; sum_ta and sum_tw are
 *   not read (the kernel forms the sums itself).  Geometry limits as for
 *   rtn_ternary_conv2d_implicit_gemm; needs no workspace.                         */
int rtn_ternary_depthwise_conv2d(const void *a_codes, const void *w_codes, int64_t Nb, int64_t C,
                                 int64_t H, int64_t W, int KH, int KW, int stride, int pad,
                                 rtn_pad_mode pad_mode, int32_t *acc_out, const rtn_epilogue *ep,
                                 float *y_out, void *stream);

/* The paper's comparison system: 2-bit quaternary weights and activations, values
 * q in {0,1,2,3} = 2*(1st bit) + (2nd bit) (Table 1, last column), and their dot
 * product D[m][n] = sum_k qa[m][k]*qw[n][k] (Section "How to Compute Dot Product
 * between Two Ternary Vectors", second half; Fig.3(b)).
 * rtn_quaternary_pack: x fp32 [rows][K] row-major (DEVICE) -> codes, with
 *   q = (x > t1) + (x > t2) + (x > t3), strict compares on the stored value, NaN -> 0,
 *   t1 <= t2 <= t3 (the usual uniform 2-bit quantizer of [0,1] is 1/6, 1/2, 5/6).
 *   fmt RTN_CODE_I8: int8 [rows][rtn_padded_k(K)] holding q; RTN_CODE_FP4: E2M1 nibbles
 *   holding q (0x0, 0x2, 0x4, 0x5), [rows][rtn_padded_k_format(FP4, K)/2] bytes;
 *   RTN_CODE_BITPLANE: the plane of first bits of all rows, uint64 [rows][Kpad/64], then
 *   the plane of second bits (bit j of word w = element 64*w + j).  Padding is 0.
 * rtn_quaternary_gemm: a_codes [M] rows, w_codes [N] rows of K codes in `fmt`;
 *   acc_out int32 [M][N].  RTN_CODE_BITPLANE runs the paper's bit-serial pattern on the
 *   vector ALU (four AND + popcount pairs per 64 products, shifts, four adders:
 *   RTN_PATH_POPC); RTN_CODE_I8 / RTN_CODE_FP4 run the matrix cores on the values
 *   (0..3 and their products are exact in both; RTN_PATH_MFMA_I8 / RTN_PATH_MFMA_FP4).
 *   K <= 2^20 so that 9*K is exact in int32 and in fp32.  No epilogue: the comparison
 *   circuit has none.                                                           */
int rtn_quaternary_pack(const float *x, int64_t rows, int64_t K, float t1, float t2, float t3,
                        rtn_code_format fmt, void *codes, void *stream);
int rtn_quaternary_gemm(rtn_code_format fmt, rtn_path path, const void *a_codes, const void *w_codes,
                        int64_t M, int64_t N, int64_t K, int32_t *acc_out, void *stream);

/* Stand-alone epilogue on stored accumulators (Eq.9 generalised, see
 * rtn_epilogue).  GEMM form: acc, y_out are [M][N] row-major.               */
int rtn_epilogue_reparam(const int32_t *acc, int64_t M, int64_t N, int64_t K,
                         const rtn_epilogue *ep, float *y_out, void *stream);
/* conv form: acc, y_out are [Nb][O][OH][OW]; geometry as in
 * rtn_ternary_conv2d_implicit_gemm; needs no workspace.                      */
int rtn_epilogue_reparam_conv2d(const int32_t *acc, int64_t Nb, int64_t C, int64_t H, int64_t W,
                                int64_t O, int KH, int KW, int stride, int pad,
                                rtn_pad_mode pad_mode, const rtn_epilogue *ep, float *y_out,
                                void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RTN_H */
