/*
 * RTN oracle -- TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow, obviously-correct CPU statement of what the reparameterized
 * ternary conv/GEMM path computes (RTN, arxiv 1912.02057).  Only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it.  It shares
 * no code with the HIP library and is never tuned for speed: plain loops,
 * OpenMP on the outermost loop only.
 *
 * Notation (paper <-> here):  A^t = t_a, W^t = t_w (Section "Reparameterized
 * Ternarization"); gamma = alpha_a, beta = beta_a (Eq.4); alpha = alpha_w;
 * a weight offset beta_w is a generalisation (beta_w = 0 gives Eq.9);
 * K = c*k*k is the length of one dot product (Section "Methodology").
 *
 * Every function below has an independent pin in tests/ (marked "not gpu").
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ O1 --
 * Ternarizer.  Eq.1: t = sign(x) if |x| > 0.5 else 0, strict inequality.
 * Eq.3 folds the affine k*x+b into two thresholds on x itself; both are the
 * special cases  t = (x > hi) - (x < lo)  with (lo,hi) = (-D,+D) resp.
 * ((-(0.5+b)/k), (0.5-b)/k).  Comparisons are on the stored fp32 value; no
 * arithmetic touches x.  NaN compares false twice -> 0.
 * x: [rows][cols]; lo/hi: one value (per_row = 0) or one per row.          */
void orc_ternarize(const float *x, int64_t rows, int64_t cols,
                   const float *lo, const float *hi, int per_row, int8_t *t)
{
#pragma omp parallel for
    for (int64_t r = 0; r < rows; ++r) {
        float l = per_row ? lo[r] : lo[0];
        float h = per_row ? hi[r] : hi[0];
        for (int64_t c = 0; c < cols; ++c) {
            float v = x[r * cols + c];
            t[r * cols + c] = (int8_t)((v > h) - (v < l));
        }
    }
}

/* ------------------------------------------------------------------ O2 --
 * Table 1 encoding: 1st bit = "non-zero" (mask), 2nd bit = sign (1 <=> +1).
 * 00 -> 0, 01 -> 0, 10 -> -1, 11 -> +1.  Canonical zero on encode is 00.
 * The table's "2-bit network true value" column (01 -> 1, 10 -> 2) shows the
 * 1st bit is the more significant one, so the 2-bit value is 2*mask + sign. */
void orc_encode_2bit(const int8_t *t, int64_t n, uint8_t *v)
{
    for (int64_t i = 0; i < n; ++i) {
        unsigned m = (t[i] != 0), s = (t[i] == 1);
        v[i] = (uint8_t)(2u * m + s);
    }
}

void orc_decode_2bit(const uint8_t *v, int64_t n, int8_t *t)
{
    for (int64_t i = 0; i < n; ++i) {
        unsigned m = (v[i] >> 1) & 1u, s = v[i] & 1u;
        t[i] = (int8_t)(m ? (s ? 1 : -1) : 0);
    }
}

/* Bit-plane split (W_1, W_2 / A_1, A_2 of the "Efficient Computation
 * Pattern" section): plane 1 holds the first bits, plane 2 the second bits.
 * Word w of a row, bit j (LSB = 0) <-> element k = 64*w + j; rows are padded
 * with zeros up to `words` 64-bit words.  The paper leaves bit order open.  */
void orc_encode_planes(const int8_t *t, int64_t rows, int64_t K, int64_t words,
                       uint64_t *mask, uint64_t *sign)
{
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t w = 0; w < words; ++w) {
            uint64_t m = 0, s = 0;
            for (int j = 0; j < 64; ++j) {
                int64_t k = 64 * w + j;
                if (k >= K) break;
                int8_t v = t[r * K + k];
                if (v != 0) m |= (uint64_t)1 << j;
                if (v == 1) s |= (uint64_t)1 << j;
            }
            mask[r * words + w] = m;
            sign[r * words + w] = s;
        }
    }
}

void orc_decode_planes(const uint64_t *mask, const uint64_t *sign, int64_t rows,
                       int64_t K, int64_t words, int8_t *t)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k) {
            uint64_t m = (mask[r * words + k / 64] >> (k % 64)) & 1u;
            uint64_t s = (sign[r * words + k / 64] >> (k % 64)) & 1u;
            t[r * K + k] = (int8_t)(m ? (s ? 1 : -1) : 0);
        }
}

/* Layout only (no arithmetic): int8 codes, rows padded with code 0 to Kpad. */
/* ----------------------------------------------------------------- O2b --
 * FP4 storage of the same ternary values.  Not the paper's: the paper's code is
 * the 2-bit one of Table 1; this is the 4-bit float of the OCP microscaling
 * formats (E2M1: 1 sign bit s, 2 exponent bits e, 1 mantissa bit m, bias 1, no
 * infinities or NaNs), which MI355X's matrix cores multiply natively:
 *   value = (-1)^s * 2^(e-1) * (1 + m/2)  for e > 0,   (-1)^s * m/2  for e = 0.
 * Its 16 code points include -1, 0, +1 exactly; a ternary value is stored as the
 * nibble that decodes to it with a canonical zero (0x0): +1 -> 0x2, -1 -> 0xA.
 * Two elements per byte, element 2j in the low nibble of byte j; a row holds
 * Kpad elements (Kpad/2 bytes), the padding is 0.                             */
double orc_e2m1_value(int nibble)
{
    int s = (nibble >> 3) & 1, e = (nibble >> 1) & 3, m = nibble & 1;
    double mag = e > 0 ? ldexp(1.0 + 0.5 * m, e - 1) : 0.5 * m;
    return s ? -mag : mag;
}

void orc_encode_fp4(const int8_t *t, int64_t rows, int64_t K, int64_t Kpad, uint8_t *out)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t j = 0; j < Kpad / 2; ++j) {
            int byte = 0;
            for (int h = 0; h < 2; ++h) {
                int64_t k = 2 * j + h;
                int v = k < K ? t[r * K + k] : 0;
                int nib = 0;
                /* the code point whose value is v (zero: the one without the sign bit) */
                for (int c = 15; c >= 0; --c)
                    if (orc_e2m1_value(c) == (double)v && !(v == 0 && c == 8)) nib = c;
                byte |= nib << (4 * h);
            }
            out[r * (Kpad / 2) + j] = (uint8_t)byte;
        }
}

/* returns the number of nibbles that do not decode to -1, 0 or +1 (they are written as 0) */
int64_t orc_decode_fp4(const uint8_t *codes, int64_t rows, int64_t K, int64_t Kpad, int8_t *t)
{
    int64_t bad = 0;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k) {
            int nib = (codes[r * (Kpad / 2) + k / 2] >> (4 * (k & 1))) & 15;
            double v = orc_e2m1_value(nib);
            if (v == 1.0 || v == -1.0 || v == 0.0) {
                t[r * K + k] = (int8_t)v;
            } else {
                t[r * K + k] = 0;
                ++bad;
            }
        }
    return bad;
}

void orc_pad_rows_i8(const int8_t *t, int64_t rows, int64_t K, int64_t Kpad, int8_t *out)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < Kpad; ++k)
            out[r * Kpad + k] = (k < K) ? t[r * K + k] : 0;
}

/* Layout only: [N][C][H][W] codes -> channel-innermost [N][H][W][Cpad].     */
void orc_nchw_to_nhwc_i8(const int8_t *t, int64_t N, int64_t C, int64_t H, int64_t W,
                         int64_t Cpad, int8_t *out)
{
    for (int64_t n = 0; n < N; ++n)
        for (int64_t h = 0; h < H; ++h)
            for (int64_t w = 0; w < W; ++w)
                for (int64_t c = 0; c < Cpad; ++c)
                    out[((n * H + h) * W + w) * Cpad + c] =
                        (c < C) ? t[((n * C + c) * H + h) * W + w] : 0;
}

/* ------------------------------------------------------------------ O4 --
 * Side sums of Eq.9's constant: 1 (x) W^t = sum of a ternary vector.        */
void orc_row_sums(const int8_t *t, int64_t rows, int64_t K, int32_t *s)
{
    for (int64_t r = 0; r < rows; ++r) {
        int64_t a = 0;
        for (int64_t k = 0; k < K; ++k) a += t[r * K + k];
        s[r] = (int32_t)a;
    }
}

/* Channel sum at every (n,h,w) of an [N][C][H][W] code tensor.  For a weight
 * tensor [O][I][KH][KW] this is the per-tap sum over input channels.        */
void orc_pixel_sums(const int8_t *t, int64_t N, int64_t C, int64_t H, int64_t W, int32_t *s)
{
    for (int64_t n = 0; n < N; ++n)
        for (int64_t h = 0; h < H; ++h)
            for (int64_t w = 0; w < W; ++w) {
                int64_t a = 0;
                for (int64_t c = 0; c < C; ++c) a += t[((n * C + c) * H + h) * W + w];
                s[(n * H + h) * W + w] = (int32_t)a;
            }
}

/* ------------------------------------------------------------------ O3 --
 * D[m][n] = sum_k t_a[m][k] * t_w[n][k]: the ternary dot product W^t (x) A^t
 * of Eq.8/Eq.9 by its definition.  int64 accumulate, |D| <= K checked, int32
 * stored (the circuit of Fig.3(a) keeps 32-bit counters).  Returns 0, or -1
 * if an accumulator left [-K, K].                                           */
int orc_gemm_acc(const int8_t *ta, const int8_t *tw, int64_t M, int64_t N, int64_t K, int32_t *D)
{
    int bad = 0;
#pragma omp parallel for
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int64_t)ta[m * K + k] * (int64_t)tw[n * K + k];
            if (acc > K || acc < -K) bad = 1;
            D[m * N + n] = (int32_t)acc;
        }
    return bad ? -1 : 0;
}

/* Second route to the same D, Eq.8 on the bit planes:
 * c = W_1 AND A_1;  D = bC(c) - 2*bC((W_2 XOR A_2) AND c).                  */
void orc_gemm_acc_popc(const uint64_t *ma, const uint64_t *sa, const uint64_t *mw,
                       const uint64_t *sw, int64_t M, int64_t N, int64_t words, int32_t *D)
{
#pragma omp parallel for
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t nz = 0, df = 0;
            for (int64_t w = 0; w < words; ++w) {
                uint64_t c = ma[m * words + w] & mw[n * words + w];
                nz += __builtin_popcountll(c);
                df += __builtin_popcountll((sa[m * words + w] ^ sw[n * words + w]) & c);
            }
            D[m * N + n] = (int32_t)(nz - 2 * df);
        }
}

/* ------------------------------------------------------------------ O5 --
 * Four-term reparameterization (Eq.9 with a weight offset added), in double,
 * rounded once to fp32:
 *   y = aa*aw*D + aa*bw*Sa + ba*aw*Sw + Kv*ba*bw ;  then ReLU (phi of Eq.9)
 *   if asked; then the BN affine that follows ReLU in RTN's layer order.
 * stride_* = 0 broadcasts one scalar, 1 indexes per row (a) / per column (w).
 * bw, bn_scale, bn_shift may be NULL (=> 0, 1, 0).                           */
static double apply_tail(double y, int relu, const float *bs, const float *bh, int64_t n)
{
    if (relu && y < 0.0) y = 0.0;
    if (bs) y = (double)bs[n] * y + (double)(bh ? bh[n] : 0.0f);
    return y;
}

void orc_gemm_epilogue(const int32_t *D, int64_t M, int64_t N, int64_t K,
                       const int32_t *Sa, const int32_t *Sw,
                       const float *aa, const float *ba, int stride_a,
                       const float *aw, const float *bw, int stride_w,
                       int relu, const float *bn_scale, const float *bn_shift, float *y)
{
#pragma omp parallel for
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double a_a = aa[m * stride_a], b_a = ba[m * stride_a];
            double a_w = aw[n * stride_w], b_w = bw ? bw[n * stride_w] : 0.0;
            double v = a_a * a_w * (double)D[m * N + n] + a_a * b_w * (double)Sa[m] +
                       b_a * a_w * (double)Sw[n] + (double)K * b_a * b_w;
            y[m * N + n] = (float)apply_tail(v, relu, bn_scale, bn_shift, n);
        }
}

/* ------------------------------------------------------------------ O6 --
 * Check of O3-O5, not part of them: the direct dot product of the
 * reparameterized values, sum_k (aa*t_a+ba)*(aw*t_w+bw), in double.          */
void orc_gemm_direct(const int8_t *ta, const int8_t *tw, int64_t M, int64_t N, int64_t K,
                     const float *aa, const float *ba, int stride_a,
                     const float *aw, const float *bw, int stride_w, double *y)
{
#pragma omp parallel for
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double a_a = aa[m * stride_a], b_a = ba[m * stride_a];
            double a_w = aw[n * stride_w], b_w = bw ? bw[n * stride_w] : 0.0;
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += (a_a * ta[m * K + k] + b_a) * (a_w * tw[n * K + k] + b_w);
            y[m * N + n] = acc;
        }
}

/* --------------------------------------------------------------- conv ----
 * Convolution as the dot product over a c*k*k patch (im2col view, footnote
 * of Section "Methodology"); cross-correlation, zero padding:
 *   ih = oh*stride - pad + kh,  iw = ow*stride - pad + kw,
 *   OH = floor((H + 2*pad - KH)/stride) + 1.
 * ta: [Nb][C][H][W], tw: [O][C][KH][KW], D: [Nb][O][OH][OW].
 * A tap outside the image contributes nothing to D (code 0).               */
typedef struct {
    int64_t Nb, C, H, W, O, KH, KW, stride, pad, OH, OW;
} orc_geom;

static orc_geom make_geom(int64_t Nb, int64_t C, int64_t H, int64_t W, int64_t O,
                          int64_t KH, int64_t KW, int64_t stride, int64_t pad)
{
    orc_geom g = {Nb, C, H, W, O, KH, KW, stride, pad,
                  (H + 2 * pad - KH) / stride + 1, (W + 2 * pad - KW) / stride + 1};
    return g;
}

void orc_conv_out_shape(int64_t H, int64_t W, int64_t KH, int64_t KW, int64_t stride,
                        int64_t pad, int64_t *OH, int64_t *OW)
{
    orc_geom g = make_geom(1, 1, H, W, 1, KH, KW, stride, pad);
    *OH = g.OH;
    *OW = g.OW;
}

int orc_conv_acc(const int8_t *ta, const int8_t *tw, int64_t Nb, int64_t C, int64_t H,
                 int64_t W, int64_t O, int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                 int32_t *D)
{
    orc_geom g = make_geom(Nb, C, H, W, O, KH, KW, stride, pad);
    int64_t K = C * KH * KW;
    int bad = 0;
#pragma omp parallel for
    for (int64_t nb = 0; nb < g.Nb; ++nb)
        for (int64_t o = 0; o < g.O; ++o)
            for (int64_t oh = 0; oh < g.OH; ++oh)
                for (int64_t ow = 0; ow < g.OW; ++ow) {
                    int64_t acc = 0;
                    for (int64_t c = 0; c < g.C; ++c)
                        for (int64_t kh = 0; kh < g.KH; ++kh)
                            for (int64_t kw = 0; kw < g.KW; ++kw) {
                                int64_t ih = oh * g.stride - g.pad + kh;
                                int64_t iw = ow * g.stride - g.pad + kw;
                                if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) continue;
                                acc += (int64_t)ta[((nb * g.C + c) * g.H + ih) * g.W + iw] *
                                       (int64_t)tw[((o * g.C + c) * g.KH + kh) * g.KW + kw];
                            }
                    if (acc > K || acc < -K) bad = 1;
                    D[((nb * g.O + o) * g.OH + oh) * g.OW + ow] = (int32_t)acc;
                }
    return bad ? -1 : 0;
}

/* Side sums for a padded conv.  pad_true_zero = 1: the padded border of the
 * reparameterized activation is a true 0 (what a framework conv of
 * gamma*t+beta does), so a padded tap contributes neither beta_a*w nor
 * beta_a*beta_w: Sw and Kv count in-bounds taps only.  pad_true_zero = 0:
 * the border holds code 0, i.e. the value beta_a; Sw is the whole filter
 * sum and Kv = K at every pixel (Eq.9's "C is a constant" holds verbatim).
 * Sa sums t_a over in-bounds taps in both modes (code 0 adds nothing).
 * Sa: [Nb][OH][OW], Sw: [O][OH][OW], Kv: [OH][OW].                          */
void orc_conv_sums(const int8_t *ta, const int8_t *tw, int64_t Nb, int64_t C, int64_t H,
                   int64_t W, int64_t O, int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                   int pad_true_zero, int32_t *Sa, int32_t *Sw, int32_t *Kv)
{
    orc_geom g = make_geom(Nb, C, H, W, O, KH, KW, stride, pad);
    for (int64_t oh = 0; oh < g.OH; ++oh)
        for (int64_t ow = 0; ow < g.OW; ++ow) {
            int64_t taps = 0;
            for (int64_t kh = 0; kh < g.KH; ++kh)
                for (int64_t kw = 0; kw < g.KW; ++kw) {
                    int64_t ih = oh * g.stride - g.pad + kh, iw = ow * g.stride - g.pad + kw;
                    int inb = !(ih < 0 || ih >= g.H || iw < 0 || iw >= g.W);
                    if (inb || !pad_true_zero) ++taps;
                }
            Kv[oh * g.OW + ow] = (int32_t)(taps * g.C);
            for (int64_t o = 0; o < g.O; ++o) {
                int64_t s = 0;
                for (int64_t c = 0; c < g.C; ++c)
                    for (int64_t kh = 0; kh < g.KH; ++kh)
                        for (int64_t kw = 0; kw < g.KW; ++kw) {
                            int64_t ih = oh * g.stride - g.pad + kh;
                            int64_t iw = ow * g.stride - g.pad + kw;
                            int inb = !(ih < 0 || ih >= g.H || iw < 0 || iw >= g.W);
                            if (inb || !pad_true_zero)
                                s += tw[((o * g.C + c) * g.KH + kh) * g.KW + kw];
                        }
                Sw[(o * g.OH + oh) * g.OW + ow] = (int32_t)s;
            }
            for (int64_t nb = 0; nb < g.Nb; ++nb) {
                int64_t s = 0;
                for (int64_t c = 0; c < g.C; ++c)
                    for (int64_t kh = 0; kh < g.KH; ++kh)
                        for (int64_t kw = 0; kw < g.KW; ++kw) {
                            int64_t ih = oh * g.stride - g.pad + kh;
                            int64_t iw = ow * g.stride - g.pad + kw;
                            if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) continue;
                            s += ta[((nb * g.C + c) * g.H + ih) * g.W + iw];
                        }
                Sa[(nb * g.OH + oh) * g.OW + ow] = (int32_t)s;
            }
        }
}

/* Conv form of O5.  alpha_a/beta_a are layer-wise scalars (Eq.4 and the note
 * that the factors are designed layer-wise); alpha_w/beta_w are one scalar
 * (stride_w = 0) or one per filter (stride_w = 1).  y: [Nb][O][OH][OW].      */
void orc_conv_epilogue(const int32_t *D, const int32_t *Sa, const int32_t *Sw, const int32_t *Kv,
                       int64_t Nb, int64_t O, int64_t OH, int64_t OW, float aa, float ba,
                       const float *aw, const float *bw, int stride_w, int relu,
                       const float *bn_scale, const float *bn_shift, float *y)
{
#pragma omp parallel for
    for (int64_t nb = 0; nb < Nb; ++nb)
        for (int64_t o = 0; o < O; ++o)
            for (int64_t p = 0; p < OH * OW; ++p) {
                double a_a = aa, b_a = ba;
                double a_w = aw[o * stride_w], b_w = bw ? bw[o * stride_w] : 0.0;
                int64_t i = (nb * O + o) * OH * OW + p;
                double v = a_a * a_w * (double)D[i] + a_a * b_w * (double)Sa[nb * OH * OW + p] +
                           b_a * a_w * (double)Sw[o * OH * OW + p] + (double)Kv[p] * b_a * b_w;
                y[i] = (float)apply_tail(v, relu, bn_scale, bn_shift, o);
            }
}

/* ------------------------------------------------------------------ O7 --
 * The activation handed to the next ternary layer.  RTN's layer order is
 * conv -> ReLU -> BN -> ternarize (Section "Reparameterized Ternarization":
 * BN follows ReLU so that negative values exist again), so the next layer's
 * fixed ternary input is Q applied to the fp32 output z of the epilogue above:
 *   t[nb][o][p] = (z > hi[o]) - (z < lo[o])        (Eq.1; strict, on fp32 z)
 * with one (lo, hi) per layer (per_channel = 0) or per output channel
 * (per_channel = 1).  The per-channel form is what Eq.3 needs when the BN
 * affine k*z + b is not applied but folded into the thresholds,
 * hi = (0.5-b)/k, lo = -(0.5+b)/k.  z: [Nb][O][HW] fp32, t: same shape.     */
void orc_ternarize_nchw(const float *z, int64_t Nb, int64_t O, int64_t HW,
                        const float *lo, const float *hi, int per_channel, int8_t *t)
{
#pragma omp parallel for
    for (int64_t nb = 0; nb < Nb; ++nb)
        for (int64_t o = 0; o < O; ++o) {
            float l = per_channel ? lo[o] : lo[0];
            float h = per_channel ? hi[o] : hi[0];
            for (int64_t p = 0; p < HW; ++p) {
                float v = z[(nb * O + o) * HW + p];
                t[(nb * O + o) * HW + p] = (int8_t)((v > h) - (v < l));
            }
        }
}

/* ------------------------------------------------------------------ O8 --
 * Tail of a residual block: the last conv's activation z meets the shortcut
 * r before the next block ternarizes the sum.  The adds of the network are
 * plain fp32 tensor operations, so  s = z + r  is ONE fp32 addition of the two
 * stored fp32 values (no wider intermediate), followed by max(s, 0) if relu.  */
void orc_add_relu(const float *z, const float *r, int64_t n, int relu, float *s)
{
#pragma omp parallel for
    for (int64_t i = 0; i < n; ++i) {
        volatile float v = z[i] + r[i]; /* volatile: force the fp32 rounding of the sum */
        float w = v;
        s[i] = (relu && w < 0.0f) ? 0.0f : w;
    }
}

/* ------------------------------------------------------------------ O9 --
 * Weight-only ternary layer (the 2-bit-weight / 32-bit-activation rows of the
 * ImageNet table): the weights are alpha * W^t as everywhere else (Section
 * "Weight Ternarization": scale only, no offset), the activations stay fp32:
 *   y[m][n] = alpha_w[n] * sum_k x[m][k] * t_w[n][k]
 * summed in double in index order, then the same tail as O5 (ReLU, BN affine),
 * rounded once to fp32.  aw: one scalar (stride_w = 0) or one per column.   */
void orc_wgemm(const float *x, const int8_t *tw, int64_t M, int64_t N, int64_t K,
               const float *aw, int stride_w, int relu,
               const float *bn_scale, const float *bn_shift, float *y)
{
#pragma omp parallel for
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k) s += (double)x[m * K + k] * (double)tw[n * K + k];
            double v = (double)aw[n * stride_w] * s;
            y[m * N + n] = (float)apply_tail(v, relu, bn_scale, bn_shift, n);
        }
}

/* Conv form of O9: fp32 activations x [Nb][C][H][W], ternary weights
 * alpha_w[o] * t_w [O][C][KH][KW], cross-correlation with zero padding (a padded
 * tap adds nothing), summed in double in (c, kh, kw) order, same tail.       */
void orc_wconv(const float *x, const int8_t *tw, int64_t Nb, int64_t C, int64_t H, int64_t W,
               int64_t O, int64_t KH, int64_t KW, int64_t stride, int64_t pad,
               const float *aw, int stride_w, int relu,
               const float *bn_scale, const float *bn_shift, float *y)
{
    int64_t OH = (H + 2 * pad - KH) / stride + 1, OW = (W + 2 * pad - KW) / stride + 1;
#pragma omp parallel for collapse(2)
    for (int64_t nb = 0; nb < Nb; ++nb)
        for (int64_t o = 0; o < O; ++o)
            for (int64_t oh = 0; oh < OH; ++oh)
                for (int64_t ow = 0; ow < OW; ++ow) {
                    double s = 0.0;
                    for (int64_t c = 0; c < C; ++c)
                        for (int64_t kh = 0; kh < KH; ++kh)
                            for (int64_t kw = 0; kw < KW; ++kw) {
                                int64_t ih = oh * stride - pad + kh, iw = ow * stride - pad + kw;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                s += (double)x[((nb * C + c) * H + ih) * W + iw] *
                                     (double)tw[((o * C + c) * KH + kh) * KW + kw];
                            }
                    double v = (double)aw[o * stride_w] * s;
                    y[((nb * O + o) * OH + oh) * OW + ow] = (float)apply_tail(v, relu, bn_scale, bn_shift, o);
                }
}

/* ----------------------------------------------------------------- O10 --
 * Backward of the reparameterized ternary activation  Abar^t = gamma*Q(Abar) + beta
 * (Section "Backward Update in Reparameterized Ternarization").  With g = dL/dAbar^t:
 *   dL/dgamma = sum_i A^t_i * g_i,   dL/dbeta = sum_i g_i          (Eq.6, layer-wise)
 *   dL/dAbar_i = gamma * 1[|Abar_i| <= 1] * g_i                     (Eq.7, clipped STE)
 * A^t = (a > hi) - (a < lo) as in O1.  The sums are taken in double in index
 * order; gamma*g is one fp32 product.  sums[0] = dgamma, sums[1] = dbeta.      */
void orc_act_backward(const float *a, const float *g, int64_t n, float lo, float hi, float gamma,
                      float *da, double *sums)
{
    double sg = 0.0, sb = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        int t = (a[i] > hi) - (a[i] < lo);
        sg += (double)t * (double)g[i];
        sb += (double)g[i];
        if (da) {
            volatile float p = gamma * g[i]; /* volatile: one fp32 rounding of the product */
            float q = p;
            int inside = (a[i] <= 1.0f) && (a[i] >= -1.0f); /* |a| <= 1; NaN is outside */
            da[i] = inside ? q : 0.0f;
        }
    }
    sums[0] = sg;
    sums[1] = sb;
}

/* ----------------------------------------------------------------- O11 --
 * Backward of the reparameterized ternary weights, one filter (row of K values) at a
 * time (Section "Weight Ternarization": Wbar = k_W*W + b_W, W^t = Q(Wbar),
 * Wbar^t = alpha*W^t, all three parameters per filter).  The paper prints the
 * derivatives for the activation only (Eq.6, Eq.7); these are the same two rules
 * applied to the weight transform by the chain rule.  With g = dL/dWbar^t:
 *   dL/dalpha = sum_k W^t_k * g_k                                  (as Eq.6)
 *   dL/dWbar_k = alpha * 1[|Wbar_k| <= 1] * g_k                     (as Eq.7)
 *   dL/dk_W = sum_k W_k * dL/dWbar_k,  dL/db_W = sum_k dL/dWbar_k,  dL/dW_k = k_W * dL/dWbar_k
 * Wbar is ONE fused multiply-add in fp32, W^t = (Wbar > hi) - (Wbar < lo); alpha*g and
 * k_W*(alpha*g) are one fp32 product each; the sums are taken in double in index order.
 * sums[3*o + 0..2] = dalpha, dk_W, db_W of filter o.                              */
void orc_weight_backward(const float *w, const float *g, int64_t O, int64_t K, float lo, float hi,
                         const float *kw, const float *bw, const float *alpha, float *dw, double *sums)
{
    for (int64_t o = 0; o < O; ++o) {
        double sa = 0.0, sk = 0.0, sb = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const int64_t i = o * K + k;
            float wbar = fmaf(kw[o], w[i], bw[o]);
            int t = (wbar > hi) - (wbar < lo);
            sa += (double)t * (double)g[i];
            volatile float p = alpha[o] * g[i]; /* volatile: one fp32 rounding per product */
            float q = p;
            int inside = (wbar <= 1.0f) && (wbar >= -1.0f); /* NaN is outside */
            float dwbar = inside ? q : 0.0f;
            if (inside) { /* a clipped (or NaN) weight adds nothing, not NaN * 0 */
                sk += (double)w[i] * (double)dwbar;
                sb += (double)dwbar;
            }
            if (dw) {
                volatile float r = kw[o] * dwbar;
                dw[i] = r;
            }
        }
        sums[3 * o + 0] = sa;
        sums[3 * o + 1] = sk;
        sums[3 * o + 2] = sb;
    }
}

/* Conv form of O6: direct conv of the reparameterized values in double.
 * pad_true_zero = 1 pads the value tensor (aa*t+ba) with 0.0;
 * pad_true_zero = 0 pads the code tensor with 0, i.e. the value with ba.     */
void orc_conv_direct(const int8_t *ta, const int8_t *tw, int64_t Nb, int64_t C, int64_t H,
                     int64_t W, int64_t O, int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                     int pad_true_zero, float aa, float ba, const float *aw, const float *bw,
                     int stride_w, double *y)
{
    orc_geom g = make_geom(Nb, C, H, W, O, KH, KW, stride, pad);
#pragma omp parallel for
    for (int64_t nb = 0; nb < g.Nb; ++nb)
        for (int64_t o = 0; o < g.O; ++o)
            for (int64_t oh = 0; oh < g.OH; ++oh)
                for (int64_t ow = 0; ow < g.OW; ++ow) {
                    double a_w = aw[o * stride_w], b_w = bw ? bw[o * stride_w] : 0.0;
                    double acc = 0.0;
                    for (int64_t c = 0; c < g.C; ++c)
                        for (int64_t kh = 0; kh < g.KH; ++kh)
                            for (int64_t kw = 0; kw < g.KW; ++kw) {
                                int64_t ih = oh * g.stride - g.pad + kh;
                                int64_t iw = ow * g.stride - g.pad + kw;
                                double av;
                                if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W)
                                    av = pad_true_zero ? 0.0 : (double)ba;
                                else
                                    av = (double)aa * ta[((nb * g.C + c) * g.H + ih) * g.W + iw] +
                                         (double)ba;
                                acc += av * (a_w * tw[((o * g.C + c) * g.KH + kh) * g.KW + kw] + b_w);
                            }
                    y[((nb * g.O + o) * g.OH + oh) * g.OW + ow] = acc;
                }
}

/* Rows-subset form of O3 for timing and sampled checks at sizes where the
 * full triple loop would take minutes: D_sub[i][n] for m = rows[i].          */
int orc_gemm_acc_rows(const int8_t *ta, const int8_t *tw, const int64_t *rows, int64_t R,
                      int64_t N, int64_t K, int32_t *D)
{
    int bad = 0;
#pragma omp parallel for
    for (int64_t i = 0; i < R; ++i)
        for (int64_t n = 0; n < N; ++n) {
            int64_t m = rows[i], acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int64_t)ta[m * K + k] * (int64_t)tw[n * K + k];
            if (acc > K || acc < -K) bad = 1;
            D[i * N + n] = (int32_t)acc;
        }
    return bad ? -1 : 0;
}

/* ----------------------------------------------------------------- O12 --
 * The comparison system of Section "How to Compute Dot Product between Two Ternary
 * Vectors" (second half) and Fig.3(b): 2-bit quaternary weights and activations,
 * value = 2*(1st bit) + (2nd bit) in {0,1,2,3} (Table 1's "2-bit network true
 * value" column), multiplied in the bit-serial pattern of DoReFa-Net: AND between
 * each bit of the one input and each bit of the other, a count of ones per pair of
 * bit planes, a left shift by the two bit weights, and the four partial results
 * added:   sum_k qw[k]*qa[k] = sum_{i,j in {0,1}} 2^(i+j) * bC(W_i AND A_j),
 * W_1 / A_1 the planes of the first (more significant) bits, W_0 / A_0 of the second.
 * The quantizer is not the paper's subject; the plain form used here is three
 * strict thresholds on the stored value, q = (x > t1) + (x > t2) + (x > t3).      */
void orc_quantize4(const float *x, int64_t n, float t1, float t2, float t3, int8_t *q)
{
    for (int64_t i = 0; i < n; ++i) q[i] = (int8_t)((x[i] > t1) + (x[i] > t2) + (x[i] > t3));
}

/* the definition: a plain sum of products */
int orc_qgemm_acc(const int8_t *qa, const int8_t *qw, int64_t M, int64_t N, int64_t K, int32_t *D)
{
    int bad = 0;
#pragma omp parallel for
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k) acc += (int64_t)qa[m * K + k] * (int64_t)qw[n * K + k];
            if (acc < 0 || acc > 9 * K) bad = 1;
            D[m * N + n] = (int32_t)acc;
        }
    return bad;
}

/* bit planes of quaternary values: hi = plane of first bits (weight 2), lo = plane of second
 * bits (weight 1); bit j of word w of a row is element 64*w + j, as for the ternary planes */
void orc_encode_qplanes(const int8_t *q, int64_t rows, int64_t K, int64_t words, uint64_t *hi, uint64_t *lo)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t w = 0; w < words; ++w) {
            uint64_t h = 0, l = 0;
            for (int j = 0; j < 64; ++j) {
                int64_t k = 64 * w + j;
                int v = k < K ? q[r * K + k] : 0;
                h |= (uint64_t)((v >> 1) & 1) << j;
                l |= (uint64_t)(v & 1) << j;
            }
            hi[r * words + w] = h;
            lo[r * words + w] = l;
        }
}

/* the circuit of Fig.3(b): four AND / count pairs, shifts, four adders */
void orc_qgemm_bitserial(const uint64_t *ah, const uint64_t *al, const uint64_t *wh, const uint64_t *wl,
                         int64_t M, int64_t N, int64_t words, int32_t *D)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t c11 = 0, c10 = 0, c01 = 0, c00 = 0;
            for (int64_t w = 0; w < words; ++w) {
                c11 += __builtin_popcountll(wh[n * words + w] & ah[m * words + w]);
                c10 += __builtin_popcountll(wh[n * words + w] & al[m * words + w]);
                c01 += __builtin_popcountll(wl[n * words + w] & ah[m * words + w]);
                c00 += __builtin_popcountll(wl[n * words + w] & al[m * words + w]);
            }
            D[m * N + n] = (int32_t)((c11 << 2) + (c10 << 1) + (c01 << 1) + c00);
        }
}

/* ----------------------------------------------------------------- O13 --
 * Depthwise form of the ternary convolution (the 3x3 layers of MobileNet, one of the
 * networks of the paper's ImageNet table): every channel is convolved with its own
 * k x k ternary filter, so one dot product has length K = k*k.  The reparameterized
 * output is the same four-term formula with everything per channel:
 *   y[n][c][p] = aa*aw[c]*D + aa*bw[c]*Sa + ba*aw[c]*Sw + Kv*ba*bw[c],
 * D = sum over in-bounds taps of t_a*t_w,  Sa = sum of t_a,  Sw = sum of t_w over the
 * in-bounds taps (zero padding of the reparameterized activation) or over all taps
 * with Kv = k*k (code-zero padding), Kv = number of in-bounds taps.
 * ta: [Nb][C][H][W], tw: [C][KH][KW]; y: [Nb][C][OH][OW] (fp64 evaluation, one rounding) */
void orc_dwconv(const int8_t *ta, const int8_t *tw, int64_t Nb, int64_t C, int64_t H, int64_t W,
                int64_t KH, int64_t KW, int64_t stride, int64_t pad, int pad_true_zero, float aa, float ba,
                const float *aw, const float *bw, int stride_w, int relu, const float *bn_scale,
                const float *bn_shift, int32_t *D, float *y)
{
    int64_t OH = (H + 2 * pad - KH) / stride + 1, OW = (W + 2 * pad - KW) / stride + 1;
#pragma omp parallel for
    for (int64_t nb = 0; nb < Nb; ++nb)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t oh = 0; oh < OH; ++oh)
                for (int64_t ow = 0; ow < OW; ++ow) {
                    int64_t d = 0, sa = 0, sw = 0, kv = 0;
                    for (int64_t kh = 0; kh < KH; ++kh)
                        for (int64_t kw = 0; kw < KW; ++kw) {
                            int64_t ih = oh * stride - pad + kh, iw = ow * stride - pad + kw;
                            int inb = ih >= 0 && ih < H && iw >= 0 && iw < W;
                            int w_ = tw[(c * KH + kh) * KW + kw];
                            if (inb) {
                                int a_ = ta[((nb * C + c) * H + ih) * W + iw];
                                d += a_ * w_;
                                sa += a_;
                            }
                            if (inb || !pad_true_zero) {
                                sw += w_;
                                kv += 1;
                            }
                        }
                    int64_t i = ((nb * C + c) * OH + oh) * OW + ow;
                    double a_w = aw[c * stride_w], b_w = bw ? bw[c * stride_w] : 0.0;
                    double v = (double)aa * a_w * (double)d + (double)aa * b_w * (double)sa +
                               (double)ba * a_w * (double)sw + (double)kv * (double)ba * b_w;
                    if (D) D[i] = (int32_t)d;
                    if (y) y[i] = (float)apply_tail(v, relu, bn_scale, bn_shift, c);
                }
}

/* FP4 nibbles that hold small integers (0..3 are code points of E2M1 too): decoded values,
 * and the number of nibbles whose value is not an integer in [-6, 6] */
int64_t orc_decode_fp4_int(const uint8_t *codes, int64_t rows, int64_t K, int64_t Kpad, int8_t *v)
{
    int64_t bad = 0;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k) {
            double x = orc_e2m1_value((codes[r * (Kpad / 2) + k / 2] >> (4 * (k & 1))) & 15);
            if (x != floor(x)) {
                ++bad;
                x = 0;
            }
            v[r * K + k] = (int8_t)x;
        }
    return bad;
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
