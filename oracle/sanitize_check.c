/*
 * Sanitizer run of the oracle -- TEST INFRASTRUCTURE.  Compiled together with rtn_oracle.c under
 * -fsanitize=address,undefined (tests/test_oracle_pins.py builds and runs it): every oracle
 * routine is called on exactly-sized heap buffers with ragged shapes, so that any access past
 * an end, any misaligned or overflowing operation is reported.  Values are not checked here
 * (the pins do that); the process exits 0 when nothing was reported.
 */
#include "rtn_oracle.c"
#include <stdio.h>
#include <string.h>

static unsigned long long rs = 88172645463325252ull;
static unsigned rnd(void) { rs ^= rs << 13; rs ^= rs >> 7; rs ^= rs << 17; return (unsigned)(rs >> 32); }
static int8_t *tern_buf(int64_t n) { int8_t *p = malloc(n ? n : 1); for (int64_t i = 0; i < n; ++i) p[i] = (int8_t)(rnd() % 3) - 1; return p; }
static float *f32_buf(int64_t n) { float *p = malloc((n ? n : 1) * 4); for (int64_t i = 0; i < n; ++i) p[i] = (float)(rnd() % 2001) / 1000.0f - 1.0f; return p; }

int main(void)
{
    /* rows / GEMM side */
    const int64_t M = 7, N = 5, K = 131, Kpad = 192, Kp4 = 256, words = 3;
    float *x = f32_buf(M * K), lo = -0.3f, hi = 0.4f;
    int8_t *ta = malloc(M * K), *tw = tern_buf(N * K), *back = malloc(M * K);
    orc_ternarize(x, M, K, &lo, &hi, 0, ta);
    uint8_t *v2 = malloc(M * K);
    orc_encode_2bit(ta, M * K, v2); orc_decode_2bit(v2, M * K, back);
    uint64_t *ma = malloc(M * words * 8), *sa = malloc(M * words * 8), *mw = malloc(N * words * 8), *sw = malloc(N * words * 8);
    orc_encode_planes(ta, M, K, words, ma, sa); orc_encode_planes(tw, N, K, words, mw, sw);
    orc_decode_planes(ma, sa, M, K, words, back);
    uint8_t *f4 = malloc(M * Kp4 / 2);
    orc_encode_fp4(ta, M, K, Kp4, f4); orc_decode_fp4(f4, M, K, Kp4, back); orc_decode_fp4_int(f4, M, K, Kp4, back);
    int8_t *padded = malloc(M * Kpad); orc_pad_rows_i8(ta, M, K, Kpad, padded);
    int32_t *Sa = malloc(M * 4), *Sw = malloc(N * 4), *D = malloc(M * N * 4), *D2 = malloc(M * N * 4);
    orc_row_sums(ta, M, K, Sa); orc_row_sums(tw, N, K, Sw);
    orc_gemm_acc(ta, tw, M, N, K, D); orc_gemm_acc_popc(ma, sa, mw, sw, M, N, words, D2);
    if (memcmp(D, D2, M * N * 4)) { printf("Eq.8 route differs\n"); return 1; }
    int64_t rows[3] = {0, 3, 6};
    int32_t *Dr = malloc(3 * N * 4); orc_gemm_acc_rows(ta, tw, rows, 3, N, K, Dr);
    float *aa = f32_buf(M), *ba = f32_buf(M), *aw = f32_buf(N), *bw = f32_buf(N), *y = malloc(M * N * 4);
    double *yd = malloc(M * N * 8);
    orc_gemm_epilogue(D, M, N, K, Sa, Sw, aa, ba, 1, aw, bw, 1, 1, aw, bw, y);
    orc_gemm_direct(ta, tw, M, N, K, aa, ba, 1, aw, bw, 1, yd);
    orc_wgemm(x, tw, M, N, K, aw, 1, 1, aw, bw, y);
    /* conv side: ragged image, stride 2, pad 2, 5x5 and 3x3 */
    for (int cfg = 0; cfg < 3; ++cfg) {
        const int64_t Nb = 2, C = 5, H = 7, W = 6, O = 3, KH = cfg ? 3 : 5, KW = KH, st = cfg == 2 ? 2 : 1, pad = cfg ? 1 : 2;
        int64_t OH, OW; orc_conv_out_shape(H, W, KH, KW, st, pad, &OH, &OW);
        int8_t *ca = tern_buf(Nb * C * H * W), *cw = tern_buf(O * C * KH * KW), *nhwc = malloc(Nb * H * W * 64);
        orc_nchw_to_nhwc_i8(ca, Nb, C, H, W, 64, nhwc);
        int32_t *ps = malloc(Nb * H * W * 4); orc_pixel_sums(ca, Nb, C, H, W, ps);
        int32_t *cD = malloc(Nb * O * OH * OW * 4), *cSa = malloc(Nb * OH * OW * 4), *cSw = malloc(O * OH * OW * 4), *cKv = malloc(OH * OW * 4);
        orc_conv_acc(ca, cw, Nb, C, H, W, O, KH, KW, st, pad, cD);
        float *cy = malloc(Nb * O * OH * OW * 4), *cy2 = malloc(Nb * O * OH * OW * 4);
        double *cyd = malloc(Nb * O * OH * OW * 8);
        int8_t *ct = malloc(Nb * O * OH * OW);
        for (int tz = 0; tz < 2; ++tz) {
            orc_conv_sums(ca, cw, Nb, C, H, W, O, KH, KW, st, pad, tz, cSa, cSw, cKv);
            orc_conv_epilogue(cD, cSa, cSw, cKv, Nb, O, OH, OW, 1.1f, -0.1f, aw, bw, 1, 1, aw, bw, cy);
            orc_conv_direct(ca, cw, Nb, C, H, W, O, KH, KW, st, pad, tz, 1.1f, -0.1f, aw, bw, 1, cyd);
        }
        orc_ternarize_nchw(cy, Nb, O, OH * OW, aw, bw, 1, ct);
        orc_add_relu(cy, cy, Nb * O * OH * OW, 1, cy2);
        float *cx = f32_buf(Nb * C * H * W);
        orc_wconv(cx, cw, Nb, C, H, W, O, KH, KW, st, pad, aw, 1, 0, NULL, NULL, cy);
        int8_t *dwt = tern_buf(C * KH * KW);
        int32_t *dD = malloc(Nb * C * OH * OW * 4); float *dy = malloc(Nb * C * OH * OW * 4);
        orc_dwconv(ca, dwt, Nb, C, H, W, KH, KW, st, pad, cfg & 1, 1.2f, 0.1f, aw, bw, 1, 1, aw, bw, dD, dy);
        free(ca); free(cw); free(nhwc); free(ps); free(cD); free(cSa); free(cSw); free(cKv); free(cy); free(cy2); free(cyd); free(ct); free(cx); free(dwt); free(dD); free(dy);
    }
    /* backward rules */
    const int64_t n = 1001;
    float *a1 = f32_buf(n), *g1 = f32_buf(n), *da = malloc(n * 4); double sums[2];
    orc_act_backward(a1, g1, n, -0.5f, 0.5f, 0.9f, da, sums);
    orc_act_backward(a1, g1, n, -0.5f, 0.5f, 0.9f, NULL, sums);
    const int64_t O2 = 3, K2 = 37;
    float *w2 = f32_buf(O2 * K2), *g2 = f32_buf(O2 * K2), *kw = f32_buf(O2), *bw2 = f32_buf(O2), *al = f32_buf(O2), *dw = malloc(O2 * K2 * 4);
    double *ws = malloc(O2 * 3 * 8);
    orc_weight_backward(w2, g2, O2, K2, -0.5f, 0.5f, kw, bw2, al, dw, ws);
    /* quaternary comparison */
    int8_t *qa = malloc(M * K), *qw = malloc(N * K);
    orc_quantize4(x, M * K, 0.1f, 0.3f, 0.6f, qa);
    for (int64_t i = 0; i < N * K; ++i) qw[i] = (int8_t)(rnd() & 3);
    orc_qgemm_acc(qa, qw, M, N, K, D);
    orc_encode_qplanes(qa, M, K, words, ma, sa); orc_encode_qplanes(qw, N, K, words, mw, sw);
    orc_qgemm_bitserial(ma, sa, mw, sw, M, N, words, D2);
    if (memcmp(D, D2, M * N * 4)) { printf("bit-serial route differs\n"); return 1; }
    orc_encode_fp4(qa, M, K, Kp4, f4); orc_decode_fp4_int(f4, M, K, Kp4, back);
    if (memcmp(qa, back, M * K)) { printf("fp4 round trip differs\n"); return 1; }
    printf("sanitize_check ok (%d threads)\n", orc_num_threads());
    return 0;
}
