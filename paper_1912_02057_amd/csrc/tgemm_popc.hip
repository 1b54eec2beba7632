// Ternary contraction on bit planes by Eq.8 (AND / XOR / popcount) on the
// vector ALU, plus the stand-alone epilogue kernels.
//
//   c = W_1 & A_1 ;  D = bC(c) - 2 * bC((W_2 ^ A_2) & c)
//
// Per 64 MACs a lane spends 3 logic ops and 2 popcount-accumulates on 64-bit
// words (twice that many 32-bit VALU instructions), so this path tops out near
// a tenth of the int8 matrix-core rate; it exists for the comparison the
// method's own computation pattern invites and for memory-bound shapes where
// 0.25 B/element of operand traffic matters more than ALU rate.
#include "epilogue_math.h"
#include "rtn_kernels.h"

namespace rtn {

namespace {

constexpr int PT = 64;   // output tile edge
constexpr int KC = 8;    // 64-bit words per stage
constexpr int LDW = KC + 1;  // padded LDS row pitch (words): conflict-free 8-byte reads

__global__ __launch_bounds__(256) void k_gemm_popc(PopcArgs a)
{
    __shared__ uint64_t sAm[PT * LDW], sAs[PT * LDW], sWm[PT * LDW], sWs[PT * LDW];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int64_t tilesN = (a.N + PT - 1) / PT;
    const int64_t m0 = (blockIdx.x / tilesN) * PT, n0 = (blockIdx.x % tilesN) * PT;

    int nz[4][4], df[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) nz[i][j] = df[i][j] = 0;

    for (int64_t w0 = 0; w0 < a.words; w0 += KC) {
        // stage 64 rows x KC words of each plane; a thread moves 2 words per plane
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int e = tid + 256 * i, row = e / KC, w = e % KC;
            const bool wok = w0 + w < a.words;
            const bool aok = wok && m0 + row < a.M, bok = wok && n0 + row < a.N;
            const int64_t ai = (m0 + row) * a.words + w0 + w, bi = (n0 + row) * a.words + w0 + w;
            sAm[row * LDW + w] = aok ? a.a_mask[ai] : 0;
            sAs[row * LDW + w] = aok ? a.a_sign[ai] : 0;
            sWm[row * LDW + w] = bok ? a.w_mask[bi] : 0;
            sWs[row * LDW + w] = bok ? a.w_sign[bi] : 0;
        }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < KC; ++w) {
            uint64_t am[4], as[4], wm[4], ws[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                am[i] = sAm[(ty * 4 + i) * LDW + w];
                as[i] = sAs[(ty * 4 + i) * LDW + w];
                wm[i] = sWm[(tx + 16 * i) * LDW + w];
                ws[i] = sWs[(tx + 16 * i) * LDW + w];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint64_t c = am[i] & wm[j];
                    nz[i][j] += __popcll(c);
                    df[i][j] += __popcll((as[i] ^ ws[j]) & c);
                }
        }
        __syncthreads();
    }

    const EpiArgs& ep = a.ep;
    const bool has_bn = ep.bn_scale != nullptr;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + ty * 4 + i;
        if (m >= a.M) continue;
        double aa = 0.0, ba = 0.0;
        int Sa = 0;
        if (a.y) {
            aa = pval(ep.alpha_a, m);
            ba = pval(ep.beta_a, m);
            Sa = ep.sum_ta[m];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + tx + 16 * j;
            if (n >= a.N) continue;
            const int D = nz[i][j] - 2 * df[i][j];
            if (a.acc) a.acc[m * a.N + n] = D;
            if (a.y) {
                const double bs = has_bn ? (double)ep.bn_scale[n] : 1.0;
                const double bh = (has_bn && ep.bn_shift) ? (double)ep.bn_shift[n] : 0.0;
                a.y[m * a.N + n] = reparam(aa, ba, pval(ep.alpha_w, n), pval(ep.beta_w, n), D, Sa,
                                           ep.sum_tw[n], (int)a.K, ep.relu, has_bn, bs, bh);
            }
        }
    }
}

// Stand-alone epilogue, GEMM form: one thread per output element.
__global__ __launch_bounds__(256) void k_epilogue_gemm(const int32_t* acc, int64_t M, int64_t N, int K,
                                                       EpiArgs ep, float* y)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= M * N) return;
    const int64_t m = i / N, n = i - m * N;
    const bool has_bn = ep.bn_scale != nullptr;
    const double bs = has_bn ? (double)ep.bn_scale[n] : 1.0;
    const double bh = (has_bn && ep.bn_shift) ? (double)ep.bn_shift[n] : 0.0;
    y[i] = reparam(pval(ep.alpha_a, m), pval(ep.beta_a, m), pval(ep.alpha_w, n), pval(ep.beta_w, n),
                   acc[i], ep.sum_ta[m], ep.sum_tw[n], K, ep.relu, has_bn, bs, bh);
}

// Stand-alone epilogue, conv form: one thread per output element of
// [Nb][O][OH][OW]; Sa, Sw, Kv are formed from the pixel / tap sums over the
// in-bounds taps of the output pixel.
__global__ __launch_bounds__(256) void k_epilogue_conv(const int32_t* acc, ConvGeom g, EpiArgs ep, float* y)
{
    const int64_t ohw = (int64_t)g.OH * g.OW;
    const int64_t total = (int64_t)g.Nb * g.O * ohw;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int pix = (int)(i % ohw);
    const int o = (int)((i / ohw) % g.O);
    const int64_t nb = i / (ohw * g.O);
    const int oh = pix / g.OW, ow = pix - oh * g.OW;
    int khl, khh, kwl, kwh;
    tap_range(oh, g.stride, g.pad, g.KH, g.H, khl, khh);
    tap_range(ow, g.stride, g.pad, g.KW, g.W, kwl, kwh);
    int Sa = 0;
    const int32_t* ps = ep.sum_ta + nb * g.H * g.W;
    for (int kh = khl; kh <= khh; ++kh)
        for (int kw = kwl; kw <= kwh; ++kw)
            Sa += ps[(oh * g.stride - g.pad + kh) * g.W + (ow * g.stride - g.pad + kw)];
    if (g.code_zero_pad) {
        khl = 0, khh = g.KH - 1, kwl = 0, kwh = g.KW - 1;
    }
    int Sw = 0;
    for (int kh = khl; kh <= khh; ++kh)
        for (int kw = kwl; kw <= kwh; ++kw) Sw += ep.sum_tw[((int64_t)o * g.KH + kh) * g.KW + kw];
    const int Kv = g.C * (khh - khl + 1) * (kwh - kwl + 1);
    const bool has_bn = ep.bn_scale != nullptr;
    const double bs = has_bn ? (double)ep.bn_scale[o] : 1.0;
    const double bh = (has_bn && ep.bn_shift) ? (double)ep.bn_shift[o] : 0.0;
    y[i] = reparam((double)ep.alpha_a.s, (double)ep.beta_a.s, pval(ep.alpha_w, o), pval(ep.beta_w, o),
                   acc[i], Sa, Sw, Kv, ep.relu, has_bn, bs, bh);
}

}  // namespace

hipError_t launch_gemm_popc(const PopcArgs& a, hipStream_t st)
{
    const int64_t blocks = ((a.M + PT - 1) / PT) * ((a.N + PT - 1) / PT);
    if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_gemm_popc, dim3((unsigned)blocks), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_epilogue_gemm(const int32_t* acc, int64_t M, int64_t N, int64_t K, const EpiArgs& ep,
                                float* y, hipStream_t st)
{
    const int64_t blocks = (M * N + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_epilogue_gemm, dim3((unsigned)blocks), dim3(256), 0, st, acc, M, N, (int)K, ep, y);
    return hipGetLastError();
}

hipError_t launch_epilogue_conv(const int32_t* acc, const ConvGeom& g, const EpiArgs& ep, float* y,
                                hipStream_t st)
{
    const int64_t total = (int64_t)g.Nb * g.O * g.OH * g.OW;
    const int64_t blocks = (total + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_epilogue_conv, dim3((unsigned)blocks), dim3(256), 0, st, acc, g, ep, y);
    return hipGetLastError();
}

}  // namespace rtn
