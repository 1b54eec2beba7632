// Ternary contraction on the gfx950 int8 matrix cores, with implicit-GEMM
// convolution addressing and the fused reparameterization epilogue.
//
//   D[p][q] = sum_k P[p][k] * Q[q][k]        (codes are int8 in {-1,0,+1})
//
// One kernel serves both entry points through its two operands:
//   GEMM:  P = activation codes (rows m), Q = weight codes (rows n);
//          output [M][N] row-major, lanes run along n.
//   conv:  P = weight codes [O][KH*KW*Cpad], Q = the *virtual* im2col matrix of
//          the channel-innermost activation codes (row = output pixel
//          m = (nb, oh, ow), column = (kh, kw, c)); output NCHW, lanes run
//          along pixels.  A 64-byte K-step never straddles a tap because
//          Cpad % 64 == 0, so a Q row of a K-step is 64 contiguous bytes of one
//          input pixel, or zeros when the tap falls outside the image.
//
// Tiling (wave64, v_mfma_i32_32x32x32_i8): a 256-thread block owns a BP x BQ
// output tile, its 4 waves a WGP x WGQ grid of (BP/WGP) x (BQ/WGQ) sub-tiles
// made of 32x32 MFMA tiles.  K advances 64 bytes per step (two MFMA k-slices).
// Operand tiles are staged global -> registers -> LDS with the next step's
// global loads in flight during the current step's MFMAs; two LDS stages, one
// barrier per step.  LDS rows are 64 bytes; the four 16-byte chunks of a row
// are XOR-swizzled by a function of the row so that both the 16-byte stores
// and the 16-byte fragment reads spread over all banks.
#include "epilogue_math.h"
#include "rtn_kernels.h"

namespace rtn {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct TmmParams {
    const int8_t* P;
    const int8_t* Q;
    int RP, RQ;        // valid rows of the P / Q operand
    int64_t ldP, ldQ;  // row pitch in bytes (dense operands)
    int nk;            // number of 64-byte K-steps
    int tilesP;        // number of tiles along P
    int Klogical;      // K of the epilogue's constant term (GEMM)
    ConvGeom g;        // conv only
    int32_t* acc;
    float* y;
    const int32_t* sw_cls;
    EpiArgs ep;
};

__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 3) ^ ((row >> 3) & 1); }

// Per output pixel: Sa = sum of the input-pixel channel sums over the in-bounds
// taps, Kv = C * (number of taps that count), cls = index of the border class
// whose filter sums apply.  With code-zero padding every tap counts.
__device__ __forceinline__ void pixel_terms(const ConvGeom& g, const int32_t* pix_sums, int nb, int pix,
                                         int& Sa, int& Kv, int& cls)
{
    const int oh = pix / g.OW, ow = pix - oh * g.OW;
    int khl, khh, kwl, kwh;
    tap_range(oh, g.stride, g.pad, g.KH, g.H, khl, khh);
    tap_range(ow, g.stride, g.pad, g.KW, g.W, kwl, kwh);
    const int32_t* ps = pix_sums + (int64_t)nb * g.H * g.W;
    int s = 0;
    for (int kh = khl; kh <= khh; ++kh)
        for (int kw = kwl; kw <= kwh; ++kw)
            s += ps[(oh * g.stride - g.pad + kh) * g.W + (ow * g.stride - g.pad + kw)];
    if (g.code_zero_pad) {
        khl = 0, khh = g.KH - 1, kwl = 0, kwh = g.KW - 1;
    }
    Sa = s;
    Kv = g.C * (khh - khl + 1) * (kwh - kwl + 1);
    cls = ((khl * g.KH + khh) * g.KW + kwl) * g.KW + kwh;
}

template <int BP, int BQ, int WGP, int WGQ, bool CONV>
__global__ __launch_bounds__(256) void k_tmm(TmmParams prm)
{
    static_assert(WGP * WGQ == 4, "4 waves per block");
    constexpr int WP = BP / WGP, WQ = BQ / WGQ, TP = WP / 32, TQ = WQ / 32;
    constexpr int LP = BP / 64, LQ = BQ / 64;  // 16-byte chunks per thread per K-step
    static_assert(TP >= 1 && TQ >= 1 && LP >= 1 && LQ >= 1, "tile too small");
    constexpr int STAGE_P = BP * 64, STAGE_Q = BQ * 64;

    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    int8_t* sP = smem;
    int8_t* sQ = smem + 2 * STAGE_P;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wp = wave / WGQ, wq = wave % WGQ;
    const int tileP = blockIdx.x % prm.tilesP, tileQ = blockIdx.x / prm.tilesP;
    const int p0 = tileP * BP, q0 = tileQ * BQ;
    const ConvGeom& g = prm.g;

    // ---- loader state ------------------------------------------------------
    const int8_t* gP[LP];
    bool okP[LP];
    int ldsP[LP];
#pragma unroll
    for (int i = 0; i < LP; ++i) {
        const int cid = tid + 256 * i, row = cid >> 2, c = cid & 3;
        okP[i] = p0 + row < prm.RP;
        gP[i] = prm.P + (int64_t)(p0 + row) * prm.ldP + c * 16;
        ldsP[i] = row * 64 + ((c ^ swz(row)) << 4);
    }
    const int8_t* gQ[LQ];
    bool okQ[LQ];
    int ldsQ[LQ];
    int ih0[LQ], iw0[LQ];  // conv: input coordinates of tap (0,0)
#pragma unroll
    for (int i = 0; i < LQ; ++i) {
        const int cid = tid + 256 * i, row = cid >> 2, c = cid & 3;
        okQ[i] = q0 + row < prm.RQ;
        ldsQ[i] = row * 64 + ((c ^ swz(row)) << 4);
        if (CONV) {
            const int m = okQ[i] ? q0 + row : 0;
            const int ohw = g.OH * g.OW;
            const int nb = m / ohw, pix = m - nb * ohw;
            const int oh = pix / g.OW, ow = pix - oh * g.OW;
            ih0[i] = oh * g.stride - g.pad;
            iw0[i] = ow * g.stride - g.pad;
            gQ[i] = prm.Q + (int64_t)nb * g.H * g.W * g.Cpad + c * 16;
        } else {
            ih0[i] = iw0[i] = 0;
            gQ[i] = prm.Q + (int64_t)(q0 + row) * prm.ldQ + c * 16;
        }
    }
    // conv: position of the next K-step to load, as (kh, kw, channel offset)
    int l_kh = 0, l_kw = 0, l_cc = 0;

    v4i rP[LP], rQ[LQ];
    const v4i zero4 = {0, 0, 0, 0};

    auto load_step = [&](int kt) {
#pragma unroll
        for (int i = 0; i < LP; ++i)
            rP[i] = okP[i] ? *(const v4i*)(gP[i] + (int64_t)kt * 64) : zero4;
        if (CONV) {
#pragma unroll
            for (int i = 0; i < LQ; ++i) {
                const int ih = ih0[i] + l_kh, iw = iw0[i] + l_kw;
                const bool ok = okQ[i] && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
                const int64_t off = ((int64_t)ih * g.W + iw) * g.Cpad + l_cc;
                rQ[i] = ok ? *(const v4i*)(gQ[i] + off) : zero4;
            }
            l_cc += 64;
            if (l_cc == g.Cpad) {
                l_cc = 0;
                if (++l_kw == g.KW) {
                    l_kw = 0;
                    ++l_kh;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < LQ; ++i)
                rQ[i] = okQ[i] ? *(const v4i*)(gQ[i] + (int64_t)kt * 64) : zero4;
        }
    };
    auto store_step = [&](int stage) {
#pragma unroll
        for (int i = 0; i < LP; ++i) *(v4i*)(sP + stage * STAGE_P + ldsP[i]) = rP[i];
#pragma unroll
        for (int i = 0; i < LQ; ++i) *(v4i*)(sQ + stage * STAGE_Q + ldsQ[i]) = rQ[i];
    };

    // ---- fragment addressing ------------------------------------------------
    // Lane l of an MFMA operand holds row (l & 31), 16 consecutive k-bytes of
    // the k-slice at chunk (l >> 5); both operands use the same k pairing.
    int fragP[TP][2], fragQ[TQ][2];
#pragma unroll
    for (int t = 0; t < TP; ++t) {
        const int row = wp * WP + t * 32 + (lane & 31);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) fragP[t][ks] = row * 64 + (((ks * 2 + (lane >> 5)) ^ swz(row)) << 4);
    }
#pragma unroll
    for (int t = 0; t < TQ; ++t) {
        const int row = wq * WQ + t * 32 + (lane & 31);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) fragQ[t][ks] = row * 64 + (((ks * 2 + (lane >> 5)) ^ swz(row)) << 4);
    }

    v16i acc[TP][TQ];
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
        for (int j = 0; j < TQ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // ---- main loop ------------------------------------------------------------
    load_step(0);
    store_step(0);
    __syncthreads();
    for (int kt = 0; kt < prm.nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < prm.nk;
        if (more) load_step(kt + 1);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i fa[TP], fb[TQ];
#pragma unroll
            for (int t = 0; t < TP; ++t) fa[t] = *(const v4i*)(sP + cur * STAGE_P + fragP[t][ks]);
#pragma unroll
            for (int t = 0; t < TQ; ++t) fb[t] = *(const v4i*)(sQ + cur * STAGE_Q + fragQ[t][ks]);
#pragma unroll
            for (int i = 0; i < TP; ++i)
#pragma unroll
                for (int j = 0; j < TQ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_step(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue ---------------------------------------------------------------
    // acc[i][j][r] is D at P-row  wp*WP + i*32 + 8*(r/4) + 4*(lane/32) + r%4
    //                  and Q-row  wq*WQ + j*32 + lane%32.
    const EpiArgs& ep = prm.ep;
    const bool has_bn = ep.bn_scale != nullptr;
    if (!CONV) {
        const int64_t N = prm.RQ;
        int ncol[TQ];
        bool nok[TQ];
        double aw[TQ], bw[TQ], bs[TQ], bh[TQ];
        int Sw[TQ];
#pragma unroll
        for (int j = 0; j < TQ; ++j) {
            ncol[j] = q0 + wq * WQ + j * 32 + (lane & 31);
            nok[j] = ncol[j] < prm.RQ;
            aw[j] = bw[j] = bs[j] = bh[j] = 0.0;
            Sw[j] = 0;
            if (prm.y && nok[j]) {
                aw[j] = pval(ep.alpha_w, ncol[j]);
                bw[j] = pval(ep.beta_w, ncol[j]);
                Sw[j] = ep.sum_tw[ncol[j]];
                if (has_bn) {
                    bs[j] = ep.bn_scale[ncol[j]];
                    bh[j] = ep.bn_shift ? (double)ep.bn_shift[ncol[j]] : 0.0;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < TP; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = p0 + wp * WP + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const bool mok = m < prm.RP;
                double aa = 0.0, ba = 0.0;
                int Sa = 0;
                if (prm.y && mok) {
                    aa = pval(ep.alpha_a, m);
                    ba = pval(ep.beta_a, m);
                    Sa = ep.sum_ta[m];
                }
#pragma unroll
                for (int j = 0; j < TQ; ++j) {
                    if (mok && nok[j]) {
                        const int D = acc[i][j][r];
                        const int64_t idx = (int64_t)m * N + ncol[j];
                        if (prm.acc) prm.acc[idx] = D;
                        if (prm.y)
                            prm.y[idx] = reparam(aa, ba, aw[j], bw[j], D, Sa, Sw[j], prm.Klogical,
                                                 ep.relu, has_bn, bs[j], bh[j]);
                    }
                }
            }
    } else {
        const int ohw = g.OH * g.OW;
        const double aa = (double)ep.alpha_a.s, ba = (double)ep.beta_a.s;
        bool mok[TQ];
        int Sa[TQ], Kv[TQ], cls[TQ];
        int64_t obase[TQ];
#pragma unroll
        for (int j = 0; j < TQ; ++j) {
            const int m = q0 + wq * WQ + j * 32 + (lane & 31);
            mok[j] = m < prm.RQ;
            const int mm = mok[j] ? m : 0;
            const int nb = mm / ohw, pix = mm - nb * ohw;
            obase[j] = (int64_t)nb * g.O * ohw + pix;
            Sa[j] = Kv[j] = cls[j] = 0;
            if (prm.y) pixel_terms(g, ep.sum_ta, nb, pix, Sa[j], Kv[j], cls[j]);
        }
#pragma unroll
        for (int i = 0; i < TP; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int o = p0 + wp * WP + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const bool ook = o < prm.RP;
                double aw = 0.0, bw = 0.0, bs = 1.0, bh = 0.0;
                if (prm.y && ook) {
                    aw = pval(ep.alpha_w, o);
                    bw = pval(ep.beta_w, o);
                    if (has_bn) {
                        bs = (double)ep.bn_scale[o];
                        bh = ep.bn_shift ? (double)ep.bn_shift[o] : 0.0;
                    }
                }
#pragma unroll
                for (int j = 0; j < TQ; ++j) {
                    if (ook && mok[j]) {
                        const int D = acc[i][j][r];
                        const int64_t idx = obase[j] + (int64_t)o * ohw;
                        if (prm.acc) prm.acc[idx] = D;
                        if (prm.y) {
                            const int Sw = prm.sw_cls[(int64_t)cls[j] * g.O + o];
                            prm.y[idx] = reparam(aa, ba, aw, bw, D, Sa[j], Sw, Kv[j], ep.relu, has_bn, bs, bh);
                        }
                    }
                }
            }
    }
}

// Filter sums per border class.  A class is the in-bounds tap rectangle
// [khl..khh] x [kwl..kwh] of an output pixel; sw_cls[class][o] is the sum of
// the per-tap channel sums of filter o over that rectangle (0 if empty).
__global__ __launch_bounds__(256) void k_conv_class_sums(const int32_t* tap, ConvGeom g, int32_t* sw_cls)
{
    const int ncls = g.KH * g.KH * g.KW * g.KW;
    const int64_t total = (int64_t)ncls * g.O;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int o = (int)(i % g.O);
    int cls = (int)(i / g.O);
    const int kwh = cls % g.KW;
    cls /= g.KW;
    const int kwl = cls % g.KW;
    cls /= g.KW;
    const int khh = cls % g.KH, khl = cls / g.KH;
    int s = 0;
    for (int kh = khl; kh <= khh; ++kh)
        for (int kw = kwl; kw <= kwh; ++kw) s += tap[((int64_t)o * g.KH + kh) * g.KW + kw];
    sw_cls[i] = s;
}

template <int BP, int BQ, int WGP, int WGQ, bool CONV>
hipError_t launch_cfg(TmmParams& prm, hipStream_t st)
{
    constexpr int smem = 2 * (BP + BQ) * 64;
    static bool attr_done = false;
    auto kern = k_tmm<BP, BQ, WGP, WGQ, CONV>;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    prm.tilesP = (prm.RP + BP - 1) / BP;
    const int64_t tilesQ = ((int64_t)prm.RQ + BQ - 1) / BQ;
    const int64_t blocks = (int64_t)prm.tilesP * tilesQ;
    if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), smem, st, prm);
    return hipGetLastError();
}

inline int64_t nblocks(int64_t rp, int64_t rq, int bp, int bq)
{
    return ((rp + bp - 1) / bp) * ((rq + bq - 1) / bq);
}

// Tile configurations, indexed as rtn_set_tile_config() documents.
constexpr int kNumTileConfigs = 6;
int g_forced_tile = -1;

template <bool CONV>
hipError_t launch_index(int cfg, TmmParams& prm, hipStream_t st)
{
    switch (cfg) {
        case 0: return launch_cfg<64, 64, 2, 2, CONV>(prm, st);
        case 1: return launch_cfg<128, 128, 2, 2, CONV>(prm, st);
        case 2: return launch_cfg<256, 256, 2, 2, CONV>(prm, st);
        case 3: return launch_cfg<64, 256, 1, 4, CONV>(prm, st);
        case 4: return launch_cfg<128, 256, 2, 2, CONV>(prm, st);
        case 5: return launch_cfg<256, 128, 2, 2, CONV>(prm, st);
        default: return hipErrorInvalidValue;
    }
}

// Heuristic: the largest tile that still gives every one of the 256 CUs a
// block (two for the tiles small enough to share a CU); P is the operand whose
// rows run along registers (GEMM: M, conv: O), Q along lanes (GEMM: N, conv: pixels).
int pick_tile(int64_t rp, int64_t rq)
{
    if (rp <= 64) return nblocks(rp, rq, 64, 256) >= 512 ? 3 : 0;
    if (rp <= 128) return nblocks(rp, rq, 128, 256) >= 512 ? 4 : (rq > 64 ? 1 : 0);
    if (rq <= 64) return 0;
    if (nblocks(rp, rq, 256, 256) >= 256) return 2;
    if (nblocks(rp, rq, 128, 128) >= 256 || rq > 64) return 1;
    return 0;
}

}  // namespace

int tile_config_count() { return kNumTileConfigs; }
void force_tile_config(int index) { g_forced_tile = index; }

hipError_t launch_conv_class_sums(const int32_t* tap_sums, const ConvGeom& g, int32_t* sw_cls,
                                  hipStream_t st)
{
    const int64_t total = (int64_t)g.KH * g.KH * g.KW * g.KW * g.O;
    hipLaunchKernelGGL(k_conv_class_sums, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       tap_sums, g, sw_cls);
    return hipGetLastError();
}

hipError_t launch_gemm_mfma(const GemmArgs& a, hipStream_t st)
{
    TmmParams prm = {};
    prm.P = a.a;
    prm.Q = a.w;
    prm.RP = (int)a.M;
    prm.RQ = (int)a.N;
    prm.ldP = prm.ldQ = a.Kpad;
    prm.nk = (int)(a.Kpad / 64);
    prm.Klogical = (int)a.K;
    prm.acc = a.acc;
    prm.y = a.y;
    prm.ep = a.ep;
    const int cfg = g_forced_tile >= 0 ? g_forced_tile : pick_tile(a.M, a.N);
    return launch_index<false>(cfg, prm, st);
}

hipError_t launch_conv_mfma(const ConvArgs& a, hipStream_t st)
{
    const ConvGeom& g = a.g;
    TmmParams prm = {};
    prm.P = a.w;
    prm.Q = a.a;
    prm.RP = g.O;
    prm.RQ = g.Nb * g.OH * g.OW;
    prm.ldP = (int64_t)g.KH * g.KW * g.Cpad;
    prm.ldQ = 0;
    prm.nk = (int)(prm.ldP / 64);
    prm.Klogical = g.C * g.KH * g.KW;
    prm.g = g;
    prm.acc = a.acc;
    prm.y = a.y;
    prm.sw_cls = a.sw_cls;
    prm.ep = a.ep;
    const int cfg = g_forced_tile >= 0 ? g_forced_tile : pick_tile(g.O, prm.RQ);
    return launch_index<true>(cfg, prm, st);
}

}  // namespace rtn
