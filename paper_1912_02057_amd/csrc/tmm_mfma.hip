// Host side of the matrix-core contraction: tile choice and the launch functions of the
// GEMM, the conv and the weight-only forms, plus the small kernels around them -- the
// conv's per-layer epilogue table, the fp32 -> 3 x bf16 splits and the int8 -> bf16
// weight copy.  The contraction kernel itself is in tmm_kernel.h.
#include <cstdlib>

#include "tmm_kernel.h"

namespace rtn {

namespace {

// The per-layer table of the conv epilogue, [4 + classes][OP] doubles with the
// row pitch OP = O rounded up to even (16-byte rows for the direct loads):
//   row 0: g1[o] = aa*aw[o]      row 1: c2[o] = aa*bw[o]
//   row 2: bn scale (1 if none)  row 3: bn shift (0 if none)
//   row 4 + class: the constant of the reparameterization for that border class.
// A class is the in-bounds tap rectangle [khl..khh] x [kwl..kwh] of an output pixel,
//   class = rid * (pad+1)^2 + cid,  rid = khl + (pad+1)*(KH-1-khh),  cid = kwl + (pad+1)*(KW-1-kwh)
// (both cuts are at most pad, so there are (pad+1)^4 classes; class 0 is the
// interior).    cst[class][o] = ba*aw[o]*Sw + Kv*ba*bw[o]
// with Sw the sum of filter o's per-tap channel sums over the rectangle and
// Kv = C * (number of taps in it): Eq.9's pre-stored constant C, one per class.
__global__ __launch_bounds__(256) void k_conv_class_consts(const int32_t* tap, ConvGeom g, EpiArgs ep, double* cst)
{
    const int p1 = g.pad + 1;
    const int nrows = 4 + conv_classes(g.pad), opitch = (g.O + 1) & ~1;
    const int64_t total = (int64_t)nrows * opitch;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int o = (int)(i % opitch);
    const int row = (int)(i / opitch);
    double v = 0.0;
    if (o < g.O) {
        const double aa = (double)ep.alpha_a.s, ba = (double)ep.beta_a.s;
        if (row == 0) {
            v = aa * pval(ep.alpha_w, o);
        } else if (row == 1) {
            v = aa * pval(ep.beta_w, o);
        } else if (row == 2) {
            v = ep.bn_scale ? (double)ep.bn_scale[o] : 1.0;
        } else if (row == 3) {
            v = (ep.bn_scale && ep.bn_shift) ? (double)ep.bn_shift[o] : 0.0;
        } else {
            const int cls = row - 4;
            const int rid = cls / (p1 * p1), cid = cls % (p1 * p1);
            const int khl = rid % p1, khh = g.KH - 1 - rid / p1;
            const int kwl = cid % p1, kwh = g.KW - 1 - cid / p1;
            int s = 0, taps = 0;
            for (int kh = khl; kh <= khh; ++kh)
                for (int kw = kwl; kw <= kwh; ++kw) {
                    s += tap ? tap[((int64_t)o * g.KH + kh) * g.KW + kw] : 0;
                    ++taps;
                }
            v = ba * pval(ep.alpha_w, o) * (double)s + (double)(g.C * taps) * ba * pval(ep.beta_w, o);
        }
    }
    cst[i] = v;
}

inline int64_t nblocks(int64_t rp, int64_t rq, int bp, int bq)
{
    return ((rp + bp - 1) / bp) * ((rq + bq - 1) / bq);
}

int g_forced_tile = -1;

// A configuration whose LDS need (ring + the conv's table, which grows with the
// pad) exceeds the CU's falls back to the smallest tile.
template <bool CONV, int TERN = 0, int DT = 0>
hipError_t launch_index(int cfg, TmmParams& prm, hipStream_t st)
{
    hipError_t e = tmm_launch_index_raw<CONV, TERN, DT>(cfg, prm, st);
    if (e == hipErrorInvalidValue && cfg != 0) e = tmm_launch_index_raw<CONV, TERN, DT>(0, prm, st);
    return e;
}

// Heuristic: the largest tile that still gives every one of the 256 CUs a
// block (two for the tiles small enough to share a CU); P is the operand whose
// rows run along registers (GEMM: M, conv: O), Q along lanes (GEMM: N, conv: pixels).
// The conv rules come from timing the ResNet-18 layer shapes at batch 256: a
// grid that fits the chip in one round beats a finer one that needs a second,
// and the short-K layers prefer more resident blocks over a deeper ring.
int pick_tile(int64_t rp, int64_t rq, bool conv)
{
    if (rp <= 64) return nblocks(rp, rq, 64, 256) >= 512 ? 7 : 0;
    if (conv) {
        const int64_t t256 = nblocks(rp, rq, 128, 256), t128 = nblocks(rp, rq, 128, 128);
        if (t256 >= 256 && t256 <= 512) return 13;
        if (t128 >= 1024) return 12;
        if (t128 >= 256 || rq > 64) return 1;
        return 0;
    }
    if (rp <= 128) return nblocks(rp, rq, 128, 256) >= 512 ? 4 : (rq > 64 ? 1 : 0);
    if (rq <= 64) return 0;
    if (nblocks(rp, rq, 256, 256) >= 256) return 2;
    if (nblocks(rp, rq, 128, 128) >= 256 || rq > 64) return 1;
    return 0;
}

}  // namespace

int tile_config_count() { return kNumTileConfigs; }
void force_tile_config(int index) { g_forced_tile = index; }

hipError_t launch_conv_class_consts(const ConvArgs& a, double* cst, hipStream_t st)
{
    const ConvGeom& g = a.g;
    const int64_t total = (int64_t)(4 + conv_classes(g.pad)) * ((g.O + 1) & ~1);
    hipLaunchKernelGGL(k_conv_class_consts, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       a.ep.sum_tw, g, a.ep, cst);
    return hipGetLastError();
}

hipError_t launch_gemm_mfma(const GemmArgs& a, hipStream_t st)
{
    TmmParams prm = {};
    prm.P = a.a;
    prm.Q = a.w;
    prm.RP = (int)a.M;
    prm.RQ = (int)a.N;
    prm.ldP = prm.ldQ = a.fp4 ? a.Kpad / 2 : a.Kpad;  // bytes per row
    prm.nk = (int)(prm.ldP / 64);
    prm.Klogical = (int)a.K;
    prm.acc = a.acc;
    prm.y = a.y;
    prm.ep = a.ep;
    const int cfg = g_forced_tile >= 0 ? g_forced_tile : pick_tile(a.M, a.N, false);
    return a.fp4 ? launch_index<false, 0, 2>(cfg, prm, st) : launch_index<false>(cfg, prm, st);
}

// ---- weight-only ternary GEMM: fp32 activations x (alpha * t_w) ----------------
// bf16 round-to-nearest-even of an fp32 value, as bits
__device__ __forceinline__ unsigned bf16_rn(float v)
{
    const unsigned u = __float_as_uint(v);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// x = hi + mid + lo with three bf16 terms: each residual is exact in fp32 and at most
// half an ulp of the term before it, so 8 + 8 + 8 significand bits cover fp32's 24.
// out: [M][3 * Kpad] bf16, the three terms of a row side by side, zero beyond K.
__global__ __launch_bounds__(256) void k_split_bf16x3(const float* x, int64_t M, int K, int Kpad, uint16_t* out)
{
    // one thread: 8 consecutive k of one row -> three 16-byte stores
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int per_row = Kpad / 8;
    if (i >= M * per_row) return;
    const int64_t m = i / per_row;
    const int k0 = (int)(i - m * per_row) * 8;
    float v[8];
    const float* src = x + m * K + k0;
    if (k0 + 8 <= K && (K & 3) == 0 && ((uintptr_t)x & 15) == 0) {
        const float4 a = *(const float4*)src, b = *(const float4*)(src + 4);
        v[0] = a.x, v[1] = a.y, v[2] = a.z, v[3] = a.w, v[4] = b.x, v[5] = b.y, v[6] = b.z, v[7] = b.w;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = k0 + e < K ? src[e] : 0.0f;
    }
    unsigned h[8], md[8], lo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        h[e] = bf16_rn(v[e]);
        const float r1 = v[e] - __uint_as_float(h[e] << 16);
        md[e] = bf16_rn(r1);
        const float r2 = r1 - __uint_as_float(md[e] << 16);
        lo[e] = bf16_rn(r2);
    }
    auto pack8 = [](const unsigned* t) {
        return make_uint4(t[0] | (t[1] << 16), t[2] | (t[3] << 16), t[4] | (t[5] << 16), t[6] | (t[7] << 16));
    };
    uint16_t* row = out + m * 3 * (int64_t)Kpad + k0;
    *(uint4*)row = pack8(h);
    *(uint4*)(row + Kpad) = pack8(md);
    *(uint4*)(row + 2 * Kpad) = pack8(lo);
}

// int8 codes [N][Kpad] -> the same values as bf16 (-1, 0, +1 are exact); 16 codes per thread
__global__ __launch_bounds__(256) void k_codes_to_bf16(const int8_t* codes, int64_t n16, uint16_t* out)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    const uint4 c = *(const uint4*)(codes + i * 16);
    const unsigned w[4] = {c.x, c.y, c.z, c.w};
    unsigned o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int t0 = (int8_t)(w[e >> 1] >> (16 * (e & 1))), t1 = (int8_t)(w[e >> 1] >> (16 * (e & 1) + 8));
        const unsigned b0 = t0 > 0 ? 0x3f80u : (t0 < 0 ? 0xbf80u : 0u), b1 = t1 > 0 ? 0x3f80u : (t1 < 0 ? 0xbf80u : 0u);
        o[e] = b0 | (b1 << 16);
    }
    uint4* dst = (uint4*)(out + i * 16);
    dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
    dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
}

// The same split for an NCHW activation tensor, written channel-innermost as the conv
// reads it: out[plane][pixel][Cpad] bf16, plane 0 = hi, 1 = mid, 2 = lo, planes
// `plane_elems` apart, channels C .. Cpad-1 zero.  A block transposes 64 pixels x 64
// channels through LDS: lanes run along pixels for the fp32 reads (256 contiguous
// bytes per channel) and along channels for the stores (128 contiguous bytes per pixel
// and plane).  LDS rows are 33 dwords (two bf16 per dword), so both phases are free of
// bank conflicts.
__global__ __launch_bounds__(256) void k_split_nchw_bf16x3(const float* x, int64_t Nb, int C, int Cpad, int HW,
                                                           int64_t plane_elems, uint16_t* out)
{
    __shared__ unsigned tile[3][64][33];
    const int64_t npix = Nb * HW;
    const int64_t pix0 = (int64_t)blockIdx.x * 64;
    const int c0 = (int)blockIdx.y * 64;
    const int tid = threadIdx.x;
    {
        const int p = tid & 63, cg = tid >> 6;  // this thread: pixel p, channels c0 + 16 cg .. + 15
        const int64_t pix = pix0 + p;
        const bool pok = pix < npix;
        const int64_t nb = pok ? pix / HW : 0;
        const int q = pok ? (int)(pix - nb * HW) : 0;
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
            unsigned w[3] = {0, 0, 0};
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int c = c0 + 16 * cg + e + s;
                const float v = (pok && c < C) ? x[(nb * C + c) * HW + q] : 0.0f;
                const unsigned h = bf16_rn(v);
                const float r1 = v - __uint_as_float(h << 16);
                const unsigned md = bf16_rn(r1);
                const float r2 = r1 - __uint_as_float(md << 16);
                const unsigned lo = bf16_rn(r2);
                w[0] |= h << (16 * s);
                w[1] |= md << (16 * s);
                w[2] |= lo << (16 * s);
            }
#pragma unroll
            for (int pl = 0; pl < 3; ++pl) tile[pl][p][8 * cg + e / 2] = w[pl];
        }
    }
    __syncthreads();
    // 3 planes x 64 pixels x 8 sixteen-byte parts = 1536 stores, 6 per thread
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        const int u = tid + 256 * i;
        const int pl = u >> 9, p = (u >> 3) & 63, part = u & 7;
        const int64_t pix = pix0 + p;
        if (pix >= npix) continue;
        const unsigned* src = &tile[pl][p][4 * part];
        *(uint4*)(out + pl * plane_elems + pix * Cpad + c0 + 8 * part) = make_uint4(src[0], src[1], src[2], src[3]);
    }
}

// table position behind wn bf16 weights
static double* wconv_table(uint16_t* wb, int64_t wn) { return (double*)(((uintptr_t)(wb + wn) + 15) & ~(uintptr_t)15); }

hipError_t launch_wconv_prepare(const int8_t* w, const ConvGeom& g0, const EpiArgs& ep, void* prepared, hipStream_t st)
{
    uint16_t* wb = (uint16_t*)prepared;
    const int64_t wn = (int64_t)g0.O * g0.KH * g0.KW * g0.Cpad;
    hipLaunchKernelGGL(k_codes_to_bf16, dim3((unsigned)((wn / 16 + 255) / 256)), dim3(256), 0, st, w, wn / 16, wb);
    ConvArgs c = {};
    c.g = g0;
    c.ep = ep;
    return launch_conv_class_consts(c, wconv_table(wb, wn), st);  // g1 = alpha_w, BN rows; the class constants are 0
}

hipError_t launch_wconv(const WConvArgs& a, hipStream_t st)
{
    const ConvGeom& g0 = a.g;  // Cpad in elements here
    const int64_t npix = (int64_t)g0.Nb * g0.H * g0.W;
    const int64_t plane = npix * g0.Cpad;
    uint16_t* a3 = (uint16_t*)a.workspace;
    uint16_t* wb = a.prepared ? (uint16_t*)a.prepared : a3 + 3 * plane;
    const int64_t wn = (int64_t)g0.O * g0.KH * g0.KW * g0.Cpad;
    double* tab = wconv_table(wb, wn);
    hipLaunchKernelGGL(k_split_nchw_bf16x3, dim3((unsigned)((npix + 63) / 64), (unsigned)(g0.Cpad / 64)), dim3(256), 0,
                       st, a.x, (int64_t)g0.Nb, g0.C, g0.Cpad, g0.H * g0.W, plane, a3);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && !a.prepared) e = launch_wconv_prepare(a.w, g0, a.ep, wb, st);
    if (e != hipSuccess) return e;
    TmmParams prm = {};
    prm.g = g0;
    prm.g.Cpad = g0.Cpad * 2;  // bytes per pixel row: the kernel's K bookkeeping is in bytes
    prm.P = (const int8_t*)wb;
    prm.Q = (const int8_t*)a3;
    prm.RP = g0.O;
    prm.RQ = (int)((int64_t)g0.Nb * g0.OH * g0.OW);
    prm.ldP = (int64_t)g0.KH * g0.KW * g0.Cpad * 2;
    prm.wwrap = (unsigned)prm.ldP;
    prm.qplane = plane * 2;
    prm.nk = (int)(3 * prm.ldP / 64);
    prm.Klogical = g0.C * g0.KH * g0.KW;
    prm.y = a.y;
    prm.cst_cls = tab;
    prm.ep = a.ep;
    const int cfg = g_forced_tile >= 0 ? g_forced_tile : pick_tile(g0.O, prm.RQ, true);
    const int bp = kTileBP[cfg];
    e = hipErrorInvalidValue;
    if (cfg == 13 || cfg == 4 || cfg == 19)
        e = tmm_launch_bf16(true, 2, prm, st);
    else if (bp >= 128)
        e = tmm_launch_bf16(true, 1, prm, st);
    else if (cfg == 3 || cfg == 7 || cfg == 9 || cfg == 14 || cfg == 15)
        e = tmm_launch_bf16(true, 3, prm, st);
    // the smallest tile also serves a table too large for the others (wide pad, tiny image)
    if (e == hipErrorInvalidValue) e = tmm_launch_bf16(true, 0, prm, st);
    return e;
}

hipError_t launch_wgemm_prepare(const int8_t* w, int64_t N, int64_t Kpad, void* prepared, hipStream_t st)
{
    const int64_t nw = N * Kpad / 16;
    hipLaunchKernelGGL(k_codes_to_bf16, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, st, w, nw, (uint16_t*)prepared);
    return hipGetLastError();
}

hipError_t launch_wgemm(const WGemmArgs& a, hipStream_t st)
{
    uint16_t* a3 = (uint16_t*)a.workspace;
    uint16_t* wb = a.prepared ? (uint16_t*)a.prepared : a3 + (size_t)a.M * 3 * a.Kpad;
    const int64_t na = a.M * a.Kpad / 8;
    hipLaunchKernelGGL(k_split_bf16x3, dim3((unsigned)((na + 255) / 256)), dim3(256), 0, st, a.x, a.M, (int)a.K,
                       (int)a.Kpad, a3);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && !a.prepared) e = launch_wgemm_prepare(a.w, a.N, a.Kpad, wb, st);
    if (e != hipSuccess) return e;
    TmmParams prm = {};
    prm.P = (const int8_t*)a3;
    prm.Q = (const int8_t*)wb;
    prm.RP = (int)a.M;
    prm.RQ = (int)a.N;
    prm.ldP = 3 * a.Kpad * 2;
    prm.ldQ = a.Kpad * 2;
    prm.wwrap = (unsigned)(a.Kpad * 2);
    prm.nk = (int)(prm.ldP / 64);
    prm.Klogical = (int)a.K;
    prm.y = a.y;
    prm.ep = a.ep;
    const int cfg = g_forced_tile >= 0 ? g_forced_tile : pick_tile(a.M, a.N, false);
    return tmm_launch_bf16(false, kTileBP[cfg] >= 256 ? 2 : (kTileBP[cfg] >= 128 ? 1 : 0), prm, st);
}

hipError_t launch_conv_mfma(const ConvArgs& a, hipStream_t st)
{
    const ConvGeom& g = a.g;
    TmmParams prm = {};
    prm.P = a.w;
    prm.Q = a.a;
    prm.RP = g.O;
    prm.RQ = g.Nb * g.OH * g.OW;
    prm.g = g;
    if (a.fp4) prm.g.Cpad = g.Cpad / 2;  // the kernel's K bookkeeping is in bytes
    prm.ldP = (int64_t)g.KH * g.KW * prm.g.Cpad;
    prm.ldQ = 0;
    prm.nk = (int)(prm.ldP / 64);
    prm.Klogical = g.C * g.KH * g.KW;
    prm.acc = a.acc;
    prm.y = a.y;
    prm.cst_cls = a.cst_cls;
    prm.ep = a.ep;
    prm.codes = a.codes;
    prm.ldc = a.ldc;
    prm.thr_lo = a.thr_lo;
    prm.thr_hi = a.thr_hi;
    prm.res = a.res;
    prm.relu_out = a.relu_out;
    // outputs beyond what stays in the memory-side cache take the non-temporal hint
    {
        const int64_t out_bytes = (int64_t)g.Nb * g.O * g.OH * g.OW * 4 * ((a.acc ? 1 : 0) + (a.y ? 1 : 0));
        prm.nt_out = out_bytes > (int64_t)128 << 20;
    }
    int cfg = g_forced_tile >= 0 ? g_forced_tile : pick_tile(g.O, prm.RQ, true);
    // a 64-filter layer with a centred stride-1 window: the variant that keeps the
    // tile's input pixel run in LDS (measured faster there; on par or slower elsewhere)
    if (g_forced_tile < 0 && cfg == 7 && halo_eligible(prm, 64)) cfg = 15;
    // ... and up to 128 filters (FP4 codes: 128 channels are 64 bytes per pixel) the 64 x 128 form of it
    // Two more choices measured on the 128- and 512-filter layers (not for the block-tail
    // epilogue, which prefers the deeper ring): the two-stage ring with four blocks per CU
    // instead of the three-stage one, and, up to 128 filters with 64-byte pixels (FP4
    // codes: 128 channels), the 64 x 128 form of the pixel-run variant.
    const bool tail_form = a.codes && (a.res != nullptr || a.y != nullptr || a.relu_out);
    if (g_forced_tile < 0 && !tail_form) {
        if (cfg == 1 && nblocks(g.O, prm.RQ, 128, 128) >= 256) cfg = 12;
        if (cfg == 12 && g.O <= 128 && halo_eligible(prm, 64)) cfg = 17;
    }
    if (!a.codes) return a.fp4 ? launch_index<true, 0, 2>(cfg, prm, st) : launch_index<true>(cfg, prm, st);
    const bool tail = a.res != nullptr || a.y != nullptr || a.relu_out;
    // the block-tail epilogue prefetches its residual values only for the tiles with
    // 64 accumulators per lane: prefer 128x128 over 128x256 there
    if (tail && g_forced_tile < 0 && cfg == 13) cfg = 12;
    // FP4 block tails, from a sweep over all configurations on the ResNet-18 shapes: the pixel-run
    // tile with the whole 9-step weight slab resident (123.5 against 126.9 us on the 64-filter
    // layers), and the two-stage 128 x 128 ring on the 512-filter layers (40.6 against 42.4 us)
    if (tail && a.fp4 && g_forced_tile < 0) {
        if (cfg == 15 && prm.nk <= 9) cfg = 14;
        if (cfg == 1 && nblocks(g.O, prm.RQ, 128, 128) >= 256) cfg = 12;
    }
    if (a.fp4) return tail ? launch_index<true, 2, 2>(cfg, prm, st) : launch_index<true, 1, 2>(cfg, prm, st);
    return tail ? launch_index<true, 2>(cfg, prm, st) : launch_index<true, 1>(cfg, prm, st);
}

}  // namespace rtn
