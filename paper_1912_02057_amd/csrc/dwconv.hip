// Depthwise ternary convolution (one k x k ternary filter per channel; the 3x3 layers of
// MobileNet, one of the networks the paper evaluates) with the per-channel four-term
// reparameterization.  A dot product here has only k*k terms, so there is nothing for the
// matrix cores to do: the kernel is a streaming one, 1 byte read and 4 bytes written per
// output.  A block owns 64 consecutive output pixels x 64 channels.  In the compute phase
// lanes run along channels -- the codes are channel-innermost, so a thread's dword is 4
// channels of one input pixel and 16 threads read 64 contiguous bytes -- and a thread forms
// its 4 pixels x 4 channels; the results cross an LDS tile so that in the store phase lanes
// run along pixels, where the NCHW output of a channel is contiguous.
#include "epilogue_math.h"
#include "rtn_kernels.h"

namespace rtn {

namespace {

constexpr int DW_PX = 64, DW_CH = 64, DW_PITCH = DW_PX + 1;  // LDS tile [channel][pixel], padded

// Byte e of each of four dwords -> one dword (a 4 x 4 byte transpose, one row of it).
__device__ __forceinline__ int gather_byte(int w0, int w1, int w2, int w3, int e)
{
    const unsigned sel = 0x04000400u + 0x00000101u * (unsigned)e;  // bytes: lo[e], hi[e] of each pair
    const unsigned p01 = __builtin_amdgcn_perm((unsigned)w1, (unsigned)w0, 0x0c0c0400u + 0x00000101u * (unsigned)e);
    const unsigned p23 = __builtin_amdgcn_perm((unsigned)w3, (unsigned)w2, 0x0c0c0400u + 0x00000101u * (unsigned)e);
    (void)sel;
    return (int)(p01 | (p23 << 16));
}

// KS = 3: the 3 x 3 window unrolled.  The nine taps of a channel are gathered into three dwords
// (byte transposes of the fetched code words), so that D, Sa and Sw of a channel are three
// 4-way byte dot products each: against the channel's filter codes, against ones, and of the
// filter codes against the per-pixel mask of taps that count.  KS = 0: any window, one tap and
// one channel at a time.
template <int KS>
__global__ __launch_bounds__(256) void k_dwconv(DwConvArgs a)
{
    __shared__ int tD[DW_CH * DW_PITCH];
    __shared__ float tY[DW_CH * DW_PITCH];
    const ConvGeom& g = a.g;
    const int tid = threadIdx.x;
    const int64_t ohw = (int64_t)g.OH * g.OW, total = (int64_t)g.Nb * ohw;
    const int64_t m0 = (int64_t)blockIdx.x * DW_PX;
    const int cb = (int)blockIdx.y * DW_CH;  // first channel of this block's slab
    const EpiArgs& ep = a.ep;
    const bool has_bn = ep.bn_scale != nullptr;
    const double aa = (double)ep.alpha_a.s, ba = (double)ep.beta_a.s;
    {
        const int cq = tid & 15, pg = tid >> 4;  // channels cb + 4 cq .. + 3, pixels m0 + 4 pg .. + 3
        const int c0 = cb + 4 * cq;
        const int KH = KS ? KS : g.KH, KW = KS ? KS : g.KW;
        // 3 x 3: the filter codes of each channel as three dwords (taps 0-3, 4-7, 8), read from the
        // channel's row of tap codes (the row is padded with zeros)
        int wq[4][3];
        if (KS) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int c = c0 + e < g.C ? c0 + e : g.C - 1;
                const int* wr = (const int*)(a.w + (int64_t)c * a.Kp);
                const bool cok = c0 + e < g.C;
                wq[e][0] = cok ? wr[0] : 0;
                wq[e][1] = cok ? wr[1] : 0;
                wq[e][2] = cok ? (wr[2] & 0xff) : 0;
            }
        }
        double awv[4], bwv[4], bsv[4], bhv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int c = c0 + e < g.C ? c0 + e : g.C - 1;
            awv[e] = pval(ep.alpha_w, c);
            bwv[e] = pval(ep.beta_w, c);
            bsv[e] = has_bn ? (double)ep.bn_scale[c] : 1.0;
            bhv[e] = (has_bn && ep.bn_shift) ? (double)ep.bn_shift[c] : 0.0;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int pl = 4 * pg + q;
            const int64_t m = m0 + pl;
            const bool mok = m < total;
            const int64_t mm = mok ? m : 0;
            // (Nb*OH*OW < 2^31: divisions by host-made magic numbers)
            const int nb = (int)fastdiv((uint32_t)mm, g.div_ohw), pix = (int)(mm - (int64_t)nb * ohw);
            const int oh = (int)fastdiv((uint32_t)pix, g.div_ow), ow = pix - oh * g.OW;
            const int ih0 = oh * g.stride - g.pad, iw0 = ow * g.stride - g.pad;
            const int8_t* img = a.a + (int64_t)nb * g.H * g.W * g.Cpad + c0;
            int d[4] = {0, 0, 0, 0}, sa[4] = {0, 0, 0, 0}, sw[4] = {0, 0, 0, 0};
            int kv = 0;
            if (KS) {
                // All taps are fetched first, from coordinates clamped into the image (every load is
                // in bounds and nothing waits between them); a tap outside the image is zeroed after.
                int words[12];
                unsigned cnt[3] = {0, 0, 0};  // byte t of cnt[t / 4]: 1 if tap t counts for Sw and Kv
#pragma unroll
                for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                    for (int kw = 0; kw < 3; ++kw) {
                        const int ih = min(max(ih0 + kh, 0), g.H - 1), iw = min(max(iw0 + kw, 0), g.W - 1);
                        words[kh * 3 + kw] = *(const int*)(img + ((int64_t)ih * g.W + iw) * g.Cpad);
                    }
#pragma unroll
                for (int t = 0; t < 9; ++t) {
                    const int kh = t / 3, kw = t % 3;
                    const bool inb = (unsigned)(ih0 + kh) < (unsigned)g.H && (unsigned)(iw0 + kw) < (unsigned)g.W;
                    words[t] = inb ? words[t] : 0;
                    const bool counts = inb || g.code_zero_pad;
                    kv += counts;
                    cnt[t >> 2] |= (unsigned)counts << (8 * (t & 3));
                }
                words[9] = words[10] = words[11] = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
#pragma unroll
                    for (int h = 0; h < 3; ++h) {
                        const int av = gather_byte(words[4 * h], words[4 * h + 1], words[4 * h + 2], words[4 * h + 3], e);
                        d[e] = __builtin_amdgcn_sdot4(av, wq[e][h], d[e], false);
                        sa[e] = __builtin_amdgcn_sdot4(av, 0x01010101, sa[e], false);
                        sw[e] = __builtin_amdgcn_sdot4(wq[e][h], (int)cnt[h], sw[e], false);
                    }
                }
            } else {
                for (int kh = 0; kh < KH; ++kh)
                    for (int kw = 0; kw < KW; ++kw) {
                        const bool inb = (unsigned)(ih0 + kh) < (unsigned)g.H && (unsigned)(iw0 + kw) < (unsigned)g.W;
                        const int ih = min(max(ih0 + kh, 0), g.H - 1), iw = min(max(iw0 + kw, 0), g.W - 1);
                        int word = *(const int*)(img + ((int64_t)ih * g.W + iw) * g.Cpad);
                        word = inb ? word : 0;
                        const bool counts = inb || g.code_zero_pad;
                        kv += counts;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int w_ = c0 + e < g.C ? (int)a.w[(int64_t)(c0 + e) * a.Kp + kh * KW + kw] : 0;
                            const int a_ = (int)(int8_t)(word >> (8 * e));
                            d[e] += a_ * w_;
                            sa[e] += a_;
                            sw[e] += counts ? w_ : 0;
                        }
                    }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                tD[(4 * cq + e) * DW_PITCH + pl] = d[e];
                if (a.y)
                    tY[(4 * cq + e) * DW_PITCH + pl] =
                        reparam(aa, ba, awv[e], bwv[e], d[e], sa[e], sw[e], kv, ep.relu, has_bn, bsv[e], bhv[e]);
            }
        }
    }
    __syncthreads();
    // store phase: lane = pixel, the four waves take the channels round-robin
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t m = m0 + lane;
    if (m >= total) return;
    const int nb = (int)fastdiv((uint32_t)m, g.div_ohw), pix = (int)(m - (int64_t)nb * ohw);
    for (int cl = wave; cl < DW_CH; cl += 4) {
        const int c = cb + cl;
        if (c >= g.C) break;
        const int64_t i = ((int64_t)nb * g.C + c) * ohw + pix;
        if (a.acc) a.acc[i] = tD[cl * DW_PITCH + lane];
        if (a.y) a.y[i] = tY[cl * DW_PITCH + lane];
    }
}

// ---- 3 x 3, pad <= 1: the common case with the per-output work cut down ---------------
// The kernel above spends its time in the vector ALU: coordinate and clamp arithmetic per tap
// and thread, and the four-term formula in fp64 with its products formed per output.  Here
//  * the addressing is prepared once per pixel (one thread each, kept in LDS): the 32-bit byte
//    offsets of the nine taps, with an out-of-range offset for a tap outside the image (the
//    codes are read through a buffer resource, whose out-of-range loads return 0), and the
//    border class (which of the first / last window row and column are cut off: 4 x 4
//    classes; class 0 when the pad mode counts every tap);
//  * Eq.9's constant C = beta_a*alpha_w*Sw + Kv*beta_a*beta_w is prepared once per block for
//    every (class, channel);
//  * a thread forms D and Sa of its 4 pixels x 4 channels from the nine code dwords by two
//    4 x 4 byte transposes (8 byte-permutes each) and byte dot products, and evaluates
//    y = g1*D + c2*Sa + C[class] in fp64 (ReLU, BN, one rounding) with its four channels'
//    factors held in registers; results cross the [channel][pixel] LDS tile;
//  * a block walks several consecutive pixel tiles, so the per-channel set-up is paid once;
//  * the store phase (lanes along pixels, NCHW-contiguous) only copies.
// CHB = channels per block (64, or 32 for layers with at most 32 channels, whose blocks then
// own 128 pixels); offsets are 32-bit: the code tensor must be below 2 GiB.  NT: fp32 outputs
// above 128 MiB are stored with the non-temporal hint, as the matrix-core conv does.
// Dynamic LDS: one tile (CHB x (PXB + 1) dwords) per requested output, y first.
template <int CHB, bool NT>
__global__ __launch_bounds__(256) void k_dwconv3(DwConvArgs a)
{
    constexpr int NCQ = CHB / 4, PXB = 4096 / CHB, PITCH = PXB + 1;
    __shared__ __attribute__((aligned(16))) unsigned po[PXB][12];  // byte offsets of the 9 taps (3 pad words)
    __shared__ int pm[PXB];                                          // border class
    __shared__ __attribute__((aligned(16))) double cst[16][CHB];
    extern __shared__ int dw_tiles[];
    float* tY = (float*)dw_tiles;
    int* tD = dw_tiles + (a.y ? CHB * PITCH : 0);
    const ConvGeom& g = a.g;
    const int tid = threadIdx.x;
    const int64_t ohw = (int64_t)g.OH * g.OW, total = (int64_t)g.Nb * ohw;
    const int cb = (int)blockIdx.y * CHB;
    const EpiArgs& ep = a.ep;
    const bool has_bn = ep.bn_scale != nullptr;
    const double aa = (double)ep.alpha_a.s, ba = (double)ep.beta_a.s;
    // ---- once per block: the class constants and this thread's channel factors ----------
    if (a.y) {
        // (pad <= 1 and an image at least as long as the window: a window is cut at one end of an
        // axis at most, 3 x 3 classes; the others exist only for images shorter than 3)
        const bool tiny = g.H < 3 || g.W < 3;  // only then both ends of an axis can be cut
        const int nax = tiny ? 4 : 3;
        for (int idx = tid; idx < nax * nax * CHB; idx += 256) {
            const int k = idx / CHB, cl = idx - k * CHB;
            const int c = cb + cl < g.C ? cb + cl : g.C - 1;
            const int* wr = (const int*)(a.w + (int64_t)c * a.Kp);
            const int rc = k / nax, cc = k - rc * nax;
            const int cls = rc * 4 + cc;
            unsigned cnt[3] = {0, 0, 0};
            int kv = 0;
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const int kh = t / 3, kw = t % 3;
                const bool out = (kh == 0 && (rc & 1)) || (kh == 2 && (rc & 2)) || (kw == 0 && (cc & 1)) || (kw == 2 && (cc & 2));
                kv += !out;
                cnt[t >> 2] |= (unsigned)!out << (8 * (t & 3));
            }
            int sw = __builtin_amdgcn_sdot4(wr[0], (int)cnt[0], 0, false);
            sw = __builtin_amdgcn_sdot4(wr[1], (int)cnt[1], sw, false);
            sw = __builtin_amdgcn_sdot4(wr[2] & 0xff, (int)cnt[2], sw, false);
            const double aw = pval(ep.alpha_w, c), bw = pval(ep.beta_w, c);
            cst[cls][cl] = ba * aw * (double)sw + (double)kv * ba * bw;
        }
    }
    const int cq = tid % NCQ, pg = tid / NCQ;
    const int c0 = cb + 4 * cq;
    int wq[4][3];
    double g1[4], c2[4], bs[4], bh[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const bool cok = c0 + e < g.C;
        const int c = cok ? c0 + e : g.C - 1;
        const int* wr = (const int*)(a.w + (int64_t)c * a.Kp);
        wq[e][0] = cok ? wr[0] : 0;
        wq[e][1] = cok ? wr[1] : 0;
        wq[e][2] = cok ? (wr[2] & 0xff) : 0;
        g1[e] = c2[e] = bh[e] = 0.0;
        bs[e] = 1.0;
        if (a.y) {
            g1[e] = aa * pval(ep.alpha_w, c);
            c2[e] = aa * pval(ep.beta_w, c);
            bs[e] = has_bn ? (double)ep.bn_scale[c] : 1.0;
            bh[e] = (has_bn && ep.bn_shift) ? (double)ep.bn_shift[c] : 0.0;
        }
    }
    const double relu_floor = __builtin_canonicalize(ep.relu ? 0.0 : -__builtin_inf());
    // A block walks tiles_per_block consecutive pixel tiles of its channel slab, so the
    // preparation above is paid once; two barriers per tile (a thread reaches the first one
    // of the next tile only after its copies of this one).
    for (int tt = 0; tt < a.tiles_per_block; ++tt) {
    const int64_t m0 = ((int64_t)blockIdx.x * a.tiles_per_block + tt) * PXB;
    if (m0 >= total) break;  // block-uniform
    // ---- phase 0: per-pixel preparation, the nine taps of a pixel dealt out over the block's
    // wave groups (so that the work spreads over the CU's four SIMDs) -----------------------
    {
        constexpr int PARTS = 256 / PXB;
        const int px = tid % PXB, part = tid / PXB;
        int64_t m = m0 + px;
        m = m < total ? m : total - 1;  // pixels past the end repeat the last one; never stored
        const int nb = (int)fastdiv((uint32_t)m, g.div_ohw), pix = (int)(m - (int64_t)nb * ohw);
        const int oh = (int)fastdiv((uint32_t)pix, g.div_ow), ow = pix - oh * g.OW;
        const int ih0 = oh * g.stride - g.pad, iw0 = ow * g.stride - g.pad;
        unsigned rowin = 0, colin = 0;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            rowin |= (unsigned)((unsigned)(ih0 + k) < (unsigned)g.H) << k;
            colin |= (unsigned)((unsigned)(iw0 + k) < (unsigned)g.W) << k;
        }
        // a tap outside the image gets an offset past the end of the buffer: the buffer load
        // returns 0 for it (no clamping, no masking of the loaded word)
        const unsigned corner = (unsigned)(((nb * g.H + ih0) * g.W + iw0) * g.Cpad);
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            if (t % PARTS != part) continue;
            const int kh = t / 3, kw = t % 3;
            const bool inb = ((rowin >> kh) & (colin >> kw) & 1u) != 0;
            po[px][t] = inb ? corner + (unsigned)((kh * g.W + kw) * g.Cpad) : 0x80000000u;
        }
        if (part == 0) {
            // pad <= 1: only the first or the last window row / column can be outside
            const unsigned rc = ((rowin & 1u) ^ 1u) | (((rowin >> 2) & 1u) ^ 1u) << 1;
            const unsigned cc = ((colin & 1u) ^ 1u) | (((colin >> 2) & 1u) ^ 1u) << 1;
            pm[px] = (int)(g.code_zero_pad ? 0u : rc * 4u + cc);
        }
    }
    __syncthreads();
    // ---- phase 1: 4 pixels x 4 channels per thread ---------------------------------------
    {
        if (c0 < g.C) {
            // the code tensor as a raw buffer: 32-bit lane offsets on a uniform base, and loads past
            // num_records (the out-of-image taps' offsets, 2^31 + channel) return 0
            const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                (void*)a.a, 0, (int)((int64_t)g.Nb * g.H * g.W * g.Cpad), 0x00020000);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int pl = 4 * pg + q;
                const uint4 o0 = *(const uint4*)&po[pl][0], o1 = *(const uint4*)&po[pl][4], o2 = *(const uint4*)&po[pl][8];
                const unsigned off[9] = {o0.x, o0.y, o0.z, o0.w, o1.x, o1.y, o1.z, o1.w, o2.x};
                int w[9];
#pragma unroll
                for (int t = 0; t < 9; ++t) w[t] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, off[t] + (unsigned)c0, 0, 0);
                // two 4 x 4 byte transposes: out[e] = byte e of (w0, w1, w2, w3)
                int av[2][4];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const unsigned x0 = (unsigned)w[4 * h], x1 = (unsigned)w[4 * h + 1], x2 = (unsigned)w[4 * h + 2],
                                   x3 = (unsigned)w[4 * h + 3];
                    // perm(hi, lo, sel): selector byte values 0-3 pick from lo, 4-7 from hi
                    const unsigned t01l = __builtin_amdgcn_perm(x1, x0, 0x05010400u);  // x0.0 x1.0 x0.1 x1.1
                    const unsigned t01h = __builtin_amdgcn_perm(x1, x0, 0x07030602u);  // x0.2 x1.2 x0.3 x1.3
                    const unsigned t23l = __builtin_amdgcn_perm(x3, x2, 0x05010400u);
                    const unsigned t23h = __builtin_amdgcn_perm(x3, x2, 0x07030602u);
                    av[h][0] = (int)__builtin_amdgcn_perm(t23l, t01l, 0x05040100u);  // x0.0 x1.0 x2.0 x3.0
                    av[h][1] = (int)__builtin_amdgcn_perm(t23l, t01l, 0x07060302u);
                    av[h][2] = (int)__builtin_amdgcn_perm(t23h, t01h, 0x05040100u);
                    av[h][3] = (int)__builtin_amdgcn_perm(t23h, t01h, 0x07060302u);
                }
                const double* crow = &cst[pm[pl]][4 * cq];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int a8 = (int)__builtin_amdgcn_ubfe((unsigned)w[8], 8 * e, 8);  // tap 8 of channel e, low byte
                    int d = __builtin_amdgcn_sdot4(av[0][e], wq[e][0], 0, false);
                    d = __builtin_amdgcn_sdot4(av[1][e], wq[e][1], d, false);
                    d = __builtin_amdgcn_sdot4(a8, wq[e][2], d, false);
                    if (a.acc) tD[(4 * cq + e) * PITCH + pl] = d;
                    if (a.y) {
                        int sa = __builtin_amdgcn_sdot4(av[0][e], 0x01010101, 0, false);
                        sa = __builtin_amdgcn_sdot4(av[1][e], 0x01010101, sa, false);
                        sa = __builtin_amdgcn_sdot4(a8, 0x00000001, sa, false);
                        double y = g1[e] * (double)d + c2[e] * (double)sa + crow[e];
                        y = __builtin_fmax(y, relu_floor);
                        y = bs[e] * y + bh[e];
                        tY[(4 * cq + e) * PITCH + pl] = (float)y;
                    }
                }
            }
        }
    }
    __syncthreads();
    // ---- phase 2: lanes along pixels, channels round-robin over the wave groups; copy only
    const int pl = tid % PXB;
    const int64_t m = m0 + pl;
    if (m < total) {
    const int nb = (int)fastdiv((uint32_t)m, g.div_ohw), pix = (int)(m - (int64_t)nb * ohw);
    constexpr int STEP = 256 / PXB;  // wave groups that share the channels
    const int nch = g.C - cb < CHB ? g.C - cb : CHB;
    const int cl0 = tid / PXB;
    const int64_t i0 = ((int64_t)nb * g.C + cb + cl0) * ohw + pix;
    const int64_t istep = (int64_t)STEP * ohw;
    if (a.y) {
        float* yp = a.y + i0;
        const float* tp = tY + cl0 * PITCH + pl;
#pragma unroll 4
        for (int cl = cl0; cl < nch; cl += STEP) {
            const float v = *tp;
            if (NT)
                __builtin_nontemporal_store(v, yp);
            else
                *yp = v;
            yp += istep;
            tp += STEP * PITCH;
        }
    }
    if (a.acc) {
        int* dp = a.acc + i0;
        const int* tp = tD + cl0 * PITCH + pl;
#pragma unroll 4
        for (int cl = cl0; cl < nch; cl += STEP) {
            *dp = *tp;
            dp += istep;
            tp += STEP * PITCH;
        }
    }
    }  // m < total
    }  // tiles
}

}  // namespace

hipError_t launch_dwconv(const DwConvArgs& a, hipStream_t st)
{
    const int64_t total = (int64_t)a.g.Nb * a.g.OH * a.g.OW;
    if (a.g.KH == 3 && a.g.KW == 3 && a.g.pad <= 1 &&
        (int64_t)a.g.Nb * a.g.H * a.g.W * a.g.Cpad < ((int64_t)1 << 31)) {
        const bool nt = total * a.g.C * 4 > ((int64_t)128 << 20);
        const size_t ntile = (a.y ? 1 : 0) + (a.acc ? 1 : 0);  // LDS tiles
        DwConvArgs b = a;
        // enough blocks for a dozen per CU, each walking up to 16 pixel tiles
        const int chb = a.g.C <= 32 ? 32 : 64;
        const int64_t tiles = (total + 4096 / chb - 1) / (4096 / chb) * ((a.g.C + chb - 1) / chb);
        int64_t tpb = tiles / (256 * 12);
        b.tiles_per_block = (int)(tpb < 1 ? 1 : (tpb > 16 ? 16 : tpb));
        if (a.g.C <= 32) {
            const int64_t nb = ((total + 127) / 128 + b.tiles_per_block - 1) / b.tiles_per_block;
            if (nb <= 0 || nb > 0x7fffffff) return hipErrorInvalidValue;
            const dim3 grid((unsigned)nb, (unsigned)((a.g.C + 31) / 32));
            if (nt)
                hipLaunchKernelGGL((k_dwconv3<32, true>), grid, dim3(256), ntile * 32 * 129 * 4, st, b);
            else
                hipLaunchKernelGGL((k_dwconv3<32, false>), grid, dim3(256), ntile * 32 * 129 * 4, st, b);
        } else {
            const int64_t nb = ((total + 63) / 64 + b.tiles_per_block - 1) / b.tiles_per_block;
            if (nb <= 0 || nb > 0x7fffffff) return hipErrorInvalidValue;
            const dim3 grid((unsigned)nb, (unsigned)((a.g.C + 63) / 64));
            if (nt)
                hipLaunchKernelGGL((k_dwconv3<64, true>), grid, dim3(256), ntile * 64 * 65 * 4, st, b);
            else
                hipLaunchKernelGGL((k_dwconv3<64, false>), grid, dim3(256), ntile * 64 * 65 * 4, st, b);
        }
        return hipGetLastError();
    }
    const int64_t blocks = (total + DW_PX - 1) / DW_PX;
    if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks, (unsigned)(a.g.Cpad / DW_CH));
    if (a.g.KH == 3 && a.g.KW == 3)
        hipLaunchKernelGGL(k_dwconv<3>, grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(k_dwconv<0>, grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace rtn
