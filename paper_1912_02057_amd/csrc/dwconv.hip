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

}  // namespace

hipError_t launch_dwconv(const DwConvArgs& a, hipStream_t st)
{
    const int64_t total = (int64_t)a.g.Nb * a.g.OH * a.g.OW;
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
