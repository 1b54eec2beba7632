// Ternarize + pack kernels (Eq.1 / Eq.3 thresholds, Table 1 encoding) for gfx950.
//
// t = (x > hi) - (x < lo) on the stored fp32 value.  The kernels are pure
// streaming: coalesced fp32 reads, code writes, and the side sum of t per GEMM
// row / per pixel taken with wavefront reductions (64-wide ballots and
// cross-lane adds).  They are HBM-bound: 4 B read per element, 1 B (int8) or
// 0.25 B (two bit planes) written.
#include <mutex>
#include <type_traits>

#include "rtn_kernels.h"

namespace rtn {

namespace {

__device__ __forceinline__ float thr(const Param& p, int64_t i) { return p.ptr ? p.ptr[i] : p.s; }

__device__ __forceinline__ int tern(float v, float lo, float hi) { return (int)(v > hi) - (int)(v < lo); }

// FP4 (E2M1) code of a ternary value: +1 -> 0x2, -1 -> 0xA, 0 -> 0x0.
__device__ __forceinline__ uint32_t nib(int t) { return (uint32_t)((t & 1) << 1) | (uint32_t)((t >> 28) & 8); }
// Four int8 codes in a dword (bytes 0x00, 0x01, 0xFF) -> their four FP4 nibbles in 16 bits,
// element 0 in the lowest nibble.
__device__ __forceinline__ uint32_t i8x4_to_fp4(uint32_t w)
{
    const uint32_t t = ((w << 1) & 0x02020202u) | ((w >> 4) & 0x08080808u);  // one nibble per byte
    const uint32_t r = (t | (t >> 4)) & 0x00ff00ffu;
    return (r | (r >> 8)) & 0xffffu;
}

__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ---- rows layout, int8 codes -------------------------------------------
// One wavefront per row, four rows per 256-thread block.  Each lane handles 4
// consecutive elements per step (one 16-byte load when VEC4), so a wave reads
// 1 KiB and writes 256 B per step, both fully coalesced.
template <bool VEC4>
__global__ __launch_bounds__(256) void k_pack_rows_i8(PackArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.rows) return;
    const float lo = thr(a.lo, row), hi = thr(a.hi, row);
    const float* xr = a.x + row * a.K;
    int8_t* cr = (int8_t*)a.codes + row * a.Kpad;
    int sum = 0;
    for (int64_t k0 = 0; k0 < a.Kpad; k0 += 256) {
        const int64_t k = k0 + 4 * lane;
        if (k >= a.Kpad) break;
        int t0 = 0, t1 = 0, t2 = 0, t3 = 0;
        if (VEC4) {
            if (k < a.K) {  // K % 4 == 0: the whole quad is in range
                const float4 v = *(const float4*)(xr + k);
                t0 = tern(v.x, lo, hi);
                t1 = tern(v.y, lo, hi);
                t2 = tern(v.z, lo, hi);
                t3 = tern(v.w, lo, hi);
            }
        } else {
            if (k + 0 < a.K) t0 = tern(xr[k + 0], lo, hi);
            if (k + 1 < a.K) t1 = tern(xr[k + 1], lo, hi);
            if (k + 2 < a.K) t2 = tern(xr[k + 2], lo, hi);
            if (k + 3 < a.K) t3 = tern(xr[k + 3], lo, hi);
        }
        sum += t0 + t1 + t2 + t3;
        const uint32_t packed = (uint32_t)(t0 & 0xff) | ((uint32_t)(t1 & 0xff) << 8) |
                                ((uint32_t)(t2 & 0xff) << 16) | ((uint32_t)(t3 & 0xff) << 24);
        *(uint32_t*)(cr + k) = packed;
    }
    if (a.sum_t) {
        sum = wave_sum(sum);
        if (lane == 0) a.sum_t[row] = sum;
    }
}

// ---- rows layout, FP4 codes ------------------------------------------------
// As above with two codes per byte.  A step covers 512 elements: every lane loads
// elements 4l .. 4l+3 of the first and of the second 256 (two fully coalesced 1 KiB
// reads per wave) and packs each quad into 16 bits.  A dword of output is 8 consecutive
// elements, i.e. the quads of lanes 2j and 2j+1: the even lane assembles the dword of
// the first half, the odd lane that of the second half, after one exchange with its
// neighbour, so every lane stores one dword per step.  Kpad % 128 == 0.
template <bool VEC4>
__global__ __launch_bounds__(256) void k_pack_rows_fp4(PackArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.rows) return;
    const float lo = thr(a.lo, row), hi = thr(a.hi, row);
    const float* xr = a.x + row * a.K;
    uint8_t* cr = (uint8_t*)a.codes + row * (a.Kpad >> 1);
    const bool odd = lane & 1;
    int sum = 0;
    for (int64_t k0 = 0; k0 < a.Kpad; k0 += 512) {
        uint32_t h[2];
#pragma unroll
        for (int part = 0; part < 2; ++part) {
            const int64_t k = k0 + 256 * part + 4 * lane;
            int t[4] = {0, 0, 0, 0};
            if (VEC4) {
                if (k < a.K) {  // K % 4 == 0: the whole quad is in range
                    const float4 v = *(const float4*)(xr + k);
                    t[0] = tern(v.x, lo, hi), t[1] = tern(v.y, lo, hi), t[2] = tern(v.z, lo, hi), t[3] = tern(v.w, lo, hi);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (k + e < a.K) t[e] = tern(xr[k + e], lo, hi);
            }
            sum += t[0] + t[1] + t[2] + t[3];
            h[part] = nib(t[0]) | (nib(t[1]) << 4) | (nib(t[2]) << 8) | (nib(t[3]) << 12);
        }
        // even lane: needs the neighbour's first-half quad; odd lane: the neighbour's second-half quad
        const uint32_t recv = (uint32_t)__shfl_xor((int)(odd ? h[0] : h[1]), 1, 64);
        const uint32_t word = odd ? (recv | (h[1] << 16)) : (h[0] | (recv << 16));
        const int64_t kw = k0 + (odd ? 256 + 4 * (lane - 1) : 4 * lane);  // first element of the dword
        if (kw < a.Kpad) *(uint32_t*)(cr + (kw >> 1)) = word;
    }
    if (a.sum_t) {
        sum = wave_sum(sum);
        if (lane == 0) a.sum_t[row] = sum;
    }
}

// ---- rows layout, bit planes --------------------------------------------
// One wavefront per row.  Lane l reads element 64*w + l, so one 64-wide ballot
// of (x > hi) / (x < lo) *is* plane word w; the row sum is popcount(pos) -
// popcount(neg) on the scalar unit.  Four words are produced per step and
// written by lanes 0..3 as one 32-byte store.
__global__ __launch_bounds__(256) void k_pack_rows_planes(PackArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.rows) return;
    const float lo = thr(a.lo, row), hi = thr(a.hi, row);
    const float* xr = a.x + row * a.K;
    const int64_t words = a.Kpad >> 6;
    uint64_t* mrow = (uint64_t*)a.codes + row * words;
    uint64_t* srow = (uint64_t*)a.codes + a.rows * words + row * words;
    int sum = 0;
    for (int64_t w0 = 0; w0 < words; w0 += 4) {
        float v[4];
        bool ok[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t k = (w0 + i) * 64 + lane;
            ok[i] = k < a.K;
            v[i] = ok[i] ? xr[k] : 0.0f;
        }
        uint64_t mword = 0, sword = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint64_t pos = __ballot(ok[i] && v[i] > hi);
            const uint64_t neg = __ballot(ok[i] && v[i] < lo);
            sum += __popcll(pos) - __popcll(neg);
            if (lane == i) {
                mword = pos | neg;
                sword = pos;
            }
        }
        if (lane < 4 && w0 + lane < words) {
            mrow[w0 + lane] = mword;
            srow[w0 + lane] = sword;
        }
    }
    if (a.sum_t && lane == 0) a.sum_t[row] = sum;
}

// ---- NCHW layout, int8 codes, channel-innermost output -------------------
// A block owns 64 consecutive pixels of the flattened (image, pixel) index, so
// its output -- 64 rows of Cpad bytes -- is one contiguous run of the
// [N][H][W][Cpad] tensor, whatever H*W is.  lane <-> pixel: every load (fixed
// channel, 64 pixels) is a coalesced 256-byte read.  Wave w owns the 16-channel
// groups g = w, w+4, ...; a lane packs its 16 codes of a group into 16 bytes
// and parks them in an LDS image of the output run, which the block then
// streams out with consecutive lanes writing consecutive 16-byte chunks (full
// cache lines).  Channel sums are combined through LDS.
template <bool FP4>
__global__ __launch_bounds__(256) void k_pack_nchw_i8(PackArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t tile[];  // [64][Cpad], FP4: [64][Cpad / 2]
    __shared__ int part[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t total = a.N * a.HW;
    const int64_t q0 = (int64_t)blockIdx.x * 64, q = q0 + lane;
    const bool pin = q < total;
    const int64_t n = pin ? q / a.HW : 0;
    const int64_t p = pin ? q - n * a.HW : 0;
    const float lo = thr(a.lo, n), hi = thr(a.hi, n);
    const float* xn = a.x + n * a.K * a.HW + p;
    const int groups = (int)(a.Kpad >> 4);
    const int64_t rowb = FP4 ? a.Kpad >> 1 : a.Kpad;  // bytes of a pixel's code row
    int sum = 0;
    for (int g = wave; g < groups; g += 4) {
        uint32_t w4[4] = {0, 0, 0, 0};
        float v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t c = (int64_t)g * 16 + j;
            v[j] = (pin && c < a.K) ? xn[c * a.HW] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t c = (int64_t)g * 16 + j;
            const int t = (pin && c < a.K) ? tern(v[j], lo, hi) : 0;
            sum += t;
            w4[j >> 2] |= (uint32_t)(t & 0xff) << (8 * (j & 3));
        }
        if (FP4)
            *(uint2*)(tile + (size_t)lane * rowb + g * 8) =
                make_uint2(i8x4_to_fp4(w4[0]) | (i8x4_to_fp4(w4[1]) << 16), i8x4_to_fp4(w4[2]) | (i8x4_to_fp4(w4[3]) << 16));
        else
            *(uint4*)(tile + (size_t)lane * rowb + g * 16) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
    }
    part[wave][lane] = sum;
    __syncthreads();
    if (a.sum_t && wave == 0 && pin) a.sum_t[q] = part[0][lane] + part[1][lane] + part[2][lane] + part[3][lane];
    const int64_t valid = total - q0 < 64 ? total - q0 : 64;
    const int chunks = (int)(valid * (rowb >> 4));
    uint8_t* out = (uint8_t*)a.codes + q0 * rowb;
    for (int e = threadIdx.x; e < chunks; e += 256) *(uint4*)(out + (size_t)e * 16) = *(const uint4*)(tile + (size_t)e * 16);
}

// ---- NCHW layout, int8 codes, 16-byte loads ---------------------------------
// Variant for H*W % 4 == 0 and a 16-byte aligned input.  A block owns
// PB = 4*LPR consecutive pixels; LPR lanes read one channel's run of them with
// one 16-byte load each (lane l: pixels 4q..4q+3, q = l % LPR), and the
// SUBS = 64/LPR lane groups of a wave read channels 16 apart.  Channels go in
// groups of 64*SUBS: wave w, lane group s take channels 16*(w*SUBS+s) .. +15 of
// the group, so a lane ends up with, for each of its 4 pixels, 16 code bytes
// that are contiguous in the channel-innermost output.  They are parked in a
// PB x (64*SUBS)-byte LDS image (always 16 KiB; 16-byte slots XOR-swizzled by
// the pixel quad to spread banks) and streamed out with consecutive lanes
// writing consecutive 16-byte pieces of a pixel's 64*SUBS contiguous bytes.
// LPR = 64 gives the widest pixel runs; the smaller ones trade them for more
// blocks (a tensor with few pixels and many channels) and fewer passes.
// FP4: the same with 8-byte slots (16 channels = 8 bytes), i.e. an 8 KiB LDS image.
template <int LPR, bool FP4>
__global__ __launch_bounds__(256) void k_pack_nchw_i8_v4(PackArgs a)
{
    constexpr int SUBS = 64 / LPR, PB = 4 * LPR, SLOT = FP4 ? 8 : 16, NSLOT = 4 * SUBS, RB = SLOT * NSLOT;
    constexpr int CG = 64 * SUBS;  // channels per group
    __shared__ __attribute__((aligned(16))) uint8_t tile[PB * RB];
    __shared__ int part[4 * SUBS][PB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int quad = lane % LPR, cblk = wave * SUBS + lane / LPR;
    const int64_t total = a.N * a.HW;
    const int64_t q0 = (int64_t)blockIdx.x * PB, q = q0 + 4 * quad;
    const bool pin = q < total;  // total % 4 == 0: all four pixels or none
    const int64_t n = pin ? q / a.HW : 0;
    const int64_t p = pin ? q - n * a.HW : 0;
    const float lo = thr(a.lo, n), hi = thr(a.hi, n);
    const float* xn = a.x + n * a.K * a.HW + p;
    const int ngroup = (int)((a.Kpad + CG - 1) / CG);
    const int64_t valid = total - q0 < PB ? total - q0 : PB;
    const int64_t rowb = FP4 ? a.Kpad >> 1 : a.Kpad;
    uint8_t* out = (uint8_t*)a.codes + q0 * rowb;
    int sum[4] = {0, 0, 0, 0};
    for (int cg = 0; cg < ngroup; ++cg) {
        float4 v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t c = (int64_t)cg * CG + cblk * 16 + j;
            v[j] = (pin && c < a.K) ? *(const float4*)(xn + c * a.HW) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        uint32_t w4[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int k = 0; k < 4; ++k) w4[i][k] = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t c = (int64_t)cg * CG + cblk * 16 + j;
            const bool ok = pin && c < a.K;
            const float e[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = ok ? tern(e[i], lo, hi) : 0;
                sum[i] += t;
                if (FP4)
                    w4[i][j >> 3] |= nib(t) << (4 * (j & 7));
                else
                    w4[i][j >> 2] |= (uint32_t)(t & 0xff) << (8 * (j & 3));
            }
        }
        if (cg > 0) __syncthreads();  // previous group fully streamed out
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint8_t* slot = tile + (4 * quad + i) * RB + (cblk ^ (quad & (NSLOT - 1))) * SLOT;
            if (FP4)
                *(uint2*)slot = make_uint2(w4[i][0], w4[i][1]);
            else
                *(uint4*)slot = make_uint4(w4[i][0], w4[i][1], w4[i][2], w4[i][3]);
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < PB * NSLOT / 256; ++k) {
            const int e = tid + 256 * k, px = e / NSLOT, pp = e % NSLOT;
            const int logical = pp ^ ((px >> 2) & (NSLOT - 1));
            const int64_t cbyte = (int64_t)cg * RB + logical * SLOT;  // the last group may overhang the row
            if (px < valid && cbyte < rowb) {
                if (FP4)
                    *(uint2*)(out + (size_t)px * rowb + cbyte) = *(const uint2*)(tile + e * SLOT);
                else
                    *(uint4*)(out + (size_t)px * rowb + cbyte) = *(const uint4*)(tile + e * SLOT);
            }
        }
    }
    if (a.sum_t) {
#pragma unroll
        for (int i = 0; i < 4; ++i) part[cblk][4 * quad + i] = sum[i];
        __syncthreads();
        if (tid < valid && tid < PB) {
            int s = 0;
#pragma unroll
            for (int b = 0; b < 4 * SUBS; ++b) s += part[b][tid];
            a.sum_t[q0 + tid] = s;
        }
    }
}

// ---- NCHW layout, the common case in straight-line form ------------------------
// The kernel above spends more time in the vector ALU than in memory (bounds
// selects and 64-bit address arithmetic per element).  This one is for tensors
// where none of that is needed: H*W % 4 == 0, C a multiple of the block's channel
// group CG = 64*SUBS, the whole tensor below 4 GiB (a lane's byte offset fits 32
// bits and is added to a wave-uniform base, so a load costs no vector instruction
// besides itself).  Same tiling and LDS image as above.  Per element: two
// compares, two selects and an OR into the code word when the thresholds are
// ordered (ORDERED: scalar thresholds, lo <= hi checked by the entry point, so
// x > hi and x < lo exclude each other), else the subtract form.  The side sum is
// taken from the packed words (SUM).  An FP4 row whose padding exceeds the last
// group (C % 128 == 64) gets its zero half written directly.
template <int LPR, bool FP4, bool SUM, bool ORDERED>
__global__ __launch_bounds__(256) void k_pack_nchw_fast(PackArgs a)
{
    constexpr int SUBS = 64 / LPR, PB = 4 * LPR, SLOT = FP4 ? 8 : 16, NSLOT = 4 * SUBS, RB = SLOT * NSLOT;
    constexpr int CG = 64 * SUBS;
    constexpr int NW = FP4 ? 2 : 4;  // code words per pixel and lane
    __shared__ __attribute__((aligned(16))) uint8_t tile[PB * RB];
    __shared__ int part[SUM ? 4 * SUBS : 1][SUM ? PB : 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int quad = lane % LPR, cblk = wave * SUBS + lane / LPR;
    const int64_t total = a.N * a.HW;
    const int64_t q0 = (int64_t)blockIdx.x * PB;
    int64_t q = q0 + 4 * quad;
    q = q < total ? q : total - 4;  // total % 4 == 0; lanes past the end redo the last quad, never stored
    const int HW = (int)a.HW, K = (int)a.K;
    const int n = (int)(q / HW), p = (int)(q - (int64_t)n * HW);
    const float lo = thr(a.lo, n), hi = thr(a.hi, n);
    const uint32_t off = (uint32_t)((((int64_t)n * K + cblk * 16) * HW + p) * 4);
    const int ngroup = K / CG;
    const int64_t valid = total - q0 < PB ? total - q0 : PB;
    const int rowb = (int)(FP4 ? a.Kpad >> 1 : a.Kpad);
    uint8_t* out = (uint8_t*)a.codes + q0 * rowb;
    int sum[4] = {0, 0, 0, 0}, usum[4] = {0, 0, 0, 0};
    (void)usum;
    for (int cg = 0; cg < ngroup; ++cg) {
        float4 v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float* base = a.x + (int64_t)(cg * CG + j) * HW;  // wave-uniform
            v[j] = *(const float4*)((const char*)base + off);
        }
        uint32_t w[4][NW];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int k = 0; k < NW; ++k) w[i][k] = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float e[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
            const int sh = FP4 ? 4 * (j & 7) : 8 * (j & 3);
            const uint32_t cp = (FP4 ? 0x2u : 0x01u) << sh, cn = (FP4 ? 0xAu : 0xFFu) << sh;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t c;
                if (ORDERED) {
                    c = e[i] > hi ? cp : 0u;
                    c = e[i] < lo ? cn : c;
                } else {
                    // t in {-1, 0, 1}: the int8 code is t's low byte, the FP4 code (t << 1) & 0xA
                    c = ((uint32_t)tern(e[i], lo, hi) << (FP4 ? sh + 1 : sh)) & cn;
                }
                w[i][FP4 ? j >> 3 : j >> 2] |= c;
            }
        }
        if (SUM) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int k = 0; k < NW; ++k) {
                    if (FP4) {
                        sum[i] = __builtin_amdgcn_sdot8((int)w[i][k], 0x11111111, sum[i], false);
                        usum[i] = (int)__builtin_amdgcn_udot8(w[i][k], 0x11111111u, (unsigned)usum[i], false);
                    } else {
                        sum[i] = __builtin_amdgcn_sdot4((int)w[i][k], 0x01010101, sum[i], false);
                    }
                }
        }
        if (cg > 0) __syncthreads();  // previous group fully streamed out
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint8_t* slot = tile + (4 * quad + i) * RB + (cblk ^ (quad & (NSLOT - 1))) * SLOT;
            if (FP4)
                *(uint2*)slot = make_uint2(w[i][0], w[i][1]);
            else
                *(uint4*)slot = make_uint4(w[i][0], w[i][1], w[i][2], w[i][3]);
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < PB * NSLOT / 256; ++k) {
            const int e = tid + 256 * k, px = e / NSLOT, pp = e % NSLOT;
            const int logical = pp ^ ((px >> 2) & (NSLOT - 1));
            const int cbyte = cg * RB + logical * SLOT;
            if (px < valid) {
                if (FP4)
                    *(uint2*)(out + (size_t)px * rowb + cbyte) = *(const uint2*)(tile + e * SLOT);
                else
                    *(uint4*)(out + (size_t)px * rowb + cbyte) = *(const uint4*)(tile + e * SLOT);
            }
        }
    }
    // the zero codes behind the last group (FP4 rows are padded to 128 codes)
    const int donebytes = ngroup * RB, padu = (rowb - donebytes) >> 4;  // 16-byte units per pixel
    for (int e = tid; e < PB * padu; e += 256) {
        const int px = e / padu, u = e - px * padu;
        if (px < valid) *(uint4*)(out + (size_t)px * rowb + donebytes + 16 * u) = make_uint4(0, 0, 0, 0);
    }
    if (SUM) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int t = sum[i];
            if (FP4) {
                // nibbles as integers: +1 is 2 signed and unsigned, -1 is -6 signed and 10 unsigned
                const int neg = (usum[i] - sum[i]) >> 4, pos = (sum[i] + 6 * neg) >> 1;
                t = pos - neg;
            }
            part[cblk][4 * quad + i] = t;
        }
        __syncthreads();
        if (tid < valid && tid < PB) {
            int s = 0;
#pragma unroll
            for (int b = 0; b < 4 * SUBS; ++b) s += part[b][tid];
            a.sum_t[q0 + tid] = s;
        }
    }
}

// ---- NCHW layout, int8 codes, small images whose H*W is not a multiple of 4 ---
// One 1024-thread block per image.  The image's C*H*W floats are one contiguous,
// 16-byte aligned run (C*H*W % 4 == 0), read with 16-byte loads regardless of
// where the channel rows start; element e is channel e / HW, pixel e % HW.  Codes
// are dropped byte by byte into an LDS image [HW][Cpad + 4] (the 4 pad bytes put
// consecutive pixels of a channel on consecutive banks), which is then streamed
// out in 16-byte pieces, every piece adding its 16 codes to its pixel's sum.
template <bool FP4>
__global__ __launch_bounds__(1024) void k_pack_nchw_i8_flat(PackArgs a, FastDiv div_hw)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t img[];  // [HW][Cpad + 4], then int psum[HW]
    const int tid = threadIdx.x;
    const int64_t n = blockIdx.x;
    const int HW = (int)a.HW, K = (int)a.K, Kpad = (int)a.Kpad, pitch = Kpad + 4;
    int* psum = (int*)(img + (size_t)HW * pitch);
    const float lo = thr(a.lo, n), hi = thr(a.hi, n);
    const float* xn = a.x + n * a.K * a.HW;
    for (int p = tid; p < HW; p += 1024) psum[p] = 0;
    // channels K .. Kpad-1 of every pixel are zero codes
    const int padc = Kpad - K;
    for (int e = tid; e < HW * padc; e += 1024) {
        const int p = e / padc;
        img[p * pitch + K + (e - p * padc)] = 0;
    }
    const int nvec = K * HW / 4;
    for (int v0 = tid; v0 < nvec; v0 += 4 * 1024) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int vi = v0 + u * 1024;
            v[u] = vi < nvec ? *(const float4*)(xn + 4 * (int64_t)vi) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int vi = v0 + u * 1024;
            if (vi < nvec) {
                int c = (int)fastdiv((uint32_t)(4 * vi), div_hw), p = 4 * vi - c * HW;
                const float e[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    img[p * pitch + c] = (uint8_t)(tern(e[i], lo, hi) & 0xff);
                    if (++p == HW) {
                        p = 0;
                        ++c;
                    }
                }
            }
        }
    }
    __syncthreads();
    const int np = Kpad / 16;
    const int rowb = FP4 ? Kpad >> 1 : Kpad;
    uint8_t* out = (uint8_t*)a.codes + n * a.HW * rowb;
    for (int e = tid; e < HW * np; e += 1024) {
        const int p = e / np, piece = e - p * np;
        const uint32_t* src = (const uint32_t*)(img + p * pitch + piece * 16);
        const uint4 w = make_uint4(src[0], src[1], src[2], src[3]);
        if (FP4)
            *(uint2*)(out + (size_t)p * rowb + piece * 8) =
                make_uint2(i8x4_to_fp4(w.x) | (i8x4_to_fp4(w.y) << 16), i8x4_to_fp4(w.z) | (i8x4_to_fp4(w.w) << 16));
        else
            *(uint4*)(out + (size_t)p * rowb + piece * 16) = w;
        if (a.sum_t) {
            int s = 0;
            s = __builtin_amdgcn_sdot4((int)w.x, 0x01010101, s, false);
            s = __builtin_amdgcn_sdot4((int)w.y, 0x01010101, s, false);
            s = __builtin_amdgcn_sdot4((int)w.z, 0x01010101, s, false);
            s = __builtin_amdgcn_sdot4((int)w.w, 0x01010101, s, false);
            atomicAdd(&psum[p], s);
        }
    }
    if (a.sum_t) {
        __syncthreads();
        for (int p = tid; p < HW; p += 1024) a.sum_t[n * a.HW + p] = psum[p];
    }
}

// ---- NCHW layout, bit planes ---------------------------------------------
// Same tiling; wave w owns the 64-channel words w, w+4, ...; a lane builds the
// mask and sign words of its pixel bit by bit.
__global__ __launch_bounds__(256) void k_pack_nchw_planes(PackArgs a)
{
    __shared__ int part[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tiles = (a.HW + 63) >> 6;
    const int64_t n = blockIdx.x / tiles;
    const int64_t p = ((int64_t)blockIdx.x - n * tiles) * 64 + lane;
    const bool pin = p < a.HW;
    const float lo = thr(a.lo, n), hi = thr(a.hi, n);
    const float* xn = a.x + n * a.K * a.HW;
    const int64_t words = a.Kpad >> 6;
    const int64_t rows = a.N * a.HW;
    uint64_t* mrow = (uint64_t*)a.codes + (n * a.HW + p) * words;
    uint64_t* srow = (uint64_t*)a.codes + rows * words + (n * a.HW + p) * words;
    int sum = 0;
    for (int64_t w = wave; w < words; w += 4) {
        uint64_t m = 0, s = 0;
        for (int j0 = 0; j0 < 64; j0 += 16) {
            float v[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int64_t c = w * 64 + j0 + j;
                v[j] = (pin && c < a.K) ? xn[c * a.HW + p] : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int64_t c = w * 64 + j0 + j;
                const bool ok = pin && c < a.K;
                const uint64_t pos = ok && v[j] > hi, neg = ok && v[j] < lo;
                m |= (pos | neg) << (j0 + j);
                s |= pos << (j0 + j);
                sum += (int)pos - (int)neg;
            }
        }
        if (pin) {
            mrow[w] = m;
            srow[w] = s;
        }
    }
    if (a.sum_t) {
        part[wave][lane] = sum;
        __syncthreads();
        if (wave == 0 && pin)
            a.sum_t[n * a.HW + p] = part[0][lane] + part[1][lane] + part[2][lane] + part[3][lane];
    }
}

}  // namespace

hipError_t launch_pack_rows_i8(const PackArgs& a, hipStream_t st)
{
    const dim3 grid((unsigned)((a.rows + 3) / 4)), block(256);
    const bool vec4 = (a.K % 4 == 0) && (((uintptr_t)a.x) % 16 == 0);
    if (vec4)
        hipLaunchKernelGGL(k_pack_rows_i8<true>, grid, block, 0, st, a);
    else
        hipLaunchKernelGGL(k_pack_rows_i8<false>, grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_pack_rows_fp4(const PackArgs& a, hipStream_t st)
{
    const dim3 grid((unsigned)((a.rows + 3) / 4)), block(256);
    const bool vec4 = (a.K % 4 == 0) && (((uintptr_t)a.x) % 16 == 0);
    if (vec4)
        hipLaunchKernelGGL(k_pack_rows_fp4<true>, grid, block, 0, st, a);
    else
        hipLaunchKernelGGL(k_pack_rows_fp4<false>, grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_pack_rows_planes(const PackArgs& a, hipStream_t st)
{
    const dim3 grid((unsigned)((a.rows + 3) / 4)), block(256);
    hipLaunchKernelGGL(k_pack_rows_planes, grid, block, 0, st, a);
    return hipGetLastError();
}

template <bool FP4>
hipError_t launch_pack_nchw_codes(const PackArgs& a, hipStream_t st)
{
    const size_t smem = (size_t)64 * (FP4 ? a.Kpad / 2 : a.Kpad);  // LDS image of the block's output run
    if (smem > 128 * 1024) return hipErrorInvalidValue;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void*)k_pack_nchw_i8<FP4>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    if (a.HW % 4 == 0 && ((uintptr_t)a.x) % 16 == 0 && a.K % 64 == 0 && a.N * a.K * a.HW < ((int64_t)1 << 30)) {
        // straight-line kernel; the widest pixel runs that still give every CU several blocks
        const int64_t px = a.N * a.HW;
        const int lpr = (a.K % 256 == 0 && px < 2048 * 256) ? 16 : (a.K % 128 == 0 && px < 4096 * 256) ? 32 : 64;
        const bool ordered = !a.lo.ptr && !a.hi.ptr, sum = a.sum_t != nullptr;
        const dim3 grid((unsigned)((px + 4 * lpr - 1) / (4 * lpr)));
        auto go = [&](auto L, auto S, auto O) {
            hipLaunchKernelGGL((k_pack_nchw_fast<decltype(L)::value, FP4, decltype(S)::value, decltype(O)::value>), grid,
                               dim3(256), 0, st, a);
        };
        auto go2 = [&](auto L) {
            using T = std::true_type;
            using F = std::false_type;
            if (sum)
                ordered ? go(L, T{}, T{}) : go(L, T{}, F{});
            else
                ordered ? go(L, F{}, T{}) : go(L, F{}, F{});
        };
        if (lpr == 16)
            go2(std::integral_constant<int, 16>{});
        else if (lpr == 32)
            go2(std::integral_constant<int, 32>{});
        else
            go2(std::integral_constant<int, 64>{});
        return hipGetLastError();
    }
    if (a.HW % 4 == 0 && ((uintptr_t)a.x) % 16 == 0) {
        // widest pixel runs that still give every CU several blocks and one pass over
        // the channels where the row is long enough
        const int64_t px = a.N * a.HW;
        if (a.Kpad >= 256 && px < 2048 * 256) {
            hipLaunchKernelGGL((k_pack_nchw_i8_v4<16, FP4>), dim3((unsigned)((px + 63) / 64)), dim3(256), 0, st, a);
        } else if (a.Kpad >= 128 && px < 4096 * 256) {
            hipLaunchKernelGGL((k_pack_nchw_i8_v4<32, FP4>), dim3((unsigned)((px + 127) / 128)), dim3(256), 0, st, a);
        } else {
            hipLaunchKernelGGL((k_pack_nchw_i8_v4<64, FP4>), dim3((unsigned)((px + 255) / 256)), dim3(256), 0, st, a);
        }
        return hipGetLastError();
    }
    // small images with H*W % 4 != 0: one block per image over the flat C*H*W run
    const size_t flat_smem = (size_t)a.HW * (a.Kpad + 4) + (size_t)a.HW * 4;
    if ((a.K * a.HW) % 4 == 0 && ((uintptr_t)a.x) % 16 == 0 && flat_smem <= 64 * 1024 && a.HW >= 4 &&
        a.K * a.HW < ((int64_t)1 << 30) && a.N <= 0x7fffffff) {
        hipLaunchKernelGGL(k_pack_nchw_i8_flat<FP4>, dim3((unsigned)a.N), dim3(1024), flat_smem, st, a,
                           make_fastdiv((uint32_t)a.HW));
        return hipGetLastError();
    }
    const dim3 grid((unsigned)((a.N * a.HW + 63) / 64)), block(256);
    hipLaunchKernelGGL(k_pack_nchw_i8<FP4>, grid, block, smem, st, a);
    return hipGetLastError();
}

hipError_t launch_pack_nchw_i8(const PackArgs& a, hipStream_t st) { return launch_pack_nchw_codes<false>(a, st); }
hipError_t launch_pack_nchw_fp4(const PackArgs& a, hipStream_t st) { return launch_pack_nchw_codes<true>(a, st); }

hipError_t launch_pack_nchw_planes(const PackArgs& a, hipStream_t st)
{
    const dim3 grid((unsigned)(((a.HW + 63) / 64) * a.N)), block(256);
    hipLaunchKernelGGL(k_pack_nchw_planes, grid, block, 0, st, a);
    return hipGetLastError();
}

// ---- backward of the reparameterized ternary activation (Eq.6, Eq.7) -----------
// One block: 16384 consecutive elements (64 per thread).  Writes dL/dAbar and the
// block's two partial sums (dgamma, dbeta) in double; a second single-block kernel
// adds the partials in index order, so the result does not depend on scheduling.
namespace {
constexpr int kBwdPerBlock = 16384;

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// NT: the gradient tensor is stored with the non-temporal hint (tensors above 128 MiB, which
// the memory-side cache cannot keep for the next kernel anyway)
template <bool VEC, bool NT = false>
__global__ __launch_bounds__(256) void k_act_backward(ActBwdArgs p)
{
    __shared__ double red[2][4];
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kBwdPerBlock;
    double sg = 0.0, sb = 0.0;
    auto one = [&](float a, float g, float& da) {
        const int t = (int)(a > p.hi) - (int)(a < p.lo);
        sg += (double)t * (double)g;
        sb += (double)g;
        const float prod = __fmul_rn(p.gamma, g);  // one fp32 product, never fused
        da = (a <= 1.0f && a >= -1.0f) ? prod : 0.0f;
    };
    if (VEC) {
#pragma unroll 4
        for (int i = 0; i < kBwdPerBlock / 1024; ++i) {
            const int64_t e = base + (int64_t)(i * 256 + tid) * 4;
            if (e + 4 <= p.n) {
                const float4 a = *(const float4*)(p.a + e), g = *(const float4*)(p.g + e);
                float4 d;
                one(a.x, g.x, d.x), one(a.y, g.y, d.y), one(a.z, g.z, d.z), one(a.w, g.w, d.w);
                if (p.da) {
                    if (NT)
                        __builtin_nontemporal_store(f32x4{d.x, d.y, d.z, d.w}, (f32x4*)(p.da + e));
                    else
                        *(float4*)(p.da + e) = d;
                }
            } else {
                for (int64_t k = e; k < p.n; ++k) {
                    float d;
                    one(p.a[k], p.g[k], d);
                    if (p.da) p.da[k] = d;
                }
            }
        }
    } else {
#pragma unroll 4
        for (int i = 0; i < kBwdPerBlock / 256; ++i) {
            const int64_t e = base + i * 256 + tid;
            if (e < p.n) {
                float d;
                one(p.a[e], p.g[e], d);
                if (p.da) p.da[e] = d;
            }
        }
    }
    sg = wave_sum(sg);
    sb = wave_sum(sb);
    if ((tid & 63) == 0) red[0][tid >> 6] = sg, red[1][tid >> 6] = sb;
    __syncthreads();
    if (tid == 0) {
        p.partials[2 * (int64_t)blockIdx.x] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        p.partials[2 * (int64_t)blockIdx.x + 1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
}

__global__ __launch_bounds__(256) void k_sum_partials(const double* partials, int64_t nblocks, double* out)
{
    __shared__ double red[2][4];
    const int tid = threadIdx.x;
    double sg = 0.0, sb = 0.0;
    for (int64_t b = tid; b < nblocks; b += 256) sg += partials[2 * b], sb += partials[2 * b + 1];
    sg = wave_sum(sg);
    sb = wave_sum(sb);
    if ((tid & 63) == 0) red[0][tid >> 6] = sg, red[1][tid >> 6] = sb;
    __syncthreads();
    if (tid == 0) {
        out[0] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        out[1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
}

// Weight side (Section "Weight Ternarization": Wbar = k_W*W + b_W per filter, W^t = Q(Wbar),
// Wbar^t = alpha*W^t): the rules of Eq.6 / Eq.7 carried through the weight transform by the
// chain rule.  One block per filter; a lane walks the filter with stride 256 (elements, or
// groups of four where the layout allows 16-byte accesses), so a wave reads whole lines.
// The three sums are formed in double, per lane in index order, then over the wave and
// over the four waves in a fixed order: reproducible run to run.
template <bool VEC>
__global__ __launch_bounds__(256) void k_weight_backward(WeightBwdArgs p)
{
    __shared__ double red[3][4];
    const int64_t o = blockIdx.x;
    const float kw = p.kw[o], bw = p.bw[o], al = p.alpha[o];
    const float* w = p.w + o * p.K;
    const float* g = p.g + o * p.K;
    float* dw = p.dw ? p.dw + o * p.K : nullptr;
    double sa = 0.0, sk = 0.0, sb = 0.0;
    auto element = [&](float wv, float gv) -> float {
        const float wbar = __fmaf_rn(kw, wv, bw);
        const int t = (int)(wbar > p.hi) - (int)(wbar < p.lo);
        sa += (double)t * (double)gv;
        const bool inside = wbar <= 1.0f && wbar >= -1.0f;  // NaN is outside
        const float dwbar = inside ? __fmul_rn(al, gv) : 0.0f;
        if (inside) {  // a clipped (or NaN) weight adds nothing, not NaN * 0
            sk += (double)wv * (double)dwbar;
            sb += (double)dwbar;
        }
        return __fmul_rn(kw, dwbar);
    };
    if (VEC) {  // K % 4 == 0 and 16-byte aligned tensors: every filter starts on a 16-byte boundary
        const int64_t k4n = p.K >> 2;
#pragma unroll 2
        for (int64_t k4 = threadIdx.x; k4 < k4n; k4 += 256) {
            const float4 wv = ((const float4*)w)[k4], gv = ((const float4*)g)[k4];
            float4 d;
            d.x = element(wv.x, gv.x);
            d.y = element(wv.y, gv.y);
            d.z = element(wv.z, gv.z);
            d.w = element(wv.w, gv.w);
            if (dw) ((float4*)dw)[k4] = d;
        }
    } else {
        for (int64_t k = threadIdx.x; k < p.K; k += 256) {
            const float d = element(w[k], g[k]);
            if (dw) dw[k] = d;
        }
    }
    sa = wave_sum(sa);
    sk = wave_sum(sk);
    sb = wave_sum(sb);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        red[0][wave] = sa;
        red[1][wave] = sk;
        red[2][wave] = sb;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        const int c = threadIdx.x;
        p.sums[3 * o + c] = (red[c][0] + red[c][1]) + (red[c][2] + red[c][3]);
    }
}
}  // namespace

int64_t act_backward_blocks(int64_t n) { return (n + kBwdPerBlock - 1) / kBwdPerBlock; }

hipError_t launch_act_backward(const ActBwdArgs& p, hipStream_t st)
{
    const int64_t nb = act_backward_blocks(p.n);
    const bool vec = (((uintptr_t)p.a | (uintptr_t)p.g | (uintptr_t)p.da) & 15) == 0;
    if (vec && p.da && p.n * 4 > ((int64_t)128 << 20))
        hipLaunchKernelGGL((k_act_backward<true, true>), dim3((unsigned)nb), dim3(256), 0, st, p);
    else if (vec)
        hipLaunchKernelGGL(k_act_backward<true>, dim3((unsigned)nb), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL(k_act_backward<false>, dim3((unsigned)nb), dim3(256), 0, st, p);
    hipLaunchKernelGGL(k_sum_partials, dim3(1), dim3(256), 0, st, p.partials, nb, p.sums);
    return hipGetLastError();
}

// The form for callers that cannot allocate: the per-block partial sums go to a fixed
// array in device memory instead of a caller workspace.  Every GPU holds its own copy of
// the array at its own address, looked up once per device (the array's name is only a
// host-side handle and is never passed to a kernel).  k_act_backward writes partials
// 0 .. nblocks-1 before k_sum_partials reads exactly those, so what an earlier call left
// in the array is never read and nothing needs clearing.
namespace {
constexpr int64_t kStaticBwdBlocks = 65536;  // 1 MiB of partial sums
__device__ __align__(256) double g_act_bwd_scratch[2 * kStaticBwdBlocks];
constexpr int kMaxDevices = 64;
double* g_act_bwd_scratch_ptr[kMaxDevices] = {};
std::mutex g_act_bwd_scratch_mutex;
}  // namespace

int64_t act_backward_static_max_n() { return kStaticBwdBlocks * kBwdPerBlock; }

hipError_t launch_act_backward_static(ActBwdArgs p, hipStream_t st)
{
    if (act_backward_blocks(p.n) > kStaticBwdBlocks) return hipErrorInvalidValue;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    {
        std::lock_guard<std::mutex> lock(g_act_bwd_scratch_mutex);
        if (!g_act_bwd_scratch_ptr[dev]) {
            double* ptr = nullptr;
            e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(g_act_bwd_scratch));
            if (e != hipSuccess) return e;
            if (!ptr) return hipErrorInvalidSymbol;
            g_act_bwd_scratch_ptr[dev] = ptr;
        }
        p.partials = g_act_bwd_scratch_ptr[dev];
    }
    return launch_act_backward(p, st);
}

hipError_t launch_weight_backward(const WeightBwdArgs& p, hipStream_t st)
{
    const bool vec = (p.K & 3) == 0 && (((uintptr_t)p.w | (uintptr_t)p.g | (uintptr_t)p.dw) & 15) == 0;
    if (vec)
        hipLaunchKernelGGL(k_weight_backward<true>, dim3((unsigned)p.O), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL(k_weight_backward<false>, dim3((unsigned)p.O), dim3(256), 0, st, p);
    return hipGetLastError();
}


}  // namespace rtn
