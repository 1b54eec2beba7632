// Ternarize + pack kernels (Eq.1 / Eq.3 thresholds, Table 1 encoding) for gfx950.
//
// t = (x > hi) - (x < lo) on the stored fp32 value.  The kernels are pure
// streaming: coalesced fp32 reads, code writes, and the side sum of t per GEMM
// row / per pixel taken with wavefront reductions (64-wide ballots and
// cross-lane adds).  They are HBM-bound: 4 B read per element, 1 B (int8) or
// 0.25 B (two bit planes) written.
#include "rtn_kernels.h"

namespace rtn {

namespace {

__device__ __forceinline__ float thr(const Param& p, int64_t i) { return p.ptr ? p.ptr[i] : p.s; }

__device__ __forceinline__ int tern(float v, float lo, float hi) { return (int)(v > hi) - (int)(v < lo); }

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
// Block = one image n and 64 consecutive pixels; lane <-> pixel, so every load
// (fixed channel, 64 pixels) is a coalesced 256-byte read.  Wave w owns the
// 16-channel groups g = w, w+4, ...; a lane packs its 16 codes of a group into
// one 16-byte store at [n][p][g*16].  Channel sums are combined through LDS.
__global__ __launch_bounds__(256) void k_pack_nchw_i8(PackArgs a)
{
    __shared__ int part[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tiles = (a.HW + 63) >> 6;
    const int64_t n = blockIdx.x / tiles;
    const int64_t p = ((int64_t)blockIdx.x - n * tiles) * 64 + lane;
    const bool pin = p < a.HW;
    const float lo = thr(a.lo, n), hi = thr(a.hi, n);
    const float* xn = a.x + n * a.K * a.HW;
    int8_t* out = (int8_t*)a.codes + (n * a.HW + p) * a.Kpad;
    const int groups = (int)(a.Kpad >> 4);
    int sum = 0;
    for (int g = wave; g < groups; g += 4) {
        uint32_t q[4] = {0, 0, 0, 0};
        float v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t c = (int64_t)g * 16 + j;
            v[j] = (pin && c < a.K) ? xn[c * a.HW + p] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t c = (int64_t)g * 16 + j;
            const int t = (pin && c < a.K) ? tern(v[j], lo, hi) : 0;
            sum += t;
            q[j >> 2] |= (uint32_t)(t & 0xff) << (8 * (j & 3));
        }
        if (pin) *(uint4*)(out + g * 16) = make_uint4(q[0], q[1], q[2], q[3]);
    }
    if (a.sum_t) {
        part[wave][lane] = sum;
        __syncthreads();
        if (wave == 0 && pin)
            a.sum_t[n * a.HW + p] = part[0][lane] + part[1][lane] + part[2][lane] + part[3][lane];
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

hipError_t launch_pack_rows_planes(const PackArgs& a, hipStream_t st)
{
    const dim3 grid((unsigned)((a.rows + 3) / 4)), block(256);
    hipLaunchKernelGGL(k_pack_rows_planes, grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_pack_nchw_i8(const PackArgs& a, hipStream_t st)
{
    const dim3 grid((unsigned)(((a.HW + 63) / 64) * a.N)), block(256);
    hipLaunchKernelGGL(k_pack_nchw_i8, grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_pack_nchw_planes(const PackArgs& a, hipStream_t st)
{
    const dim3 grid((unsigned)(((a.HW + 63) / 64) * a.N)), block(256);
    hipLaunchKernelGGL(k_pack_nchw_planes, grid, block, 0, st, a);
    return hipGetLastError();
}

}  // namespace rtn
