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
// A block owns 64 consecutive pixels of the flattened (image, pixel) index, so
// its output -- 64 rows of Cpad bytes -- is one contiguous run of the
// [N][H][W][Cpad] tensor, whatever H*W is.  lane <-> pixel: every load (fixed
// channel, 64 pixels) is a coalesced 256-byte read.  Wave w owns the 16-channel
// groups g = w, w+4, ...; a lane packs its 16 codes of a group into 16 bytes
// and parks them in an LDS image of the output run, which the block then
// streams out with consecutive lanes writing consecutive 16-byte chunks (full
// cache lines).  Channel sums are combined through LDS.
__global__ __launch_bounds__(256) void k_pack_nchw_i8(PackArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t tile[];  // [64][Cpad]
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
        *(uint4*)(tile + (size_t)lane * a.Kpad + g * 16) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
    }
    part[wave][lane] = sum;
    __syncthreads();
    if (a.sum_t && wave == 0 && pin) a.sum_t[q] = part[0][lane] + part[1][lane] + part[2][lane] + part[3][lane];
    const int64_t valid = total - q0 < 64 ? total - q0 : 64;
    const int chunks = (int)(valid * groups);
    uint8_t* out = (uint8_t*)a.codes + q0 * a.Kpad;
    for (int e = threadIdx.x; e < chunks; e += 256) *(uint4*)(out + (size_t)e * 16) = *(const uint4*)(tile + (size_t)e * 16);
}

// ---- NCHW layout, int8 codes, 16-byte loads ---------------------------------
// Variant for H*W % 4 == 0 and a 16-byte aligned input: a block owns 256
// consecutive pixels; lane l holds pixels 4l..4l+3 and reads them with one
// 16-byte load per channel (a wave reads 1 KiB per channel).  Channels go in
// chunks of 64: wave w takes channels 16w..16w+15 of the chunk, so a lane ends
// up with, for each of its 4 pixels, the 16 code bytes that are contiguous in
// the channel-innermost output.  They are parked in a 256 x 64-byte LDS image
// (16-byte slots XOR-swizzled by lane to spread banks) and streamed out with
// 4 consecutive lanes writing the 64 contiguous bytes of a pixel.
__global__ __launch_bounds__(256) void k_pack_nchw_i8_v4(PackArgs a)
{
    __shared__ __attribute__((aligned(16))) uint8_t tile[256 * 64];
    __shared__ int part[4][256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t total = a.N * a.HW;
    const int64_t q0 = (int64_t)blockIdx.x * 256, q = q0 + 4 * lane;
    const bool pin = q < total;  // total % 4 == 0: all four pixels or none
    const int64_t n = pin ? q / a.HW : 0;
    const int64_t p = pin ? q - n * a.HW : 0;
    const float lo = thr(a.lo, n), hi = thr(a.hi, n);
    const float* xn = a.x + n * a.K * a.HW + p;
    const int nchunk = (int)(a.Kpad >> 6);
    const int64_t valid = total - q0 < 256 ? total - q0 : 256;
    uint8_t* out = (uint8_t*)a.codes + q0 * a.Kpad;
    int sum[4] = {0, 0, 0, 0};
    for (int cb = 0; cb < nchunk; ++cb) {
        float4 v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t c = (int64_t)cb * 64 + wave * 16 + j;
            v[j] = (pin && c < a.K) ? *(const float4*)(xn + c * a.HW) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        uint32_t w4[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int k = 0; k < 4; ++k) w4[i][k] = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t c = (int64_t)cb * 64 + wave * 16 + j;
            const bool ok = pin && c < a.K;
            const float e[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = ok ? tern(e[i], lo, hi) : 0;
                sum[i] += t;
                w4[i][j >> 2] |= (uint32_t)(t & 0xff) << (8 * (j & 3));
            }
        }
        if (cb > 0) __syncthreads();  // previous chunk fully streamed out
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *(uint4*)(tile + (4 * lane + i) * 64 + ((wave ^ (lane & 3)) << 4)) =
                make_uint4(w4[i][0], w4[i][1], w4[i][2], w4[i][3]);
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int e = tid + 256 * k, px = e >> 2, pp = e & 3;
            const int logical = pp ^ ((px >> 2) & 3);
            if (px < valid)
                *(uint4*)(out + (size_t)px * a.Kpad + cb * 64 + logical * 16) = *(const uint4*)(tile + e * 16);
        }
    }
    if (a.sum_t) {
#pragma unroll
        for (int i = 0; i < 4; ++i) part[wave][4 * lane + i] = sum[i];
        __syncthreads();
        if (tid < valid) a.sum_t[q0 + tid] = part[0][tid] + part[1][tid] + part[2][tid] + part[3][tid];
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
    const size_t smem = (size_t)64 * a.Kpad;  // LDS image of the block's output run
    if (smem > 128 * 1024) return hipErrorInvalidValue;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void*)k_pack_nchw_i8,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    if (a.HW % 4 == 0 && ((uintptr_t)a.x) % 16 == 0) {
        const dim3 grid4((unsigned)((a.N * a.HW + 255) / 256));
        hipLaunchKernelGGL(k_pack_nchw_i8_v4, grid4, dim3(256), 0, st, a);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)((a.N * a.HW + 63) / 64)), block(256);
    hipLaunchKernelGGL(k_pack_nchw_i8, grid, block, smem, st, a);
    return hipGetLastError();
}

hipError_t launch_pack_nchw_planes(const PackArgs& a, hipStream_t st)
{
    const dim3 grid((unsigned)(((a.HW + 63) / 64) * a.N)), block(256);
    hipLaunchKernelGGL(k_pack_nchw_planes, grid, block, 0, st, a);
    return hipGetLastError();
}

}  // namespace rtn
