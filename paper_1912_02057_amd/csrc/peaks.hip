// Measurement aids (not part of the hot path): the achievable ceilings the roofline
// fractions are quoted against, measured on the machine the benchmark runs on.
//   rtn_peaks_mfma   -- a register-only loop of matrix-core instructions (no memory traffic),
//                       the rate the contraction kernels cannot exceed at the clock the chip
//                       sustains under that load;
//   rtn_peaks_stream -- a plain streaming read, write or copy of a buffer, the HBM rate a
//                       simple kernel reaches.
// Built into its own small library (librtn_peaks.so) that only bench.py loads.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));

// KIND 0: v_mfma_i32_32x32x32_i8, 1: v_mfma_f32_32x32x64_f8f6f4 on FP4 operands.  Four
// independent accumulator tiles per wave, as a 64 x 64 wave tile has.
template <int KIND>
__global__ __launch_bounds__(256) void k_mfma_loop(const v4i* in, float* out, int iters)
{
    const v4i a = in[threadIdx.x], b = in[threadIdx.x + 256];
    float total = 0.f;
    if (KIND == 0) {
        v16i c0 = {}, c1 = {}, c2 = {}, c3 = {};
        for (int i = 0; i < iters; ++i) {
            c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c3, 0, 0, 0);
        }
        for (int r = 0; r < 16; ++r) total += (float)(c0[r] + c1[r] + c2[r] + c3[r]);
    } else {
        const v8i A = {a[0], a[1], a[2], a[3], 0, 0, 0, 0}, B = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
        v16f c0 = {}, c1 = {}, c2 = {}, c3 = {};
        for (int i = 0; i < iters; ++i) {
            c0 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, c0, 4, 4, 0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, c1, 4, 4, 0, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, c2, 4, 4, 0, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, c3, 4, 4, 0, 0, 0, 0);
        }
        for (int r = 0; r < 16; ++r) total += c0[r] + c1[r] + c2[r] + c3[r];
    }
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = total;
}

// KIND 0: copy, 1: read (sum, written only if it hits an impossible value), 2: write
template <int KIND>
__global__ __launch_bounds__(256) void k_stream(f4* dst, const f4* src, size_t n16)
{
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
        if (KIND == 0) dst[i] = src[i];
        if (KIND == 1) acc += src[i];
        if (KIND == 2) dst[i] = f4{1.f, 2.f, 3.f, 4.f};
    }
    if (KIND == 1 && acc[0] + acc[1] + acc[2] + acc[3] == 1.2345e38f) dst[0] = acc;
}

}  // namespace

extern "C" {

// in: 8 KiB of operand bytes (device); out: blocks * 256 floats (device).  Returns the
// number of multiply-accumulates the launch performs, or -1 on a launch error.
double rtn_peaks_mfma(int kind, int blocks, int iters, const void* in, void* out, void* stream)
{
    if (blocks <= 0 || iters <= 0 || !in || !out) return -1.0;
    if (kind == 0)
        hipLaunchKernelGGL(k_mfma_loop<0>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const v4i*)in, (float*)out, iters);
    else if (kind == 1)
        hipLaunchKernelGGL(k_mfma_loop<1>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const v4i*)in, (float*)out, iters);
    else
        return -1.0;
    if (hipGetLastError() != hipSuccess) return -1.0;
    return (double)blocks * 4.0 * iters * 4.0 * 32.0 * 32.0 * (kind == 0 ? 32.0 : 64.0);
}

// dst / src: device buffers of `bytes` bytes (a multiple of 16).  Returns 0, or -1 on error.
int rtn_peaks_stream(int kind, void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src || bytes < 16 || (bytes & 15) || kind < 0 || kind > 2) return -1;
    const size_t n16 = bytes / 16;
    const unsigned grid = 256 * 16;
    if (kind == 0) hipLaunchKernelGGL(k_stream<0>, dim3(grid), dim3(256), 0, (hipStream_t)stream, (f4*)dst, (const f4*)src, n16);
    if (kind == 1) hipLaunchKernelGGL(k_stream<1>, dim3(grid), dim3(256), 0, (hipStream_t)stream, (f4*)dst, (const f4*)src, n16);
    if (kind == 2) hipLaunchKernelGGL(k_stream<2>, dim3(grid), dim3(256), 0, (hipStream_t)stream, (f4*)dst, (const f4*)src, n16);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // extern "C"
