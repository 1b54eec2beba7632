// Device-side arithmetic of the four-term reparameterization (Eq.9 with a
// weight offset), shared by the fused and the stand-alone epilogue kernels.
#pragma once
#include "rtn_kernels.h"

namespace rtn {

__device__ __forceinline__ double pval(const Param& p, int64_t i)
{
    return p.ptr ? (double)p.ptr[i] : (double)p.s;
}

// y = aa*aw*D + aa*bw*Sa + ba*aw*Sw + Kv*ba*bw in fp64, then ReLU, then the BN
// affine, rounded once to fp32.  fp64 keeps the result within one fp32 ulp of
// the exact value even when the four terms cancel.
__device__ __forceinline__ float reparam(double aa, double ba, double aw, double bw, int D, int Sa,
                                         int Sw, int Kv, int relu, bool has_bn, double bs, double bh)
{
    double v = aa * aw * (double)D + aa * bw * (double)Sa + ba * aw * (double)Sw +
               (double)Kv * ba * bw;
    if (relu) v = v < 0.0 ? 0.0 : v;
    if (has_bn) v = bs * v + bh;
    return (float)v;
}

// In-bounds tap range of one output coordinate: taps k in [lo, hi] satisfy
// 0 <= o*stride - pad + k < extent.
__device__ __forceinline__ void tap_range(int o, int stride, int pad, int ksize, int extent, int& lo,
                                          int& hi)
{
    const int i0 = o * stride - pad;
    lo = i0 < 0 ? -i0 : 0;
    hi = extent - 1 - i0;
    hi = hi > ksize - 1 ? ksize - 1 : hi;
}

}  // namespace rtn
