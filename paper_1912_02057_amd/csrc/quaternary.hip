// The paper's comparison system on this hardware: 2-bit quaternary weights and activations
// (values 0..3, Table 1's last column) and their dot product.  Section "How to Compute Dot
// Product between Two Ternary Vectors" computes it bit-serially (AND between each bit of the
// inputs, shifts, four adders, Fig.3(b)); here that pattern runs on the vector ALU over bit
// planes (k_qgemm_popc), and the same integers also come out of the matrix cores, since 0..3
// are exact both as int8 and as FP4 (E2M1: 0x0, 0x2, 0x4, 0x5) -- those two forms reuse the
// ternary GEMM kernel unchanged.
#include "rtn_kernels.h"

namespace rtn {

namespace {

__device__ __forceinline__ int quant4(float v, float t1, float t2, float t3)
{
    return (int)(v > t1) + (int)(v > t2) + (int)(v > t3);  // strict compares, NaN -> 0
}
// E2M1 code point of 0, 1, 2, 3
__device__ __forceinline__ uint32_t nib_q(int q) { return q == 3 ? 5u : (uint32_t)q << 1; }

// rows layout, int8 (FP4 = false) or FP4 nibbles: one wave per row, a step covers 512 elements
// in two coalesced halves (see the ternary FP4 row kernel for the dword assembly).
template <bool FP4>
__global__ __launch_bounds__(256) void k_pack_rows_q4(QPackArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.rows) return;
    const float* xr = a.x + row * a.K;
    uint8_t* cr = (uint8_t*)a.codes + row * (FP4 ? a.Kpad >> 1 : a.Kpad);
    const bool odd = lane & 1;
    for (int64_t k0 = 0; k0 < a.Kpad; k0 += 512) {
        uint32_t h[2];
#pragma unroll
        for (int part = 0; part < 2; ++part) {
            const int64_t k = k0 + 256 * part + 4 * lane;
            int q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) q[e] = k + e < a.K ? quant4(xr[k + e], a.t1, a.t2, a.t3) : 0;
            if (FP4) {
                h[part] = nib_q(q[0]) | (nib_q(q[1]) << 4) | (nib_q(q[2]) << 8) | (nib_q(q[3]) << 12);
            } else if (k < a.Kpad) {
                *(uint32_t*)(cr + k) = (uint32_t)q[0] | ((uint32_t)q[1] << 8) | ((uint32_t)q[2] << 16) | ((uint32_t)q[3] << 24);
            }
        }
        if (FP4) {
            const uint32_t recv = (uint32_t)__shfl_xor((int)(odd ? h[0] : h[1]), 1, 64);
            const uint32_t word = odd ? (recv | (h[1] << 16)) : (h[0] | (recv << 16));
            const int64_t kw = k0 + (odd ? 256 + 4 * (lane - 1) : 4 * lane);
            if (kw < a.Kpad) *(uint32_t*)(cr + (kw >> 1)) = word;
        }
    }
}

// rows layout, bit planes: lane l reads element 64 w + l, so a 64-wide ballot of a bit of q is
// that bit's plane word.  The buffer holds the plane of first (more significant) bits of all
// rows, then the plane of second bits.
__global__ __launch_bounds__(256) void k_pack_rows_qplanes(QPackArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.rows) return;
    const float* xr = a.x + row * a.K;
    const int64_t words = a.Kpad >> 6;
    uint64_t* hrow = (uint64_t*)a.codes + row * words;
    uint64_t* lrow = (uint64_t*)a.codes + a.rows * words + row * words;
    for (int64_t w = 0; w < words; ++w) {
        const int64_t k = w * 64 + lane;
        const int q = k < a.K ? quant4(xr[k], a.t1, a.t2, a.t3) : 0;
        const uint64_t hb = __ballot((q & 2) != 0), lb = __ballot((q & 1) != 0);
        if (lane == 0) {
            hrow[w] = hb;
            lrow[w] = lb;
        }
    }
}

// Bit-serial dot product on the planes: per 64 element pairs a lane spends four ANDs and four
// popcount-accumulates (the four adders of Fig.3(b)); the shifts by the bit weights are applied
// once, to the four sums.  64 x 64 output tile per block, 4 x 4 outputs per thread.
constexpr int PT = 64, KC = 8, LDW = KC + 1;

__global__ __launch_bounds__(256) void k_qgemm_popc(QPopcArgs a)
{
    __shared__ uint64_t sAh[PT * LDW], sAl[PT * LDW], sWh[PT * LDW], sWl[PT * LDW];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int64_t tilesN = (a.N + PT - 1) / PT;
    const int64_t m0 = (blockIdx.x / tilesN) * PT, n0 = (blockIdx.x % tilesN) * PT;
    int c11[4][4], cx[4][4], c00[4][4];  // cx = count(Wh & Al) + count(Wl & Ah): both carry weight 2
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) c11[i][j] = cx[i][j] = c00[i][j] = 0;
    for (int64_t w0 = 0; w0 < a.words; w0 += KC) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int e = tid + 256 * i, row = e / KC, w = e % KC;
            const bool wok = w0 + w < a.words;
            const bool aok = wok && m0 + row < a.M, bok = wok && n0 + row < a.N;
            const int64_t ai = (m0 + row) * a.words + w0 + w, bi = (n0 + row) * a.words + w0 + w;
            sAh[row * LDW + w] = aok ? a.a_hi[ai] : 0;
            sAl[row * LDW + w] = aok ? a.a_lo[ai] : 0;
            sWh[row * LDW + w] = bok ? a.w_hi[bi] : 0;
            sWl[row * LDW + w] = bok ? a.w_lo[bi] : 0;
        }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < KC; ++w) {
            uint64_t ah[4], al[4], wh[4], wl[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ah[i] = sAh[(ty * 4 + i) * LDW + w];
                al[i] = sAl[(ty * 4 + i) * LDW + w];
                wh[i] = sWh[(tx + 16 * i) * LDW + w];
                wl[i] = sWl[(tx + 16 * i) * LDW + w];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    c11[i][j] += __popcll(wh[j] & ah[i]);
                    cx[i][j] += __popcll(wh[j] & al[i]);
                    cx[i][j] += __popcll(wl[j] & ah[i]);
                    c00[i][j] += __popcll(wl[j] & al[i]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + ty * 4 + i;
        if (m >= a.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + tx + 16 * j;
            if (n < a.N) a.acc[m * a.N + n] = (c11[i][j] << 2) + (cx[i][j] << 1) + c00[i][j];
        }
    }
}

}  // namespace

hipError_t launch_pack_rows_q4(const QPackArgs& a, int fmt, hipStream_t st)
{
    const dim3 grid((unsigned)((a.rows + 3) / 4)), block(256);
    if (fmt == 0)
        hipLaunchKernelGGL(k_pack_rows_q4<false>, grid, block, 0, st, a);
    else if (fmt == 2)
        hipLaunchKernelGGL(k_pack_rows_q4<true>, grid, block, 0, st, a);
    else
        hipLaunchKernelGGL(k_pack_rows_qplanes, grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_qgemm_popc(const QPopcArgs& a, hipStream_t st)
{
    const int64_t blocks = ((a.M + PT - 1) / PT) * ((a.N + PT - 1) / PT);
    if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_qgemm_popc, dim3((unsigned)blocks), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace rtn
