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
//          input pixel, or 64 zero bytes when the tap falls outside the image.
//
// Tiling (wave64, v_mfma_i32_32x32x32_i8): a 256-thread block owns a BP x BQ
// output tile, its 4 waves a WGP x WGQ grid of (BP/WGP) x (BQ/WGQ) sub-tiles
// made of 32x32 MFMA tiles.  K advances 64 bytes per step (two MFMA k-slices).
//
// Data movement: operand tiles go global -> LDS directly (global_load_lds,
// 16 bytes per lane, no register staging) into NS ring stages, NS steps ahead
// of the MFMAs; completion is tracked by hand with s_waitcnt vmcnt and ONE
// workgroup barrier per K-step placed between the two k-slices, so that the
// fragments of the next slice are always in flight behind 16 MFMAs.  A wave's
// direct load writes 1 KiB of LDS, lane l at +16*l, i.e. 16 rows of 64 bytes;
// which global 16-byte chunk a lane fetches is permuted (XOR swizzle by row) so
// that the 16-byte fragment reads of 16 consecutive rows hit all 64 banks.
//
// Variants of the same kernel (template parameters of k_tmm):
//   HC   conv tiles that keep their run of input pixels in LDS (stride 1, centred window);
//   TERN conv whose epilogue ternarizes its output for the next layer (1), also after
//        the residual add and second ReLU of a block tail (2);
//   DT   1: bf16 operands with fp32 accumulators (v_mfma_f32_32x32x16_bf16) for the
//        weight-only ternary GEMM / conv, whose fp32 activations are split exactly
//        into three bf16 terms laid along K;
//        2: codes stored as FP4 (E2M1) nibbles, two per byte, multiplied by
//        v_mfma_f32_32x32x64_f8f6f4 with fp32 accumulators.  -1, 0, +1 are exact in
//        E2M1 (0xA, 0x0, 0x2), every product is exact and the fp32 sums are integers
//        below 2^24, so D is the same integer the int8 form produces -- at twice the
//        matrix-core rate and half the operand bytes (a 64-byte K-step is 128 codes).
// This header holds the kernel template and its launcher; the instantiations are spread
// over several translation units (tmm_inst_*.hip) so that they compile in parallel.
#pragma once
#include <type_traits>

#include "epilogue_math.h"
#include "rtn_kernels.h"

namespace rtn {

struct TmmParams {
    const int8_t* P;
    const int8_t* Q;
    int RP, RQ;        // valid rows of the P / Q operand
    int64_t ldP, ldQ;  // row pitch in bytes (dense operands)
    int nk;            // number of 64-byte K-steps
    int tilesP;        // number of tiles along P
    int ntiles;        // tilesP * tilesQ
    int band_tiles;    // 8 * tilesQ
    FastDiv div_band;
    int Klogical;      // K of the epilogue's constant term (GEMM)
    int hrows;         // halo variant: input pixels held in LDS (multiple of 16)
    ConvGeom g;        // conv only
    int32_t* acc;
    float* y;
    const double* cst_cls;  // conv: [class][O] constants (see k_conv_class_consts)
    EpiArgs ep;
    // conv, ternarizing epilogue: the output is the next layer's code tensor
    // [pixel][ldc] (int8, channel-innermost) instead of acc / y
    int8_t* codes;
    int ldc;
    Param thr_lo, thr_hi;  // vector: per output channel
    // ... optionally after a residual add (res, fp32 NCHW, nullable) and a second
    // ReLU; the fp32 value that is ternarized is also stored when y is given
    const float* res;
    int relu_out;
    int nt_out;  // conv: store the fp32 / int32 outputs with the non-temporal hint
    // bf16 operands (DT = 1): the weight rows (GEMM: Q, conv: P) are wwrap bytes long and
    // are walked again from the start each time the K offset passes their end; the
    // conv's three activation planes lie qplane bytes apart
    unsigned wwrap;
    int64_t qplane;
};

// Launch of tile configuration `cfg` (the numbering rtn_set_tile_config() documents) of the
// kernel on int8 (DT = 0) or FP4 (DT = 2) codes, GEMM (CONV = false) or conv with the plain
// (TERN = 0), ternarizing (1) or block-tail (2) epilogue.  hipErrorInvalidValue: the
// configuration does not fit this problem.  Defined in tmm_dispatch.inc, instantiated one
// (CONV, TERN, DT) triple per translation unit.
template <bool CONV, int TERN, int DT>
hipError_t tmm_launch_index_raw(int cfg, TmmParams& prm, hipStream_t st);
// The bf16-operand variants of the weight-only path: variant 0 = 64x64, 1 = 128x128,
// 2 = the largest (conv: 128x256, GEMM: 256x256), conv only: 3 = 64x256.
hipError_t tmm_launch_bf16(bool conv, int variant, TmmParams& prm, hipStream_t st);

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// 16 zero bytes every out-of-image tap reads from.
__device__ __attribute__((aligned(16))) int g_zero16[4] = {0, 0, 0, 0};
// Border classes of a conv window and the LDS bytes of the epilogue table of a
// BP-channel tile: rows g1, c2, bn scale, bn shift, then one row per class.
__host__ __device__ inline int conv_classes(int pad)
{
    const int p1 = pad + 1;
    return p1 * p1 * p1 * p1;
}
// The copy of that table a block keeps in LDS holds only the classes that can occur.
// Along one axis a window is cut by tcut taps at the low end and bcut at the high end;
// when the image is at least as long as the window it is never cut at both ends, which
// leaves 2 pad + 1 axis classes (0 = uncut, 1 .. pad = tcut, pad + 1 .. 2 pad = pad + bcut)
// instead of (pad+1)^2 (tcut + (pad+1) bcut, the numbering of the prepared table).
__host__ __device__ inline bool conv_compact(const ConvGeom& g) { return g.H >= g.KH && g.W >= g.KW; }
__host__ __device__ inline int conv_axis_classes(const ConvGeom& g)
{
    return conv_compact(g) ? 2 * g.pad + 1 : (g.pad + 1) * (g.pad + 1);
}
__host__ __device__ inline int conv_lds_classes(const ConvGeom& g)
{
    return conv_axis_classes(g) * conv_axis_classes(g);
}
__host__ __device__ inline int conv_axis_class(bool compact, int pad, int tcut, int bcut)
{
    return compact ? (bcut ? pad + bcut : tcut) : tcut + (pad + 1) * bcut;
}
// axis class of the LDS copy -> axis class of the prepared table
__host__ __device__ inline int conv_axis_global(bool compact, int pad, int a)
{
    return compact ? (a <= pad ? a : (pad + 1) * (a - pad)) : a;
}
__host__ __device__ inline int conv_table_bytes(int bp, const ConvGeom& g) { return (4 + conv_lds_classes(g)) * bp * 8; }

// chunk swizzle of a 64-byte LDS row (depends on row & 15 only)
__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 3) ^ ((row >> 3) & 1); }

// chunk swizzle of a pixel row of the halo image: HC-byte rows, HC/16 chunks
template <int HC>
__device__ __forceinline__ int halo_swz(int row)
{
    return HC == 64 ? swz(row) : ((row >> 1) & 7);
}

// Direct global -> LDS load: every lane fetches 16 bytes at gptr; the wave's
// 1 KiB lands at LDS byte offset lds_off (wave-uniform) + 16 * lane.
// Both statements overwrite M0.  It cannot be named as a clobber (the compiler keeps M0
// reserved and warns that a clobber of it is not honoured); it is safe because on this
// target the compiler itself writes M0 only immediately before an instruction that
// reads it, never across other code, so no value of its own lives in M0 here.
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_off)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_off), "v"(gptr) : "memory");
}

// Same, with the address split into a wave-uniform 64-bit base (SGPR pair) and
// a per-lane unsigned 32-bit byte offset: nothing to add per lane per K-step.
__device__ __forceinline__ void dma16_base(const void* sbase, unsigned voff, unsigned lds_off)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_off), "v"(voff), "s"(sbase)
                 : "memory");
}

// Pin a wave-uniform pointer into scalar registers (the "s" operands above must
// not be handed a vector register pair, which instruction selection may
// otherwise choose for a uniform value).
__device__ __forceinline__ const int8_t* uniform_ptr(const int8_t* p)
{
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const int8_t*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

template <int N>
__device__ __forceinline__ void wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wait_lgkm0() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
// Workgroup barrier that the compiler may not move memory accesses across.
__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Wait until at most `groups` of this wave's K-step load groups (DPS loads
// each) are still in flight.
template <int DPS>
__device__ __forceinline__ void wait_groups(int groups)
{
    if (groups <= 0)
        wait_vm<0>();
    else if (groups == 1)
        wait_vm<DPS>();
    else if (groups == 2)
        wait_vm<2 * DPS>();
    else
        wait_vm<3 * DPS>();
}

// MINW = waves per SIMD the register allocation must leave room for.
//
// HC != 0 selects the halo variant of the conv (stride 1, KH = 2 pad + 1,
// KW = 2 pad + 1, Cpad = HC in {64, 128}).  There output pixel m reads input
// pixel m + (kh - pad) W + (kw - pad) of the same flattened (image, row,
// column) index space, so the BQ output pixels of a tile need the contiguous
// run of BQ + 2 pad (W + 1) input pixels around them.  The block loads that
// run once into LDS and every tap reads its fragments from there: the input
// crosses L2 -> LDS about 1.4 times instead of KH KW times, and only the
// weight tile still streams through the ring.
//
// TERN != 0 selects the conv whose epilogue ternarizes its own output (codes for
// the next layer instead of acc / y); 2 is the block-tail form of it (residual
// add, second ReLU, fp32 copy of the result).  Each is a kernel of its own so
// that its epilogue does not enter the register budget of the others.
//
// DT = 1 multiplies bf16 operands into fp32 accumulators (v_mfma_f32_32x32x16_bf16; a
// lane's 16 operand bytes are 8 bf16 of the same row, so tiles, ring and fragment
// addressing are those of the int8 form): the weight-only ternary GEMM, whose
// activations are fp32 values split into three bf16 terms laid side by side along K.
// DT = 2 multiplies FP4 (E2M1) codes (v_mfma_f32_32x32x64_f8f6f4, both operands FP4,
// no scaling): a lane's 16 operand bytes are 32 codes of one row, everything else is
// byte for byte the int8 form.  Which 32 of a K-step's 128 codes a lane holds, and in
// which nibble order, is the same for both operands, so the sum over k is unaffected.
template <int BP, int BQ, int WGP, int WGQ, int NS, int MINW, bool CONV, int TERN = 0, int HC = 0, int DT = 0>
__global__ __launch_bounds__(256, MINW) void k_tmm(TmmParams prm)
{
    static_assert(DT != 1 || (TERN == 0 && HC == 0), "bf16 operands: plain GEMM and plain conv only");
    static_assert(!TERN || CONV, "the ternarizing epilogue belongs to the conv");
    static_assert(WGP * WGQ == 4, "4 waves per block");
    constexpr bool HALO = HC != 0;
    static_assert(!HALO || (CONV && (HC == 64 || HC == 128)), "halo variant: conv with Cpad 64 or 128");
    constexpr int WP = BP / WGP, WQ = BQ / WGQ, TP = WP / 32, TQ = WQ / 32;
    constexpr int LP = BP / 64, LQ = HALO ? 0 : BQ / 64;  // direct loads per wave per K-step
    constexpr int LQA = LQ ? LQ : 1;                       // array extent
    constexpr int DPS = LP + LQ;
    constexpr int NM = TP * TQ;  // MFMAs per k-slice
    static_assert(TP >= 1 && TQ >= 1 && LP >= 1, "tile too small");
    static_assert(NS >= 2 && (NS - 2) * DPS < 64 && 3 * DPS < 64, "vmcnt range");
    constexpr int STAGE = (BP + (HALO ? 0 : BQ)) * 64;  // bytes; P tile first, then Q tile

    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    const unsigned lds0 = (unsigned)(uintptr_t)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, lives in an SGPR
    const int wp = wave / WGQ, wq = wave % WGQ;
    // Workgroups are dealt to the 8 XCDs round-robin by blockIdx; give each XCD
    // (and so each L2) one contiguous run of tiles, P-tile index fastest, so
    // tiles that share operand rows and conv halo pixels share an L2.
    const int chunk = (int)(gridDim.x >> 3);  // grid is padded to a multiple of 8
    const int bid = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);
    if (bid >= prm.ntiles) return;
    // Within that run, tiles are visited in bands of up to 8 P-tiles, P fastest,
    // so the 32 co-resident tiles of an XCD form an 8 x 4 patch of the output
    // (12 operand row-blocks per K-step instead of 18 for a 16 x 2 strip).
    const int band = (int)fastdiv((uint32_t)bid, prm.div_band);  // band = 8 * tilesQ tiles
    const int inband = bid - band * prm.band_tiles;
    const int bandw = prm.tilesP - band * 8 < 8 ? prm.tilesP - band * 8 : 8;
    const int tileQ = bandw == 8 ? (inband >> 3) : inband / bandw;
    const int tileP = band * 8 + inband - tileQ * bandw;
    const int p0 = tileP * BP, q0 = tileQ * BQ;
    const ConvGeom& g = prm.g;
    // Wave priority falls along a block's life: the waves that still have to get
    // their operand loads into the memory pipeline go first, those in the K loop
    // next, those that only have output left to store last (measured: 2-5 % on the
    // conv layers, because a new block's loads no longer queue behind other blocks'
    // stores as often).
    __builtin_amdgcn_s_setprio(3);
    // LDS: [halo pixels hrows x HC][128 zero bytes][operand ring][conv: epilogue table]
    // [ternarizing conv: BP threshold pairs]; the GEMM builds its small table over the ring
    const int zoff = HALO ? prm.hrows * HC : 0;
    const int roff = HALO ? zoff + 128 : 0;
    const int toff = roff + NS * STAGE;
    const int tab_kib = CONV ? (conv_table_bytes(BP, g) + 1023) >> 10 : 0;
    const bool want_ep = TERN || prm.y != nullptr;

    // ---- loader state ------------------------------------------------------
    // Load j of a wave covers tile rows 16*(wave + 4*j) .. +15; lane l fetches
    // row (l >> 2), logical chunk (l & 3) ^ swz(row) and lands at physical
    // chunk (l & 3) of that row.
    const int lrow = lane >> 2;
    const int lchunk = (lane & 3) ^ swz(lrow);
    // Dense operands: block-uniform base + per-lane offset (at most 256 rows of
    // at most 2^22 bytes).  The conv's Q operand needs a pointer per lane, since
    // an out-of-image tap is redirected to the zero page.
    const int8_t* baseP = prm.P + (int64_t)p0 * prm.ldP;
    const int8_t* baseQ = CONV ? prm.Q : prm.Q + (int64_t)q0 * prm.ldQ;
    unsigned offP[LP];
#pragma unroll
    for (int j = 0; j < LP; ++j) {
        int row = p0 + 16 * (wave + 4 * j) + lrow;
        row = row < prm.RP ? row : prm.RP - 1;  // tail rows: any valid data, never stored
        offP[j] = (unsigned)(row - p0) * (unsigned)prm.ldP + lchunk * 16;
    }
    const int8_t* gQ[LQA];
    unsigned offQ[LQA];
    int vmask[LQA];  // conv: bit kh = row tap valid, bit (8 + kw) = column tap valid
#pragma unroll
    for (int j = 0; j < LQ; ++j) {
        int row = q0 + 16 * (wave + 4 * j) + lrow;
        row = row < prm.RQ ? row : prm.RQ - 1;
        gQ[j] = nullptr;
        offQ[j] = 0;
        vmask[j] = 0;
        if (CONV) {
            const int ohw = g.OH * g.OW;
            const int nb = (int)fastdiv((uint32_t)row, g.div_ohw), pix = row - nb * ohw;
            const int oh = (int)fastdiv((uint32_t)pix, g.div_ow), ow = pix - oh * g.OW;
            const int ih0 = oh * g.stride - g.pad, iw0 = ow * g.stride - g.pad;
            int m = 0;
            for (int k = 0; k < g.KH; ++k) m |= ((unsigned)(ih0 + k) < (unsigned)g.H) << k;
            for (int k = 0; k < g.KW; ++k) m |= ((unsigned)(iw0 + k) < (unsigned)g.W) << (8 + k);
            vmask[j] = m;
            gQ[j] = prm.Q + (((int64_t)nb * g.H + ih0) * g.W + iw0) * g.Cpad + lchunk * 16;
        } else {
            offQ[j] = (unsigned)(row - q0) * (unsigned)prm.ldQ + lchunk * 16;
        }
    }
    // K position of the step being issued: byte offset into a dense row, or for
    // the conv's Q operand the tap (kh, kw) and the offset of its 64 channels.
    int l_kh = 0, l_kw = 0, l_cc = 0;
    int64_t is_koffP = 0, is_koffQ = 0;
    unsigned is_sbase = 0;
    int is_kh = 0, is_kw = 0;
    const int8_t* zero_page = (const int8_t*)g_zero16;

    int64_t l_plane = 0;  // DT = 1 conv: byte offset of the activation plane being walked
    int64_t l_koff = 0;   // conv: running byte offset of the step being issued within the window
    const int64_t l_rowskip = CONV ? (int64_t)(g.W - g.KW) * g.Cpad : 0;
    auto issue_begin = [&](int kt) {
        is_sbase = lds0 + (unsigned)(roff + (kt % NS) * STAGE);
        is_koffP = (int64_t)kt * 64;
        if (CONV && DT == 1) is_koffP = (int64_t)((unsigned)is_koffP % prm.wwrap);
        if (CONV && !HALO) {
            // byte offset of tap (kh, kw), channel chunk cc from a pixel's tap (0, 0):
            // (kh W + kw) Cpad + cc, kept as a running sum (scalar multiplies in this loop cost
            // matrix-core time): + 64 per step, which also carries over from the last chunk of a
            // tap to the next tap of the row, and + (W - KW) Cpad at the end of a window row
            is_kh = l_kh;
            is_kw = l_kw;
            is_koffQ = l_koff + l_plane;
            l_koff += 64;
            l_cc += 64;
            if (l_cc == g.Cpad) {
                l_cc = 0;
                if (++l_kw == g.KW) {
                    l_kw = 0;
                    ++l_kh;
                    l_koff += l_rowskip;
                    if (DT == 1 && l_kh == g.KH) {
                        l_kh = 0;
                        l_koff = 0;
                        l_plane += prm.qplane;
                    }
                }
            }
        } else {
            is_koffQ = is_koffP;
            if (DT == 1) is_koffQ = (int64_t)((unsigned)is_koffP % prm.wwrap);
        }
    };
    // the idx-th of the DPS direct loads of the step set up by issue_begin()
    auto issue_one = [&](int idx) {
        if (idx < LP) {
            dma16_base(uniform_ptr(baseP + is_koffP), offP[idx], is_sbase + (wave + 4 * idx) * 1024);
        } else {
            const int j = idx - LP;
            const unsigned dst = is_sbase + BP * 64 + (wave + 4 * j) * 1024;
            if (CONV) {
                const bool ok = ((vmask[j] >> is_kh) & (vmask[j] >> (8 + is_kw)) & 1) != 0;
                dma16(ok ? gQ[j] + is_koffQ : zero_page, dst);
            } else {
                dma16_base(uniform_ptr(baseQ + is_koffQ), offQ[j], dst);
            }
        }
    };
    auto issue = [&](int kt) {
        issue_begin(kt);
#pragma unroll
        for (int i = 0; i < DPS; ++i) issue_one(i);
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
        for (int ks = 0; ks < 2; ++ks)
            fragQ[t][ks] = BP * 64 + row * 64 + (((ks * 2 + (lane >> 5)) ^ swz(row)) << 4);
    }
    // Halo variant: the Q fragment of tap (kh, kw), channel offset cc is row
    // ml + kh W + kw of the pixel run (ml = the lane's output pixel within the
    // tile), 16 bytes at chunk q = cc/16 + 2 ks + (l >> 5), swizzled by the row
    // (halo_swz) so that 16 consecutive rows hit 16 different 16-byte bank
    // groups; a tap outside the image reads the zero bytes behind the run.
    int mlb[TQ];
    unsigned vmq[TQ];  // bit kh = row tap in the image, bit (8 + kw) = column tap in the image
#pragma unroll
    for (int j = 0; j < TQ; ++j) {
        mlb[j] = wq * WQ + j * 32 + (lane & 31);
        vmq[j] = 0;
        if (HALO) {
            int m = q0 + mlb[j];
            m = m < prm.RQ ? m : prm.RQ - 1;
            const int nb = (int)fastdiv((uint32_t)m, g.div_ohw), pix = m - nb * (g.OH * g.OW);
            const int oh = (int)fastdiv((uint32_t)pix, g.div_ow), ow = pix - oh * g.OW;
            unsigned v = 0;
            for (int k = 0; k < g.KH; ++k) v |= (unsigned)((unsigned)(oh + k - g.pad) < (unsigned)g.H) << k;
            for (int k = 0; k < g.KW; ++k) v |= (unsigned)((unsigned)(ow + k - g.pad) < (unsigned)g.W) << (8 + k);
            vmq[j] = v;
        }
    }
    int f_kh = 0, f_kw = 0, f_cc = 0, f_tapoff = 0;  // K position of the fragments being read
    auto frag_step_advance = [&]() {
        f_cc += 64;
        if (f_cc == HC) {
            f_cc = 0;
            if (++f_kw == g.KW) {
                f_kw = 0;
                ++f_kh;
            }
            f_tapoff = f_kh * g.W + f_kw;
        }
    };
    v4i fa[2][TP], fb[2][TQ];
    constexpr int NF = TP + TQ;  // fragments per k-slice
    // idx-th fragment of slice ks of step kt: P fragments first, then Q
    auto load_frag = [&](int kt, int ks, int idx) {
        const int8_t* st = smem + roff + (kt % NS) * STAGE;
        if (idx < TP) {
            fa[ks][idx] = *(const v4i*)(st + fragP[idx][ks]);
        } else if (!HALO) {
            fb[ks][idx - TP] = *(const v4i*)(st + fragQ[idx - TP][ks]);
        } else {
            const int j = idx - TP;
            const int hr = mlb[j] + f_tapoff;
            const int q = (f_cc >> 4) + ks * 2 + (lane >> 5);
            const bool ok = ((vmq[j] >> f_kh) & (vmq[j] >> (8 + f_kw)) & 1) != 0;
            const int addr = ok ? hr * HC + ((q ^ halo_swz<HC>(hr)) << 4) : zoff + ((lane >> 5) << 4);
            fb[ks][j] = *(const v4i*)(smem + addr);
        }
    };
    auto load_frags = [&](int kt, int ks) {
#pragma unroll
        for (int i = 0; i < NF; ++i) load_frag(kt, ks, i);
    };

    // conv: Sa of an output pixel -- the sum of t_a over its in-bounds taps -- is the
    // sum of all code bytes of its row of the patch matrix (out-of-image taps are zero
    // bytes), i.e. of the Q fragments this lane multiplies anyway: 4 byte-sum dot
    // products per fragment, added up beside the MFMAs.  A lane holds half of a
    // row's bytes (the other k-chunks sit in lane ^ 32); the halves meet in the epilogue.
    // FP4 codes: the row sums come from the matrix cores as well, which have cycles to spare
    // while the vector ALU does not: one 16x16x128 FP4 MFMA per Q fragment with a constant
    // operand of +1 codes.  That instruction reads lane l's 16 bytes as row l & 15, k-block
    // l >> 4, whereas the fragment holds pixel l & 31, k-chunk l >> 5: k-blocks 0 and 2 are
    // the two chunks of pixel l & 15, k-blocks 1 and 3 those of pixel 16 + (l & 15).  With
    // ones in row 0 over k-blocks 0, 2 and in row 1 over k-blocks 1, 3, output row 0 is the
    // sum of pixels 0..15 and row 1 that of pixels 16..31 (registers 0 and 1 of lanes 0..15).
    int sa_part[TQ];
    v4f sa_acc[DT == 2 ? TQ : 1];
#pragma unroll
    for (int j = 0; j < TQ; ++j) sa_part[j] = 0;
#pragma unroll
    for (int j = 0; j < (DT == 2 ? TQ : 1); ++j) sa_acc[j] = v4f{0.f, 0.f, 0.f, 0.f};
    const int sa_ones = ((lane & 15) < 2 && ((lane >> 4) & 1) == (lane & 15)) ? 0x22222222 : 0;
    const v8i SA8 = {sa_ones, sa_ones, sa_ones, sa_ones, 0, 0, 0, 0};
    (void)SA8;
    using AccV = std::conditional_t<DT != 0, v16f, v16i>;
    AccV acc[TP][TQ];
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
        for (int j = 0; j < TQ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    // One k-slice of MFMAs in a fixed issue order: after the n-th MFMA come its
    // share of the next slice's fragment reads (slice fks of step fkt) and, if
    // ISSUE, of the direct loads of step ikt; a scheduling fence after each
    // group keeps the compiler from sinking the reads back to their first use,
    // so LDS and load-issue latency hide behind matrix-core time.
    auto slice = [&](auto with_frags, auto with_issue, int ks, int fkt, int fks, int ikt) {
        constexpr bool FRAGS = decltype(with_frags)::value, ISSUE = decltype(with_issue)::value;
        if (ISSUE) issue_begin(ikt);
        if (HALO && FRAGS && fks == 0) frag_step_advance();
#pragma unroll
        for (int n = 0; n < NM; ++n) {
            if constexpr (DT == 1)
                acc[n / TQ][n % TQ] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(v8bf, fa[ks][n / TQ]), __builtin_bit_cast(v8bf, fb[ks][n % TQ]),
                    acc[n / TQ][n % TQ], 0, 0, 0);
            else if constexpr (DT == 2) {
                // cbsz = blgp = 4: both operands FP4; the upper half of the 8-register operand is unused
                const v4i pa = fa[ks][n / TQ], pb = fb[ks][n % TQ];
                const v8i A8 = {pa[0], pa[1], pa[2], pa[3], 0, 0, 0, 0}, B8 = {pb[0], pb[1], pb[2], pb[3], 0, 0, 0, 0};
                acc[n / TQ][n % TQ] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A8, B8, acc[n / TQ][n % TQ], 4, 4, 0,
                                                                                      0, 0, 0);
                if (CONV && n < TQ)
                    sa_acc[n] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(SA8, B8, sa_acc[n], 4, 4, 0, 0, 0, 0);
            } else
                acc[n / TQ][n % TQ] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ks][n / TQ], fb[ks][n % TQ],
                                                                            acc[n / TQ][n % TQ], 0, 0, 0);
            if (FRAGS) {
                // front-loaded: one read per MFMA when there are enough MFMAs,
                // so the last read is long done at the end of the slice
                constexpr int PER = (NF + NM - 1) / NM;
#pragma unroll
                for (int f = n * PER; f < (n + 1) * PER && f < NF; ++f) load_frag(fkt, fks, f);
            }
            if (ISSUE) {
#pragma unroll
                for (int d = n * DPS / NM; d < (n + 1) * DPS / NM; ++d) issue_one(d);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (CONV && DT == 0) {
#pragma unroll
            for (int j = 0; j < TQ; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) sa_part[j] = __builtin_amdgcn_sdot4(fb[ks][j][e], 0x01010101, sa_part[j], false);
        }
    };
    const std::true_type yes{};
    const std::false_type no{};

    // ---- prologue: start the first NS steps, then per-lane epilogue terms -----
    const int nk = prm.nk;
    const int npro = nk < NS ? nk : NS;
    if (TERN) {
        // thresholds of this tile's channels, (lo, hi) pairs behind the table
        // (visible to every wave after the first barrier of the main loop)
        if (tid < BP) {
            const int o = p0 + tid < prm.RP ? p0 + tid : prm.RP - 1;
            ((float2*)(smem + toff + tab_kib * 1024))[tid] = make_float2((float)pval(prm.thr_lo, o), (float)pval(prm.thr_hi, o));
        }
    }
    if (CONV && want_ep) {
        // epilogue table: rows [g1, c2, bn scale, bn shift, class constants...] of the
        // prepared per-layer table, columns p0 .. p0+BP-1, copied as they are
        // (the class rows that can occur here, see conv_lds_classes)
        const int nrows = 4 + conv_classes(g.pad), opitch = (g.O + 1) & ~1;
        const bool compact = conv_compact(g);
        const int nax = conv_axis_classes(g), lrows = 4 + nax * nax, pp = (g.pad + 1) * (g.pad + 1);
        for (int n = wave; n < tab_kib; n += 4) {
            const int lin = n * 64 + lane;  // 16-byte unit = 2 doubles
            int row = lin / (BP / 2);
            const int u = lin - row * (BP / 2);
            row = row < lrows ? row : lrows - 1;
            if (row >= 4) {
                const int c = row - 4, ra = c / nax, ca = c - ra * nax;
                row = 4 + conv_axis_global(compact, g.pad, ra) * pp + conv_axis_global(compact, g.pad, ca);
            }
            int64_t idx = (int64_t)row * opitch + p0 + 2 * u;
            const int64_t last = (int64_t)nrows * opitch - 2;
            idx = idx < last ? idx : last;  // columns past O are never used
            dma16(prm.cst_cls + idx, lds0 + (unsigned)(toff + n * 1024));
        }
    }
    if (HALO) {
        // the pixel run: 1 KiB per load, lane l lands at 16-byte unit n*64 + l; which chunk
        // of its row a lane fetches is permuted by the row swizzle.  Runs past either
        // end of the tensor re-read the end pixel (only out-of-image taps point there).
        const int total_px = g.Nb * g.H * g.W;
        const int first_px = q0 - g.pad * (g.W + 1);
        const int ninstr = prm.hrows * HC / 1024;
        for (int n = wave; n < ninstr; n += 4) {
            const int lin = n * 64 + lane;
            const int row = lin / (HC / 16), qp = lin % (HC / 16);
            int px = first_px + row;
            px = px < 0 ? 0 : (px < total_px ? px : total_px - 1);
            dma16(prm.Q + (int64_t)px * HC + ((qp ^ halo_swz<HC>(row)) << 4), lds0 + (unsigned)(n * 1024));
        }
        if (tid < 8) *(uint4*)(smem + zoff + tid * 16) = make_uint4(0, 0, 0, 0);
    }
    for (int s = 0; s < npro; ++s) issue(s);

    // Block-tail form: the residual values this lane will add, fetched now so that their
    // HBM latency passes behind the K loop (tiles whose accumulators leave the registers
    // for it; the larger tiles fetch them in the epilogue, 16 at a time).
    constexpr bool RES_EARLY = TERN == 2 && TP * TQ <= 4;
    float rv_all[RES_EARLY ? TQ : 1][RES_EARLY ? TP : 1][16];
    if constexpr (RES_EARLY) {
        const int ohw = g.OH * g.OW;
#pragma unroll
        for (int j = 0; j < TQ; ++j) {
            const int m = q0 + wq * WQ + j * 32 + (lane & 31);
            const bool mok = m < prm.RQ;
            const int mm = mok ? m : 0;
            const int nb = (int)fastdiv((uint32_t)mm, g.div_ohw), pix = mm - nb * ohw;
            const float* rp = prm.res + ((int64_t)nb * g.O * ohw + pix);
#pragma unroll
            for (int i = 0; i < TP; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int o = p0 + wp * WP + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    rv_all[j][i][r] = 0.0f;
                    if (prm.res && mok && o < prm.RP) rv_all[j][i][r] = __builtin_nontemporal_load(rp + (int64_t)o * ohw);
                }
        }
    }

    // conv: the border class of each of this lane's TQ output pixels,
    //   class = rid * (pad+1)^2 + cid,  rid = khl + (pad+1)*(KH-1-khh), cid likewise;
    //   class 0 is the interior (all taps in bounds).
    int pixcls[TQ];
#pragma unroll
    for (int j = 0; j < TQ; ++j) pixcls[j] = 0;
    if (CONV && want_ep && !g.code_zero_pad) {
        const int ohw = g.OH * g.OW;
#pragma unroll
        for (int j = 0; j < TQ; ++j) {
            int m = q0 + wq * WQ + j * 32 + (lane & 31);
            m = m < prm.RQ ? m : prm.RQ - 1;
            const int nb = (int)fastdiv((uint32_t)m, g.div_ohw), pix = m - nb * ohw;
            const int oh = (int)fastdiv((uint32_t)pix, g.div_ow), ow = pix - oh * g.OW;
            int khl, khh, kwl, kwh;
            tap_range(oh, g.stride, g.pad, g.KH, g.H, khl, khh);
            tap_range(ow, g.stride, g.pad, g.KW, g.W, kwl, kwh);
            const bool compact = conv_compact(g);
            pixcls[j] = conv_axis_class(compact, g.pad, khl, g.KH - 1 - khh) * conv_axis_classes(g) +
                        conv_axis_class(compact, g.pad, kwl, g.KW - 1 - kwh);
        }
    }
    __builtin_amdgcn_s_setprio(2);
    // ---- main loop ------------------------------------------------------------
    // Steps kt .. kt+NS-1 are in flight or resident while step kt is multiplied.
    wait_groups<DPS>(npro - 1);
    wait_lgkm0();  // the prologue's plain LDS stores (halo zero bytes, threshold pairs)
    block_barrier();
    load_frags(0, 0);
    int kt = 0;
    // Steady state: between the two k-slices, stage kt is fully in registers
    // (slice-1 fragments waited for), step kt+1 has landed for this wave
    // (all but the NS-2 younger load groups done) and, after the barrier, for
    // every wave; the freed stage is refilled with step kt+NS.
    for (; kt + NS < nk; ++kt) {
        slice(yes, no, 0, kt, 1, 0);
        wait_lgkm0();
        wait_vm<(NS - 2) * DPS>();
        block_barrier();
        slice(yes, yes, 1, kt + 1, 0, kt + NS);
    }
    // Drain: nothing left to issue.
    for (; kt + 1 < nk; ++kt) {
        slice(yes, no, 0, kt, 1, 0);
        wait_lgkm0();
        wait_vm<0>();
        block_barrier();
        slice(yes, no, 1, kt + 1, 0, 0);
    }
    slice(yes, no, 0, kt, 1, 0);
    slice(no, no, 1, 0, 0, 0);

    __builtin_amdgcn_s_setprio(0);
    // ---- epilogue ---------------------------------------------------------------
    // Large conv outputs are written with the non-temporal hint, small ones plainly.  A plain
    // store leaves its dirty lines in the cache hierarchy; when the output is larger than
    // what the memory-side cache holds they are written back while the *next* kernel
    // runs and slow it more than the hint slows this one (205 MB stored, then 205 MB
    // read: 92 us plain, 75 us with the hint).  An output that fits is stored about twice
    // as fast without the hint, and the kernel after it is not slowed (51 MB: 25 us
    // against 39 us for the pair).  The launch code decides (prm.nt_out).
    // The GEMM keeps plain stores: its 256 tiles finish together, and the cache
    // absorbs that burst faster than HBM takes it.
    // (a tag type, not a run-time test at the store: the compiler merges the two arms of such
    // a test into one plain store)
    const bool nt_out = CONV && prm.nt_out;
    auto put = [&](auto nt, auto value, auto* ptr) {
        if constexpr (decltype(nt)::value)
            __builtin_nontemporal_store(value, ptr);
        else
            *ptr = value;
    };
    const EpiArgs& ep = prm.ep;
    const bool has_bn = ep.bn_scale != nullptr;
    // ReLU and BN are applied unconditionally with neutral parameters when off:
    // max(v, -inf) = v and 1*v + 0 = v exactly, so the element code has no selects.
    const double relu_floor = __builtin_canonicalize(ep.relu ? 0.0 : -__builtin_inf());
    double* tab = (double*)(smem + (CONV ? toff : 0));
    const bool full_tile = p0 + BP <= prm.RP && q0 + BQ <= prm.RQ;
    // The element loops exist in 6 straight-line variants (interior / ragged
    // tile) x (acc only / y only / both), picked once per block.
    auto dispatch3 = [&](auto&& run, auto nt) {
        if (full_tile) {
            if (!prm.y)
                run(std::true_type{}, std::true_type{}, std::false_type{}, nt);
            else if (!prm.acc)
                run(std::true_type{}, std::false_type{}, std::true_type{}, nt);
            else
                run(std::true_type{}, std::true_type{}, std::true_type{}, nt);
        } else {
            if (!prm.y)
                run(std::false_type{}, std::true_type{}, std::false_type{}, nt);
            else if (!prm.acc)
                run(std::false_type{}, std::false_type{}, std::true_type{}, nt);
            else
                run(std::false_type{}, std::true_type{}, std::true_type{}, nt);
        }
    };
    auto dispatch = [&](auto&& run) {
        if constexpr (CONV) {
            if (nt_out) {
                dispatch3(run, std::true_type{});
                return;
            }
        }
        dispatch3(run, std::false_type{});
    };
    if (!CONV) {
        __syncthreads();  // all waves are done with the operand stages
        // y = aw*(aa*D + ba*Sw) + bw*r2 with r2 = aa*Sa + K*ba per row m; tab = [3][BP]
        if (prm.y) {
            for (int t = tid; t < BP; t += 256) {
                const int m = p0 + t;
                double aa = 0.0, ba = 0.0, r2 = 0.0;
                if (m < prm.RP) {
                    aa = pval(ep.alpha_a, m);
                    ba = pval(ep.beta_a, m);
                    if (DT != 1) r2 = aa * (double)ep.sum_ta[m] + (double)prm.Klogical * ba;
                }
                tab[t] = aa;
                tab[BP + t] = ba;
                tab[2 * BP + t] = r2;
            }
        }
        __syncthreads();
        const int64_t N = prm.RQ;
        dispatch([&](auto full, auto want_acc, auto want_y, auto nt) {
            constexpr bool FULL = decltype(full)::value, ACC = decltype(want_acc)::value,
                           Y = decltype(want_y)::value;
            // per lane: its TQ output columns, their factors and base pointers.  Set up
            // inside each variant so that a variant holds only what it uses.
            bool nok[TQ];
            double aw[TQ], bw[TQ], bs[TQ], bh[TQ], sw[TQ];
            int32_t* accp[TQ];
            float* yp[TQ];
#pragma unroll
            for (int j = 0; j < TQ; ++j) {
                const int ncol = q0 + wq * WQ + j * 32 + (lane & 31);
                nok[j] = FULL || ncol < prm.RQ;
                aw[j] = bw[j] = bh[j] = sw[j] = 0.0;
                bs[j] = 1.0;
                if (Y && nok[j]) {
                    aw[j] = pval(ep.alpha_w, ncol);
                    bw[j] = pval(ep.beta_w, ncol);
                    if (DT != 1) sw[j] = (double)ep.sum_tw[ncol];
                    if (has_bn) {
                        bs[j] = ep.bn_scale[ncol];
                        bh[j] = ep.bn_shift ? (double)ep.bn_shift[ncol] : 0.0;
                    }
                }
                accp[j] = ACC ? prm.acc + (nok[j] ? ncol : 0) : nullptr;
                yp[j] = Y ? prm.y + (nok[j] ? ncol : 0) : nullptr;
            }
#pragma unroll
            for (int i = 0; i < TP; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int t = wp * WP + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    const int m = p0 + t;
                    const bool mok = FULL || m < prm.RP;
                    double aa = 0.0, ba = 0.0, r2 = 0.0;
                    if (Y) {
                        aa = tab[t];
                        ba = tab[BP + t];
                        r2 = tab[2 * BP + t];
                    }
                    const int64_t rowoff = (int64_t)m * N;
#pragma unroll
                    for (int j = 0; j < TQ; ++j) {
                        if (FULL || (mok && nok[j])) {
                            const auto D = acc[i][j][r];
                            if (ACC) put(nt, (int)D, accp[j] + rowoff);
                            if (Y) {
                                double v = aw[j] * (aa * (double)D + ba * sw[j]) + bw[j] * r2;
                                v = __builtin_fmax(v, relu_floor);
                                put(nt, (float)(bs[j] * v + bh[j]), yp[j] + rowoff);
                            }
                        }
                    }
                    // keep the scheduler from hoisting every later load up here
                    if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                }
        });
    } else {
        // y = g1[o]*D + c2[o]*Sa[m] + Cst[class(m)][o],  g1 = aa*aw, c2 = aa*bw;
        // tab = [4 + ncls][BP]: g1, c2, bn scale, bn shift, then the class constants.
        const int ohw = g.OH * g.OW;
        const int p1 = g.pad + 1;
        (void)p1;
        // (the table was copied into LDS by the prologue's direct loads)
        int sa_full[TQ];
#pragma unroll
        for (int j = 0; j < TQ; ++j) {
            if constexpr (DT == 2) {
                const float s0 = __shfl(sa_acc[j][0], lane & 15, 64), s1 = __shfl(sa_acc[j][1], lane & 15, 64);
                sa_full[j] = (int)((lane & 16) ? s1 : s0);
            } else {
                const int mine = sa_part[j];
                sa_full[j] = mine + __shfl_xor(mine, 32, 64);
            }
        }
        if constexpr (TERN) {
            // Ternarizing epilogue (Eq.1 / Eq.3 applied to the activation of Eq.9): the
            // fp32 value z is formed exactly as below, compared with the channel's
            // thresholds, and only the code leaves the chip.  A lane's accumulator
            // registers 4 r4 .. 4 r4 + 3 are 4 consecutive channels of one pixel: one
            // dword of the channel-innermost code tensor.  Channels O .. ldc-1 get code 0.
            const float2* thr = (const float2*)(smem + toff + tab_kib * 1024);
            // STREAM: the block-tail form -- z + residual (fp32 add, as a separate add
            // kernel would do it), a second ReLU, and the fp32 result stored as well.
            const float relu_out_floor = __builtin_canonicalizef(prm.relu_out ? 0.0f : -__builtin_inff());
            auto run_codes = [&](auto full, auto stream, auto nt) {
                constexpr bool FULL = decltype(full)::value, STREAM = decltype(stream)::value;
#pragma unroll
                for (int j = 0; j < TQ; ++j) {
                    const int m = q0 + wq * WQ + j * 32 + (lane & 31);
                    const bool mok = FULL || m < prm.RQ;
                    int8_t* cp = prm.codes + (int64_t)(mok ? m : 0) * prm.ldc;
                    const double Sa = (double)sa_full[j];
                    const double* ctab = tab + (4 + pixcls[j]) * BP;
                    int64_t obase = 0;
                    if (STREAM) {
                        const int mm = mok ? m : 0;
                        const int nb = (int)fastdiv((uint32_t)mm, g.div_ohw), pix = mm - nb * ohw;
                        obase = (int64_t)nb * g.O * ohw + pix;
                    }
#pragma unroll
                    for (int i = 0; i < TP; ++i) {
                        // residual values of this lane's 16 channels, fetched ahead of their use
                        float rv[16];
                        if constexpr (RES_EARLY) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) rv[r] = rv_all[j][i][r];
                        } else if (STREAM) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int o = p0 + wp * WP + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                                rv[r] = 0.0f;
                                if (prm.res && (FULL || (mok && o < prm.RP)))
                                    rv[r] = __builtin_nontemporal_load(prm.res + obase + (int64_t)o * ohw);
                            }
                        }
                        unsigned half4[4];  // FP4 output: this lane's 4 nibbles of each channel group
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            const int t0 = wp * WP + i * 32 + 8 * r4 + 4 * (lane >> 5);
                            const int o0 = p0 + t0;
                            unsigned word = 0;
#pragma unroll
                            for (int b = 0; b < 4; ++b) {
                                const int t = t0 + b;
                                const bool ook = FULL || o0 + b < prm.RP;
                                const double g1 = tab[t], c2 = tab[BP + t], bs = tab[2 * BP + t], bh = tab[3 * BP + t];
                                const float2 th = thr[t];
                                const int D = acc[i][j][4 * r4 + b];
                                double v = g1 * (double)D + (c2 * Sa + ctab[t]);
                                v = __builtin_fmax(v, relu_floor);
                                float z = (float)(bs * v + bh);
                                if (STREAM) {
                                    z = __builtin_fmaxf(z + rv[4 * r4 + b], relu_out_floor);
                                    if (prm.y && (FULL || (mok && ook))) put(nt, z, prm.y + obase + (int64_t)(o0 + b) * ohw);
                                }
                                if constexpr (DT == 2) {
                                    // E2M1 nibble: +1 -> 0x2, -1 -> 0xA
                                    const bool pos = z > th.y, neg = z < th.x;
                                    unsigned nb4 = ((unsigned)(pos | neg) << 1) | ((unsigned)neg << 3);
                                    if (!FULL && !ook) nb4 = 0;
                                    word |= nb4 << (4 * b);
                                } else {
                                    int code = (int)(z > th.y) - (int)(z < th.x);
                                    if (!FULL && !ook) code = 0;
                                    word |= (unsigned)(code & 0xff) << (8 * b);
                                }
                            }
                            if constexpr (DT == 2) {
                                half4[r4] = word;
                            } else {
                                if (FULL || (mok && o0 < prm.ldc)) *(unsigned*)(cp + o0) = word;
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        if constexpr (DT == 2) {
                            // A dword of the FP4 code tensor is 8 consecutive channels: the 4 of this
                            // lane and the 4 of lane ^ 32 (same pixel).  The lower lane half assembles
                            // channel groups 0 and 2, the upper half groups 1 and 3; each sends the
                            // other the two 16-bit halves it needs in one cross-lane move.
                            const bool upper = (lane >> 5) != 0;
                            const unsigned send = upper ? (half4[0] | (half4[2] << 16)) : (half4[1] | (half4[3] << 16));
                            const unsigned recv = (unsigned)__shfl_xor((int)send, 32, 64);
                            const unsigned wa = upper ? ((recv & 0xffffu) | (half4[1] << 16)) : (half4[0] | (recv << 16));
                            const unsigned wb = upper ? ((recv >> 16) | (half4[3] << 16)) : (half4[2] | (recv & 0xffff0000u));
                            const int c0 = p0 + wp * WP + i * 32 + (upper ? 8 : 0);  // first channel of word wa
                            if (FULL || (mok && (c0 >> 1) < prm.ldc)) *(unsigned*)(cp + (c0 >> 1)) = wa;
                            if (FULL || (mok && ((c0 + 16) >> 1) < prm.ldc)) *(unsigned*)(cp + ((c0 + 16) >> 1)) = wb;
                        }
                    }
                    if constexpr (DT == 2) {
                        // a 64-row tile covers half of a 128-code row: the last tile along the
                        // channels also writes the zero codes of the other half
                        if (BP == 64 && wp == 0 && (p0 + BP) / 2 < prm.ldc && p0 + BP >= prm.RP && mok)
                            *(uint4*)(cp + (p0 + BP) / 2 + 16 * (lane >> 5)) = make_uint4(0, 0, 0, 0);
                    }
                }
            };
            constexpr std::integral_constant<bool, TERN == 2> tail{};
            if (TERN == 2 && nt_out) {
                if (full_tile)
                    run_codes(std::true_type{}, tail, std::true_type{});
                else
                    run_codes(std::false_type{}, tail, std::true_type{});
            } else {
                if (full_tile)
                    run_codes(std::true_type{}, tail, std::false_type{});
                else
                    run_codes(std::false_type{}, tail, std::false_type{});
            }
            return;
        }
        dispatch([&](auto full, auto want_acc, auto want_y, auto nt) {
            constexpr bool FULL = decltype(full)::value, ACC = decltype(want_acc)::value,
                           Y = decltype(want_y)::value;
            // per lane: its TQ output pixels -> Sa, class constants, output base pointers
            bool mok[TQ];
            double Sa[TQ];
            const double* ctab[TQ];
            int32_t* accp[TQ];
            float* yp[TQ];
#pragma unroll
            for (int j = 0; j < TQ; ++j) {
                const int m = q0 + wq * WQ + j * 32 + (lane & 31);
                mok[j] = FULL || m < prm.RQ;
                const int mm = mok[j] ? m : 0;
                const int nb = (int)fastdiv((uint32_t)mm, g.div_ohw), pix = mm - nb * ohw;
                const int64_t obase = (int64_t)nb * g.O * ohw + pix;
                accp[j] = ACC ? prm.acc + obase : nullptr;
                yp[j] = Y ? prm.y + obase : nullptr;
                Sa[j] = (double)sa_full[j];
                ctab[j] = tab + (4 + pixcls[j]) * BP;
            }
#pragma unroll
            for (int i = 0; i < TP; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int t = wp * WP + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    const int o = p0 + t;
                    const bool ook = FULL || o < prm.RP;
                    double g1 = 0.0, c2 = 0.0, bs = 1.0, bh = 0.0, cc[TQ];
                    if (Y) {
                        g1 = tab[t];
                        c2 = tab[BP + t];
                        bs = tab[2 * BP + t];
                        bh = tab[3 * BP + t];
#pragma unroll
                        for (int j = 0; j < TQ; ++j) cc[j] = ctab[j][t];
                    }
                    const int64_t rowoff = (int64_t)o * ohw;
#pragma unroll
                    for (int j = 0; j < TQ; ++j) {
                        if (FULL || (ook && mok[j])) {
                            const auto D = acc[i][j][r];
                            if (ACC) put(nt, (int)D, accp[j] + rowoff);
                            if (Y) {
                                double v = g1 * (double)D + (c2 * Sa[j] + cc[j]);
                                v = __builtin_fmax(v, relu_floor);
                                put(nt, (float)(bs * v + bh), yp[j] + rowoff);
                            }
                        }
                    }
                    if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                }
        });
    }
}

// LDS bytes of the epilogue tables of a BP-row tile.
inline int64_t table_bytes(int bp, bool conv, const ConvGeom& g)
{
    return conv ? (int64_t)conv_table_bytes(bp, g) : (int64_t)3 * bp * 8;
}
constexpr int64_t kMaxLds = 160 * 1024;

// Halo variant: stride 1, window centred on the output pixel, HC-byte pixel rows.
inline bool halo_eligible(const TmmParams& prm, int hc)
{
    const ConvGeom& g = prm.g;
    return g.stride == 1 && g.KH == 2 * g.pad + 1 && g.KW == 2 * g.pad + 1 && g.Cpad == hc && g.OH == g.H &&
           g.OW == g.W;
}

template <int BP, int BQ, int WGP, int WGQ, int NS, int MINW, bool CONV, int TERN = 0, int HC = 0, int DT = 0>
hipError_t launch_cfg(TmmParams& prm, hipStream_t st)
{
    constexpr int ring_bytes = NS * (BP + (HC ? 0 : BQ)) * 64;
    int64_t stage_bytes = ring_bytes;
    if (HC) {
        if (!halo_eligible(prm, HC)) return hipErrorInvalidValue;
        prm.hrows = (BQ + 2 * prm.g.pad * (prm.g.W + 1) + 15) & ~15;
        stage_bytes += (int64_t)prm.hrows * HC + 128;
    }
    int64_t smem;
    if (CONV) {
        // ring (+ halo), then the epilogue table in whole KiB
        smem = stage_bytes + ((table_bytes(BP, true, prm.g) + 1023) & ~(int64_t)1023);
        if (TERN) smem += BP * 8;  // threshold pairs of the ternarizing epilogue
    } else {
        const int64_t tb = table_bytes(BP, false, prm.g);
        smem = stage_bytes > tb ? stage_bytes : tb;
    }
    if (smem > kMaxLds) return hipErrorInvalidValue;
    static bool attr_done = false;
    auto kern = k_tmm<BP, BQ, WGP, WGQ, NS, MINW, CONV, TERN, HC, DT>;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)kMaxLds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    prm.tilesP = (prm.RP + BP - 1) / BP;
    const int64_t tilesQ = ((int64_t)prm.RQ + BQ - 1) / BQ;
    const int64_t blocks = (int64_t)prm.tilesP * tilesQ;
    if (blocks <= 0 || blocks > 0x7fffff00) return hipErrorInvalidValue;
    prm.ntiles = (int)blocks;
    if (tilesQ * 8 > 0x7fffffff) return hipErrorInvalidValue;
    prm.band_tiles = (int)(8 * tilesQ);
    prm.div_band = make_fastdiv((uint32_t)prm.band_tiles);
    const unsigned grid = (unsigned)((blocks + 7) / 8 * 8);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), (size_t)smem, st, prm);
    return hipGetLastError();
}

// Tile configurations, indexed as rtn_set_tile_config() documents: BP of each.
constexpr int kNumTileConfigs = 20;
constexpr int kTileBP[kNumTileConfigs] = {64, 128, 256, 64,  128, 256, 64, 64, 128, 64,
                                           64, 64,  128, 128, 64,  64,  64, 64, 128, 128};

}  // namespace

}  // namespace rtn
