// Internal launch interface between the C-ABI layer (rtn_api.hip) and the
// gfx950 kernels.  Everything here takes validated arguments.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rtn {

// A scalar-or-vector fp32 parameter: ptr != nullptr -> device vector, else `s`.
struct Param {
    const float* ptr;
    float s;
};

struct PackArgs {
    const float* x;
    int64_t rows;     // ROWS: d0.  NCHW: unused
    int64_t K, Kpad;  // ROWS: row length.  NCHW: C, Cpad
    int64_t N, HW;    // NCHW only
    Param lo, hi;     // vector: per row (ROWS) / per d0 (NCHW)
    void* codes;
    int32_t* sum_t;   // nullable
};

hipError_t launch_pack_rows_i8(const PackArgs& a, hipStream_t st);
// FP4 (E2M1) codes, two per byte (element 2j in the low nibble of byte j); Kpad % 128 == 0
hipError_t launch_pack_rows_fp4(const PackArgs& a, hipStream_t st);
hipError_t launch_pack_nchw_fp4(const PackArgs& a, hipStream_t st);
hipError_t launch_pack_rows_planes(const PackArgs& a, hipStream_t st);
hipError_t launch_pack_nchw_i8(const PackArgs& a, hipStream_t st);
hipError_t launch_pack_nchw_planes(const PackArgs& a, hipStream_t st);

// Backward of the reparameterized ternary activation.
struct ActBwdArgs {
    const float* a;    // pre-ternarization activation
    const float* g;    // dL/d(gamma*t + beta)
    int64_t n;
    float lo, hi, gamma;
    float* da;         // nullable
    double* partials;  // workspace: 2 doubles per block
    double* sums;      // out: {dgamma, dbeta}
};
int64_t act_backward_blocks(int64_t n);
hipError_t launch_act_backward(const ActBwdArgs& p, hipStream_t st);
// the same with the partial sums in a fixed device array of the library (p.partials ignored);
// n is limited to act_backward_static_max_n()
int64_t act_backward_static_max_n();
hipError_t launch_act_backward_static(ActBwdArgs p, hipStream_t st);

// Backward of the reparameterized ternary weights, one filter per row.
struct WeightBwdArgs {
    const float* w;      // [O][K] latent weights
    const float* g;      // [O][K] dL/d(alpha * t_w)
    int64_t O, K;
    float lo, hi;        // thresholds on k_W * w + b_W
    const float* kw;     // [O]
    const float* bw;     // [O]
    const float* alpha;  // [O]
    float* dw;           // nullable [O][K]
    double* sums;        // out [O][3]: dalpha, dk_W, db_W
};
hipError_t launch_weight_backward(const WeightBwdArgs& p, hipStream_t st);

// Epilogue parameters as the kernels see them.
struct EpiArgs {
    Param alpha_a, beta_a;  // vector: per GEMM row m (GEMM only)
    Param alpha_w, beta_w;  // vector: per output column / channel
    const int32_t* sum_ta;  // GEMM: [M]; conv: [Nb][H][W] pixel sums
    const int32_t* sum_tw;  // GEMM: [N]; conv: [O][KH][KW] tap sums
    int relu;
    const float* bn_scale;  // nullable, per output column / channel
    const float* bn_shift;
};

// Division of a 31-bit dividend by a fixed divisor as multiply-high + shift
// (round-up magic number, exact for 0 <= n < 2^31); m == 0 encodes divisor 1.
struct FastDiv {
    uint32_t m, sh;
};
inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f = {0, 0};
    if (d <= 1) return f;
    uint32_t L = 0;
    while ((1ull << L) < d) ++L;
    f.m = (uint32_t)(((1ull << (31 + L)) + d - 1) / d);
    f.sh = L - 1;
    return f;
}
__host__ __device__ inline uint32_t fastdiv(uint32_t n, FastDiv f)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return f.m ? (__umulhi(n, f.m) >> f.sh) : n;
#else
    return f.m ? (uint32_t)(((uint64_t)n * f.m) >> 32) >> f.sh : n;
#endif
}

struct ConvGeom {
    int Nb, C, Cpad, H, W, O, KH, KW, stride, pad, OH, OW;
    int code_zero_pad;  // 1: RTN_PAD_CODE_ZERO
    FastDiv div_ohw, div_ow;  // by OH*OW and by OW
};

struct GemmArgs {
    const int8_t* a;  // [M][Kpad] int8, or [M][Kpad / 2] bytes of FP4 nibbles
    const int8_t* w;  // [N][Kpad]
    int64_t M, N, K, Kpad;
    int fp4;          // 1: FP4 codes (Kpad % 128 == 0)
    int32_t* acc;  // nullable
    float* y;      // nullable (then `ep` unused)
    EpiArgs ep;
};

struct ConvArgs {
    const int8_t* a;  // [Nb][H][W][Cpad]
    const int8_t* w;  // [O][KH][KW][Cpad]
    ConvGeom g;       // g.Cpad in codes
    int fp4;          // 1: both code tensors hold FP4 nibbles, Cpad / 2 bytes per pixel (Cpad % 128 == 0)
    int32_t* acc;          // nullable, [Nb][O][OH][OW]
    float* y;              // nullable
    const double* cst_cls; // workspace: the prepared per-layer epilogue table (when y or codes)
    EpiArgs ep;
    // ternarizing epilogue (acc and y NULL): codes [Nb*OH*OW][ldc] int8, thresholds
    // scalar or per output channel
    int8_t* codes;
    int ldc;
    Param thr_lo, thr_hi;
    const float* res;  // nullable: fp32 NCHW added to the activation before it is ternarized
    int relu_out;      // ReLU after that add; with codes, `y` (nullable) receives the ternarized fp32 value
};

hipError_t launch_gemm_mfma(const GemmArgs& a, hipStream_t st);

// Weight-only ternary GEMM: y[m][n] = alpha_w[n] * sum_k x[m][k] * t_w[n][k] (+ tail of ep).
struct WGemmArgs {
    const float* x;    // [M][K] fp32
    const int8_t* w;   // [N][Kpad] int8 codes
    int64_t M, N, K, Kpad;
    float* y;          // [M][N]
    void* workspace;   // (3 M + N) * Kpad bf16
    EpiArgs ep;        // alpha_a = 1, beta_a = 0, beta_w = 0; alpha_w, relu, bn as given
    const void* prepared;  // nullable: the weights as bf16, written by launch_wgemm_prepare (then w is unused)
};
hipError_t launch_wgemm(const WGemmArgs& a, hipStream_t st);
// weight side of the above, once per layer: int8 codes [N][Kpad] -> bf16 [N][Kpad]
hipError_t launch_wgemm_prepare(const int8_t* w, int64_t N, int64_t Kpad, void* prepared, hipStream_t st);

// conv form: x fp32 NCHW, w int8 [O][KH][KW][Cpad] (g.Cpad in elements), y fp32 NCHW;
// workspace: 3 activation planes + weights as bf16, then the epilogue table
struct WConvArgs {
    const float* x;
    const int8_t* w;
    ConvGeom g;
    float* y;
    void* workspace;
    EpiArgs ep;
    const void* prepared;  // nullable: bf16 weights + epilogue table, written by launch_wconv_prepare
};
hipError_t launch_wconv(const WConvArgs& a, hipStream_t st);
// weight side of the above, once per layer (g: C, Cpad, O, KH, KW, pad are read): bf16
// weights [O][KH][KW][Cpad], then (16-byte aligned) the epilogue table
hipError_t launch_wconv_prepare(const int8_t* w, const ConvGeom& g, const EpiArgs& ep, void* prepared, hipStream_t st);
hipError_t launch_conv_mfma(const ConvArgs& a, hipStream_t st);
// Tile configuration override for tuning and tests (-1 = heuristic).
int tile_config_count();
void force_tile_config(int index);

hipError_t launch_conv_class_consts(const ConvArgs& a, double* cst, hipStream_t st);

struct PopcArgs {
    const uint64_t *a_mask, *a_sign;  // [M][words]
    const uint64_t *w_mask, *w_sign;  // [N][words]
    int64_t M, N, K, words;
    int32_t* acc;
    float* y;
    EpiArgs ep;
};
hipError_t launch_gemm_popc(const PopcArgs& a, hipStream_t st);

// The quaternary comparison system (values 0..3): quantize + pack of rows, and the bit-serial
// dot product on bit planes.  The matrix-core forms go through launch_gemm_mfma.
struct QPackArgs {
    const float* x;   // [rows][K]
    int64_t rows, K, Kpad;
    float t1, t2, t3;  // q = (x > t1) + (x > t2) + (x > t3)
    void* codes;
};
hipError_t launch_pack_rows_q4(const QPackArgs& a, int fmt, hipStream_t st);  // fmt as rtn_code_format
struct QPopcArgs {
    const uint64_t *a_hi, *a_lo;  // [M][words]: planes of the first / second bits
    const uint64_t *w_hi, *w_lo;  // [N][words]
    int64_t M, N, words;
    int32_t* acc;
};
hipError_t launch_qgemm_popc(const QPopcArgs& a, hipStream_t st);

// Depthwise ternary conv: a int8 [Nb][H][W][Cpad], w int8 [C][Kp] (one row of KH*KW tap codes per
// channel), outputs [Nb][C][OH][OW]; ep: alpha_a / beta_a scalar, alpha_w / beta_w per channel
struct DwConvArgs {
    const int8_t* a;
    const int8_t* w;
    int64_t Kp;
    ConvGeom g;  // O = C
    int32_t* acc;
    float* y;
    EpiArgs ep;
    int tiles_per_block;  // set by launch_dwconv: consecutive pixel tiles a block of the 3 x 3 kernel walks
};
hipError_t launch_dwconv(const DwConvArgs& a, hipStream_t st);

hipError_t launch_epilogue_gemm(const int32_t* acc, int64_t M, int64_t N, int64_t K,
                                const EpiArgs& ep, float* y, hipStream_t st);
hipError_t launch_epilogue_conv(const int32_t* acc, const ConvGeom& g, const EpiArgs& ep, float* y,
                                hipStream_t st);

}  // namespace rtn
