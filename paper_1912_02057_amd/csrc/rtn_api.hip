// C ABI of librtn: argument validation and dispatch.  Every check runs before
// anything is launched, so a rejected call never touches the GPU.
#include "../../include/rtn.h"

#include <hip/hip_runtime.h>

#include "rtn_kernels.h"

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return RTN_ERR_HIP;
}

constexpr int64_t kMaxDim = 0x7fffffffLL - 1024;
constexpr int64_t kMaxK = 1LL << 22;
constexpr int kMaxPad = 2;

bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }
int64_t pad64(int64_t k) { return (k + 63) / 64 * 64; }
// row length of a code tensor: FP4 rows are whole 64-byte K-steps of 128 codes
int64_t padk(rtn_code_format fmt, int64_t k) { return fmt == RTN_CODE_FP4 ? (k + 127) / 128 * 128 : pad64(k); }

// Host scalar or device vector -> kernel parameter.
int make_param(const float* p, rtn_gran gran, bool nullable, rtn::Param& out)
{
    out.ptr = nullptr;
    out.s = 0.0f;
    if (!p) return nullable ? RTN_OK : RTN_ERR_NULL;
    if (gran == RTN_SCALAR) {
        out.s = *p;
    } else if (gran == RTN_VECTOR) {
        if (!aligned(p, 4)) return RTN_ERR_ALIGN;
        out.ptr = p;
    } else {
        return RTN_ERR_UNSUPPORTED;
    }
    return RTN_OK;
}

// Validates an rtn_epilogue for the GEMM (conv = false) or conv form.  The
// matrix-core conv forms the activation sums from the codes and the table builder
// reads only weight-side sums, so those callers pass need_sum_ta = false.
int make_epilogue(const rtn_epilogue* ep, bool conv, rtn::EpiArgs& out, bool need_sum_ta = true)
{
    if (!ep) return RTN_ERR_NULL;
    if (ep->gran_a != RTN_SCALAR && ep->gran_a != RTN_VECTOR) return RTN_ERR_UNSUPPORTED;
    if (ep->gran_w != RTN_SCALAR && ep->gran_w != RTN_VECTOR) return RTN_ERR_UNSUPPORTED;
    if (conv && ep->gran_a != RTN_SCALAR) return RTN_ERR_UNSUPPORTED;
    int rc;
    if ((rc = make_param(ep->alpha_a, ep->gran_a, false, out.alpha_a)) != RTN_OK) return rc;
    if ((rc = make_param(ep->beta_a, ep->gran_a, false, out.beta_a)) != RTN_OK) return rc;
    if ((rc = make_param(ep->alpha_w, ep->gran_w, false, out.alpha_w)) != RTN_OK) return rc;
    if ((rc = make_param(ep->beta_w, ep->gran_w, true, out.beta_w)) != RTN_OK) return rc;
    if ((need_sum_ta && !ep->sum_ta) || !ep->sum_tw) return RTN_ERR_NULL;
    if (!aligned(ep->sum_ta, 4) || !aligned(ep->sum_tw, 4)) return RTN_ERR_ALIGN;
    if (ep->bn_shift && !ep->bn_scale) return RTN_ERR_NULL;
    if (!aligned(ep->bn_scale, 4) || !aligned(ep->bn_shift, 4)) return RTN_ERR_ALIGN;
    out.sum_ta = ep->sum_ta;
    out.sum_tw = ep->sum_tw;
    out.relu = ep->relu != 0;
    out.bn_scale = ep->bn_scale;
    out.bn_shift = ep->bn_shift;
    return RTN_OK;
}

int make_geom(int64_t Nb, int64_t C, int64_t H, int64_t W, int64_t O, int KH, int KW, int stride,
              int pad, rtn_pad_mode pad_mode, rtn::ConvGeom& g, rtn_code_format fmt = RTN_CODE_I8)
{
    if (Nb <= 0 || C <= 0 || H <= 0 || W <= 0 || O <= 0) return RTN_ERR_SHAPE;
    if (Nb > kMaxDim || C > kMaxDim || H > kMaxDim || W > kMaxDim || O > kMaxDim) return RTN_ERR_SHAPE;
    if (KH < 1 || KW < 1 || KH > 7 || KW > 7 || stride < 1 || stride > 64) return RTN_ERR_UNSUPPORTED;
    if (pad < 0 || pad >= KH || pad >= KW || pad > kMaxPad) return RTN_ERR_UNSUPPORTED;
    if (pad_mode != RTN_PAD_TRUE_ZERO && pad_mode != RTN_PAD_CODE_ZERO) return RTN_ERR_UNSUPPORTED;
    if (H + 2 * pad < KH || W + 2 * pad < KW) return RTN_ERR_SHAPE;
    const int64_t OH = (H + 2 * pad - KH) / stride + 1, OW = (W + 2 * pad - KW) / stride + 1;
    const int64_t Cpad = padk(fmt, C);
    if (Cpad * KH * KW > kMaxK) return RTN_ERR_SHAPE;
    if (Nb * H * W > kMaxDim || Nb * OH * OW > kMaxDim) return RTN_ERR_SHAPE;
    g.Nb = (int)Nb, g.C = (int)C, g.Cpad = (int)Cpad, g.H = (int)H, g.W = (int)W, g.O = (int)O;
    g.KH = KH, g.KW = KW, g.stride = stride, g.pad = pad, g.OH = (int)OH, g.OW = (int)OW;
    g.code_zero_pad = pad_mode == RTN_PAD_CODE_ZERO;
    g.div_ohw = rtn::make_fastdiv((uint32_t)(OH * OW));
    g.div_ow = rtn::make_fastdiv((uint32_t)OW);
    return RTN_OK;
}

}  // namespace

extern "C" {

const char* rtn_status_string(int status)
{
    switch (status) {
        case RTN_OK: return "ok";
        case RTN_ERR_NULL: return "required pointer is NULL";
        case RTN_ERR_SHAPE: return "invalid shape or size";
        case RTN_ERR_ALIGN: return "pointer not sufficiently aligned";
        case RTN_ERR_UNSUPPORTED: return "unsupported format, path, granularity or kernel geometry";
        case RTN_ERR_WORKSPACE: return "workspace missing or too small";
        case RTN_ERR_HIP: return "HIP launch failed (see rtn_last_hip_error)";
        default: return "unknown status";
    }
}

int rtn_last_hip_error(void) { return g_last_hip_error; }

int rtn_num_tile_configs(void) { return rtn::tile_config_count(); }

int rtn_set_tile_config(int index)
{
    if (index < -1 || index >= rtn::tile_config_count()) return RTN_ERR_UNSUPPORTED;
    rtn::force_tile_config(index);
    return RTN_OK;
}

int64_t rtn_padded_k(int64_t K) { return K <= 0 ? 0 : pad64(K); }

int64_t rtn_padded_k_format(rtn_code_format fmt, int64_t K)
{
    if (K <= 0 || (fmt != RTN_CODE_I8 && fmt != RTN_CODE_BITPLANE && fmt != RTN_CODE_FP4)) return 0;
    return padk(fmt, K);
}

size_t rtn_codes_bytes(rtn_code_format fmt, int64_t rows, int64_t K)
{
    if (rows <= 0 || K <= 0) return 0;
    const int64_t kp = pad64(K);
    if (fmt == RTN_CODE_I8) return (size_t)rows * (size_t)kp;
    if (fmt == RTN_CODE_BITPLANE) return (size_t)rows * (size_t)(kp / 64) * 8u * 2u;
    if (fmt == RTN_CODE_FP4) return (size_t)rows * (size_t)(padk(fmt, K) / 2);
    return 0;
}

int rtn_ternarize_pack(const float* x, rtn_layout layout, int64_t d0, int64_t d1, int64_t d2,
                       int64_t d3, const float* thr_lo, const float* thr_hi, rtn_gran thr_gran,
                       rtn_code_format fmt, void* codes, int32_t* sum_t, void* stream)
{
    if (!x || !codes || !thr_lo || !thr_hi) return RTN_ERR_NULL;
    if (layout != RTN_ROWS_K_CONTIG && layout != RTN_NCHW) return RTN_ERR_UNSUPPORTED;
    if (fmt != RTN_CODE_I8 && fmt != RTN_CODE_BITPLANE && fmt != RTN_CODE_FP4) return RTN_ERR_UNSUPPORTED;
    if (d0 <= 0 || d1 <= 0 || d2 <= 0 || d3 <= 0) return RTN_ERR_SHAPE;
    if (d0 > kMaxDim || d1 > kMaxDim || d2 > kMaxDim || d3 > kMaxDim) return RTN_ERR_SHAPE;
    if (layout == RTN_ROWS_K_CONTIG && (d2 != 1 || d3 != 1)) return RTN_ERR_SHAPE;
    if (d2 * d3 > kMaxDim || d0 * d2 * d3 > kMaxDim) return RTN_ERR_SHAPE;
    if ((double)d0 * (double)d1 * (double)d2 * (double)d3 >= 1099511627776.0) return RTN_ERR_SHAPE;
    if (!aligned(x, 4) || !aligned(codes, 16) || !aligned(sum_t, 4)) return RTN_ERR_ALIGN;

    rtn::PackArgs a = {};
    int rc;
    if ((rc = make_param(thr_lo, thr_gran, false, a.lo)) != RTN_OK) return rc;
    if ((rc = make_param(thr_hi, thr_gran, false, a.hi)) != RTN_OK) return rc;
    if (thr_gran == RTN_SCALAR && !(a.lo.s <= a.hi.s)) return RTN_ERR_SHAPE;
    a.x = x;
    a.codes = codes;
    a.sum_t = sum_t;
    a.K = d1;
    a.Kpad = padk(fmt, d1);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (layout == RTN_ROWS_K_CONTIG) {
        a.rows = d0;
        e = fmt == RTN_CODE_I8    ? rtn::launch_pack_rows_i8(a, st)
            : fmt == RTN_CODE_FP4 ? rtn::launch_pack_rows_fp4(a, st)
                                  : rtn::launch_pack_rows_planes(a, st);
    } else {
        a.N = d0;
        a.HW = d2 * d3;
        if (fmt != RTN_CODE_BITPLANE && a.Kpad > 2048) return RTN_ERR_UNSUPPORTED;
        const int64_t tiles = (a.HW + 63) / 64;
        if (tiles * a.N > kMaxDim) return RTN_ERR_SHAPE;
        e = fmt == RTN_CODE_I8    ? rtn::launch_pack_nchw_i8(a, st)
            : fmt == RTN_CODE_FP4 ? rtn::launch_pack_nchw_fp4(a, st)
                                  : rtn::launch_pack_nchw_planes(a, st);
    }
    return e == hipSuccess ? RTN_OK : hip_fail(e);
}

int rtn_ternary_gemm(rtn_code_format fmt, rtn_path path, const void* a_codes, const void* w_codes,
                     int64_t M, int64_t N, int64_t K, int32_t* acc_out, const rtn_epilogue* ep,
                     float* y_out, void* workspace, size_t workspace_bytes, void* stream)
{
    (void)workspace;
    (void)workspace_bytes;
    if (!a_codes || !w_codes) return RTN_ERR_NULL;
    if ((ep == nullptr) != (y_out == nullptr)) return RTN_ERR_NULL;
    if (!acc_out && !y_out) return RTN_ERR_NULL;
    if (fmt != RTN_CODE_I8 && fmt != RTN_CODE_BITPLANE && fmt != RTN_CODE_FP4) return RTN_ERR_UNSUPPORTED;
    if (path != RTN_PATH_AUTO && path != RTN_PATH_MFMA_I8 && path != RTN_PATH_POPC && path != RTN_PATH_MFMA_FP4)
        return RTN_ERR_UNSUPPORTED;
    if (path == RTN_PATH_AUTO)
        path = fmt == RTN_CODE_I8 ? RTN_PATH_MFMA_I8 : (fmt == RTN_CODE_FP4 ? RTN_PATH_MFMA_FP4 : RTN_PATH_POPC);
    if ((path == RTN_PATH_MFMA_I8) != (fmt == RTN_CODE_I8)) return RTN_ERR_UNSUPPORTED;
    if ((path == RTN_PATH_MFMA_FP4) != (fmt == RTN_CODE_FP4)) return RTN_ERR_UNSUPPORTED;
    if (M <= 0 || N <= 0 || K <= 0 || M > kMaxDim || N > kMaxDim || K > kMaxK) return RTN_ERR_SHAPE;
    if (!aligned(a_codes, 16) || !aligned(w_codes, 16) || !aligned(acc_out, 4) || !aligned(y_out, 4))
        return RTN_ERR_ALIGN;
    rtn::EpiArgs e = {};
    if (ep) {
        const int rc = make_epilogue(ep, false, e);
        if (rc != RTN_OK) return rc;
    }
    hipStream_t st = (hipStream_t)stream;
    hipError_t he;
    if (path == RTN_PATH_MFMA_I8 || path == RTN_PATH_MFMA_FP4) {
        rtn::GemmArgs g = {};
        g.a = (const int8_t*)a_codes;
        g.w = (const int8_t*)w_codes;
        g.M = M, g.N = N, g.K = K, g.Kpad = padk(fmt, K);
        g.fp4 = fmt == RTN_CODE_FP4;
        g.acc = acc_out;
        g.y = y_out;
        g.ep = e;
        he = rtn::launch_gemm_mfma(g, st);
    } else {
        rtn::PopcArgs p = {};
        const int64_t words = pad64(K) / 64;
        p.a_mask = (const uint64_t*)a_codes;
        p.a_sign = p.a_mask + M * words;
        p.w_mask = (const uint64_t*)w_codes;
        p.w_sign = p.w_mask + N * words;
        p.M = M, p.N = N, p.K = K, p.words = words;
        p.acc = acc_out;
        p.y = y_out;
        p.ep = e;
        he = rtn::launch_gemm_popc(p, st);
    }
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

size_t rtn_conv2d_workspace_bytes(int64_t O, int KH, int KW, int pad)
{
    if (O <= 0 || KH < 1 || KW < 1 || KH > 7 || KW > 7) return 0;
    if (pad < 0 || pad >= KH || pad >= KW || pad > kMaxPad) return 0;
    const int p1 = pad + 1;
    // [4 + classes] rows of O doubles, the row pitch rounded up to an even count
    return (size_t)((O + 1) & ~(int64_t)1) * (size_t)(4 + p1 * p1 * p1 * p1) * sizeof(double);
}

int rtn_conv2d_prepare_constants(int64_t C, int64_t O, int KH, int KW, int pad, const rtn_epilogue* ep,
                                 void* workspace, size_t workspace_bytes, void* stream)
{
    rtn::ConvArgs c = {};
    // geometry fields the table depends on: C, O, KH, KW, pad (image size is irrelevant)
    int rc = make_geom(1, C, KH, KW, O, KH, KW, 1, pad, RTN_PAD_TRUE_ZERO, c.g);
    if (rc != RTN_OK) return rc;
    if ((rc = make_epilogue(ep, true, c.ep, false)) != RTN_OK) return rc;
    if (!workspace || workspace_bytes < rtn_conv2d_workspace_bytes(O, KH, KW, pad)) return RTN_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return RTN_ERR_ALIGN;
    const hipError_t he = rtn::launch_conv_class_consts(c, (double*)workspace, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_ternary_conv2d_implicit_gemm(rtn_code_format fmt, rtn_path path, const void* a_codes,
                                     const void* w_codes, int64_t Nb, int64_t C, int64_t H, int64_t W,
                                     int64_t O, int KH, int KW, int stride, int pad,
                                     rtn_pad_mode pad_mode, int32_t* acc_out, const rtn_epilogue* ep,
                                     float* y_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!a_codes || !w_codes) return RTN_ERR_NULL;
    if ((ep == nullptr) != (y_out == nullptr)) return RTN_ERR_NULL;
    if (!acc_out && !y_out) return RTN_ERR_NULL;
    if (fmt != RTN_CODE_I8 && fmt != RTN_CODE_FP4) return RTN_ERR_UNSUPPORTED;
    if (path != RTN_PATH_AUTO && path != (fmt == RTN_CODE_I8 ? RTN_PATH_MFMA_I8 : RTN_PATH_MFMA_FP4))
        return RTN_ERR_UNSUPPORTED;
    rtn::ConvArgs c = {};
    int rc = make_geom(Nb, C, H, W, O, KH, KW, stride, pad, pad_mode, c.g, fmt);
    if (rc != RTN_OK) return rc;
    c.fp4 = fmt == RTN_CODE_FP4;
    if (!aligned(a_codes, 16) || !aligned(w_codes, 16) || !aligned(acc_out, 4) || !aligned(y_out, 4))
        return RTN_ERR_ALIGN;
    if (ep) {
        if ((rc = make_epilogue(ep, true, c.ep, false)) != RTN_OK) return rc;
        if (!workspace || workspace_bytes < rtn_conv2d_workspace_bytes(O, KH, KW, pad)) return RTN_ERR_WORKSPACE;
        if (!aligned(workspace, 16)) return RTN_ERR_ALIGN;
    }
    c.a = (const int8_t*)a_codes;
    c.w = (const int8_t*)w_codes;
    c.acc = acc_out;
    c.y = y_out;
    c.cst_cls = (const double*)workspace;
    hipStream_t st = (hipStream_t)stream;
    hipError_t he;
    he = rtn::launch_conv_mfma(c, st);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_ternary_conv2d_ternarize(rtn_code_format fmt, rtn_path path, const void* a_codes,
                                 const void* w_codes, int64_t Nb, int64_t C, int64_t H, int64_t W, int64_t O,
                                 int KH, int KW, int stride, int pad, rtn_pad_mode pad_mode,
                                 const rtn_epilogue* ep, const float* residual, int relu_out,
                                 const float* thr_lo, const float* thr_hi, rtn_gran thr_gran, float* y_out,
                                 void* codes_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!a_codes || !w_codes || !codes_out || !ep || !thr_lo || !thr_hi) return RTN_ERR_NULL;
    if (fmt != RTN_CODE_I8 && fmt != RTN_CODE_FP4) return RTN_ERR_UNSUPPORTED;
    if (path != RTN_PATH_AUTO && path != (fmt == RTN_CODE_I8 ? RTN_PATH_MFMA_I8 : RTN_PATH_MFMA_FP4))
        return RTN_ERR_UNSUPPORTED;
    rtn::ConvArgs c = {};
    int rc = make_geom(Nb, C, H, W, O, KH, KW, stride, pad, pad_mode, c.g, fmt);
    if (rc != RTN_OK) return rc;
    c.fp4 = fmt == RTN_CODE_FP4;
    if (!aligned(a_codes, 16) || !aligned(w_codes, 16) || !aligned(codes_out, 16)) return RTN_ERR_ALIGN;
    if (!aligned(residual, 4) || !aligned(y_out, 4)) return RTN_ERR_ALIGN;
    if ((rc = make_epilogue(ep, true, c.ep, false)) != RTN_OK) return rc;
    if ((rc = make_param(thr_lo, thr_gran, false, c.thr_lo)) != RTN_OK) return rc;
    if ((rc = make_param(thr_hi, thr_gran, false, c.thr_hi)) != RTN_OK) return rc;
    if (thr_gran == RTN_SCALAR && !(c.thr_lo.s <= c.thr_hi.s)) return RTN_ERR_SHAPE;
    if (!workspace || workspace_bytes < rtn_conv2d_workspace_bytes(O, KH, KW, pad)) return RTN_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return RTN_ERR_ALIGN;
    const int64_t ldc = c.fp4 ? padk(fmt, O) / 2 : pad64(O);  // bytes of an output pixel's code row
    if (ldc > kMaxDim || (double)c.g.Nb * c.g.OH * c.g.OW * (double)ldc >= 1099511627776.0) return RTN_ERR_SHAPE;
    c.a = (const int8_t*)a_codes;
    c.w = (const int8_t*)w_codes;
    c.cst_cls = (const double*)workspace;
    c.codes = (int8_t*)codes_out;
    c.ldc = (int)ldc;
    c.res = residual;
    c.relu_out = relu_out != 0;
    c.y = y_out;
    const hipError_t he = rtn::launch_conv_mfma(c, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

size_t rtn_weight_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0 || M > kMaxDim || N > kMaxDim || K > kMaxK) return 0;
    return (size_t)(3 * M + N) * (size_t)pad64(K) * 2u;
}

static int weight_gemm_impl(const float* x, const void* w_codes, const void* prepared, int64_t M, int64_t N, int64_t K,
                            const float* alpha_w, rtn_gran gran_w, int relu, const float* bn_scale,
                            const float* bn_shift, float* y_out, void* workspace, size_t workspace_bytes,
                            void* stream)
{
    if (!x || (!w_codes && !prepared) || !alpha_w || !y_out) return RTN_ERR_NULL;
    if (bn_shift && !bn_scale) return RTN_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0 || M > kMaxDim || N > kMaxDim || K > kMaxK) return RTN_ERR_SHAPE;
    // the three bf16 terms of a row sit side by side: 6 * Kpad bytes per row must stay below 2^31
    if (3 * pad64(K) * 2 * 256 > kMaxDim || M * pad64(K) > (int64_t)1 << 40) return RTN_ERR_SHAPE;
    if (!aligned(x, 4) || !aligned(w_codes, 16) || !aligned(prepared, 16) || !aligned(y_out, 4) || !aligned(bn_scale, 4) ||
        !aligned(bn_shift, 4))
        return RTN_ERR_ALIGN;
    rtn::WGemmArgs a = {};
    int rc;
    if (gran_w != RTN_SCALAR && gran_w != RTN_VECTOR) return RTN_ERR_UNSUPPORTED;
    if ((rc = make_param(alpha_w, gran_w, false, a.ep.alpha_w)) != RTN_OK) return rc;
    if (!workspace || workspace_bytes < rtn_weight_gemm_workspace_bytes(M, N, K)) return RTN_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return RTN_ERR_ALIGN;
    a.ep.alpha_a.s = 1.0f;
    a.ep.relu = relu != 0;
    a.ep.bn_scale = bn_scale;
    a.ep.bn_shift = bn_shift;
    a.x = x;
    a.w = (const int8_t*)w_codes;
    a.M = M, a.N = N, a.K = K, a.Kpad = pad64(K);
    a.y = y_out;
    a.workspace = workspace;
    a.prepared = prepared;
    const hipError_t he = rtn::launch_wgemm(a, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_ternary_weight_gemm(const float* x, const void* w_codes, int64_t M, int64_t N, int64_t K,
                            const float* alpha_w, rtn_gran gran_w, int relu, const float* bn_scale,
                            const float* bn_shift, float* y_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!w_codes) return RTN_ERR_NULL;
    return weight_gemm_impl(x, w_codes, nullptr, M, N, K, alpha_w, gran_w, relu, bn_scale, bn_shift, y_out, workspace,
                            workspace_bytes, stream);
}

size_t rtn_weight_gemm_prepared_bytes(int64_t N, int64_t K)
{
    if (N <= 0 || K <= 0 || N > kMaxDim || K > kMaxK) return 0;
    return (size_t)N * (size_t)pad64(K) * 2u;
}

int rtn_weight_gemm_prepare(const void* w_codes, int64_t N, int64_t K, void* prepared, size_t prepared_bytes,
                            void* stream)
{
    if (!w_codes || !prepared) return RTN_ERR_NULL;
    if (N <= 0 || K <= 0 || N > kMaxDim || K > kMaxK) return RTN_ERR_SHAPE;
    if (!aligned(w_codes, 16) || !aligned(prepared, 16)) return RTN_ERR_ALIGN;
    if (prepared_bytes < rtn_weight_gemm_prepared_bytes(N, K)) return RTN_ERR_WORKSPACE;
    const hipError_t he = rtn::launch_wgemm_prepare((const int8_t*)w_codes, N, pad64(K), prepared, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_ternary_weight_gemm_prepared(const float* x, const void* prepared, int64_t M, int64_t N, int64_t K,
                                     const float* alpha_w, rtn_gran gran_w, int relu, const float* bn_scale,
                                     const float* bn_shift, float* y_out, void* workspace, size_t workspace_bytes,
                                     void* stream)
{
    if (!prepared) return RTN_ERR_NULL;
    return weight_gemm_impl(x, nullptr, prepared, M, N, K, alpha_w, gran_w, relu, bn_scale, bn_shift, y_out, workspace,
                            workspace_bytes, stream);
}

size_t rtn_weight_conv2d_workspace_bytes(int64_t Nb, int64_t C, int64_t H, int64_t W, int64_t O, int KH, int KW,
                                         int pad)
{
    rtn::ConvGeom g = {};
    if (make_geom(Nb, C, H > KH ? H : KH, W > KW ? W : KW, O, KH, KW, 1, pad, RTN_PAD_TRUE_ZERO, g) != RTN_OK) return 0;
    if (H <= 0 || W <= 0) return 0;
    const size_t cp = (size_t)pad64(C);
    return (size_t)3 * (size_t)Nb * (size_t)H * (size_t)W * cp * 2u + (size_t)O * KH * KW * cp * 2u + 16u +
           rtn_conv2d_workspace_bytes(O, KH, KW, pad);
}

static int weight_conv_impl(const float* x, const void* w_codes, const void* prepared, int64_t Nb, int64_t C, int64_t H, int64_t W,
                              int64_t O, int KH, int KW, int stride, int pad, const float* alpha_w,
                              rtn_gran gran_w, int relu, const float* bn_scale, const float* bn_shift,
                              float* y_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || (!w_codes && !prepared) || (!alpha_w && !prepared) || !y_out) return RTN_ERR_NULL;
    if (bn_shift && !bn_scale) return RTN_ERR_NULL;
    rtn::WConvArgs a = {};
    int rc = make_geom(Nb, C, H, W, O, KH, KW, stride, pad, RTN_PAD_TRUE_ZERO, a.g);
    if (rc != RTN_OK) return rc;
    // three planes of K bytes each are walked by 32-bit offsets
    if (3 * (int64_t)a.g.Cpad * 2 * KH * KW > kMaxK || Nb * H * W * (int64_t)a.g.Cpad > (int64_t)1 << 36)
        return RTN_ERR_SHAPE;
    if (!aligned(x, 4) || !aligned(w_codes, 16) || !aligned(prepared, 16) || !aligned(y_out, 4) || !aligned(bn_scale, 4) ||
        !aligned(bn_shift, 4))
        return RTN_ERR_ALIGN;
    if (gran_w != RTN_SCALAR && gran_w != RTN_VECTOR) return RTN_ERR_UNSUPPORTED;
    if (!prepared && (rc = make_param(alpha_w, gran_w, false, a.ep.alpha_w)) != RTN_OK) return rc;
    if (!workspace || workspace_bytes < rtn_weight_conv2d_workspace_bytes(Nb, C, H, W, O, KH, KW, pad))
        return RTN_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return RTN_ERR_ALIGN;
    a.ep.alpha_a.s = 1.0f;
    a.ep.relu = relu != 0;
    a.ep.bn_scale = bn_scale;
    a.ep.bn_shift = bn_shift;
    a.x = x;
    a.w = (const int8_t*)w_codes;
    a.y = y_out;
    a.workspace = workspace;
    a.prepared = prepared;
    const hipError_t he = rtn::launch_wconv(a, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_ternary_weight_conv2d(const float* x, const void* w_codes, int64_t Nb, int64_t C, int64_t H, int64_t W,
                              int64_t O, int KH, int KW, int stride, int pad, const float* alpha_w,
                              rtn_gran gran_w, int relu, const float* bn_scale, const float* bn_shift,
                              float* y_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!w_codes) return RTN_ERR_NULL;
    return weight_conv_impl(x, w_codes, nullptr, Nb, C, H, W, O, KH, KW, stride, pad, alpha_w, gran_w, relu, bn_scale,
                            bn_shift, y_out, workspace, workspace_bytes, stream);
}

size_t rtn_weight_conv2d_prepared_bytes(int64_t C, int64_t O, int KH, int KW, int pad)
{
    rtn::ConvGeom g = {};
    if (make_geom(1, C, KH, KW, O, KH, KW, 1, pad, RTN_PAD_TRUE_ZERO, g) != RTN_OK) return 0;
    return (size_t)O * KH * KW * (size_t)pad64(C) * 2u + 16u + rtn_conv2d_workspace_bytes(O, KH, KW, pad);
}

int rtn_weight_conv2d_prepare(const void* w_codes, int64_t C, int64_t O, int KH, int KW, int pad,
                              const float* alpha_w, rtn_gran gran_w, const float* bn_scale, const float* bn_shift,
                              void* prepared, size_t prepared_bytes, void* stream)
{
    if (!w_codes || !alpha_w || !prepared) return RTN_ERR_NULL;
    if (bn_shift && !bn_scale) return RTN_ERR_NULL;
    rtn::ConvGeom g = {};
    int rc = make_geom(1, C, KH, KW, O, KH, KW, 1, pad, RTN_PAD_TRUE_ZERO, g);
    if (rc != RTN_OK) return rc;
    if (!aligned(w_codes, 16) || !aligned(prepared, 16) || !aligned(bn_scale, 4) || !aligned(bn_shift, 4))
        return RTN_ERR_ALIGN;
    if (gran_w != RTN_SCALAR && gran_w != RTN_VECTOR) return RTN_ERR_UNSUPPORTED;
    if (prepared_bytes < rtn_weight_conv2d_prepared_bytes(C, O, KH, KW, pad)) return RTN_ERR_WORKSPACE;
    rtn::EpiArgs ep = {};
    if ((rc = make_param(alpha_w, gran_w, false, ep.alpha_w)) != RTN_OK) return rc;
    ep.alpha_a.s = 1.0f;
    ep.bn_scale = bn_scale;
    ep.bn_shift = bn_shift;
    const hipError_t he = rtn::launch_wconv_prepare((const int8_t*)w_codes, g, ep, prepared, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_ternary_weight_conv2d_prepared(const float* x, const void* prepared, int64_t Nb, int64_t C, int64_t H,
                                       int64_t W, int64_t O, int KH, int KW, int stride, int pad, int relu,
                                       float* y_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!prepared) return RTN_ERR_NULL;
    return weight_conv_impl(x, nullptr, prepared, Nb, C, H, W, O, KH, KW, stride, pad, nullptr, RTN_SCALAR, relu, nullptr,
                            nullptr, y_out, workspace, workspace_bytes, stream);
}

size_t rtn_activation_backward_workspace_bytes(int64_t n)
{
    if (n <= 0 || n > ((int64_t)1 << 40)) return 0;
    return (size_t)rtn::act_backward_blocks(n) * 2u * sizeof(double);
}

int rtn_activation_backward(const float* a, const float* grad_out, int64_t n, const float* thr_lo,
                            const float* thr_hi, const float* gamma, float* grad_in, double* grad_gamma_beta,
                            void* workspace, size_t workspace_bytes, void* stream)
{
    if (!a || !grad_out || !thr_lo || !thr_hi || !gamma || !grad_gamma_beta) return RTN_ERR_NULL;
    if (n <= 0 || n > ((int64_t)1 << 40) || rtn::act_backward_blocks(n) > kMaxDim) return RTN_ERR_SHAPE;
    if (!(*thr_lo <= *thr_hi)) return RTN_ERR_SHAPE;
    if (!aligned(a, 4) || !aligned(grad_out, 4) || !aligned(grad_in, 4) || !aligned(grad_gamma_beta, 8))
        return RTN_ERR_ALIGN;
    if (!workspace || workspace_bytes < rtn_activation_backward_workspace_bytes(n)) return RTN_ERR_WORKSPACE;
    if (!aligned(workspace, 8)) return RTN_ERR_ALIGN;
    rtn::ActBwdArgs p = {};
    p.a = a, p.g = grad_out, p.n = n;
    p.lo = *thr_lo, p.hi = *thr_hi, p.gamma = *gamma;
    p.da = grad_in;
    p.partials = (double*)workspace;
    p.sums = grad_gamma_beta;
    const hipError_t he = rtn::launch_act_backward(p, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int64_t rtn_activation_backward_static_max_n(void) { return rtn::act_backward_static_max_n(); }

int rtn_activation_backward_static(const float* a, const float* grad_out, int64_t n, const float* thr_lo,
                                   const float* thr_hi, const float* gamma, float* grad_in,
                                   double* grad_gamma_beta, void* stream)
{
    if (!a || !grad_out || !thr_lo || !thr_hi || !gamma || !grad_gamma_beta) return RTN_ERR_NULL;
    if (n <= 0 || n > rtn::act_backward_static_max_n()) return RTN_ERR_SHAPE;
    if (!(*thr_lo <= *thr_hi)) return RTN_ERR_SHAPE;
    if (!aligned(a, 4) || !aligned(grad_out, 4) || !aligned(grad_in, 4) || !aligned(grad_gamma_beta, 8))
        return RTN_ERR_ALIGN;
    rtn::ActBwdArgs p = {};
    p.a = a, p.g = grad_out, p.n = n;
    p.lo = *thr_lo, p.hi = *thr_hi, p.gamma = *gamma;
    p.da = grad_in;
    p.sums = grad_gamma_beta;
    const hipError_t he = rtn::launch_act_backward_static(p, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_weight_backward(const float* w, const float* grad_out, int64_t O, int64_t K, const float* thr_lo,
                        const float* thr_hi, const float* k_w, const float* b_w, const float* alpha,
                        float* grad_w, double* grad_params, void* stream)
{
    if (!w || !grad_out || !thr_lo || !thr_hi || !k_w || !b_w || !alpha || !grad_params) return RTN_ERR_NULL;
    if (O <= 0 || K <= 0 || O > kMaxDim || K > kMaxK) return RTN_ERR_SHAPE;
    if (!(*thr_lo <= *thr_hi)) return RTN_ERR_SHAPE;
    if (!aligned(w, 4) || !aligned(grad_out, 4) || !aligned(grad_w, 4) || !aligned(k_w, 4) || !aligned(b_w, 4) ||
        !aligned(alpha, 4) || !aligned(grad_params, 8))
        return RTN_ERR_ALIGN;
    rtn::WeightBwdArgs p = {};
    p.w = w, p.g = grad_out, p.O = O, p.K = K;
    p.lo = *thr_lo, p.hi = *thr_hi;
    p.kw = k_w, p.bw = b_w, p.alpha = alpha;
    p.dw = grad_w;
    p.sums = grad_params;
    const hipError_t he = rtn::launch_weight_backward(p, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_ternary_depthwise_conv2d(const void* a_codes, const void* w_codes, int64_t Nb, int64_t C, int64_t H,
                                 int64_t W, int KH, int KW, int stride, int pad, rtn_pad_mode pad_mode,
                                 int32_t* acc_out, const rtn_epilogue* ep, float* y_out, void* stream)
{
    if (!a_codes || !w_codes) return RTN_ERR_NULL;
    if ((ep == nullptr) != (y_out == nullptr)) return RTN_ERR_NULL;
    if (!acc_out && !y_out) return RTN_ERR_NULL;
    rtn::DwConvArgs d = {};
    int rc = make_geom(Nb, C, H, W, C, KH, KW, stride, pad, pad_mode, d.g);
    if (rc != RTN_OK) return rc;
    if (!aligned(a_codes, 16) || !aligned(w_codes, 16) || !aligned(acc_out, 4) || !aligned(y_out, 4)) return RTN_ERR_ALIGN;
    if (ep) {
        if (ep->gran_a != RTN_SCALAR) return RTN_ERR_UNSUPPORTED;
        if (ep->gran_w != RTN_SCALAR && ep->gran_w != RTN_VECTOR) return RTN_ERR_UNSUPPORTED;
        if ((rc = make_param(ep->alpha_a, ep->gran_a, false, d.ep.alpha_a)) != RTN_OK) return rc;
        if ((rc = make_param(ep->beta_a, ep->gran_a, false, d.ep.beta_a)) != RTN_OK) return rc;
        if ((rc = make_param(ep->alpha_w, ep->gran_w, false, d.ep.alpha_w)) != RTN_OK) return rc;
        if ((rc = make_param(ep->beta_w, ep->gran_w, true, d.ep.beta_w)) != RTN_OK) return rc;
        if (ep->bn_shift && !ep->bn_scale) return RTN_ERR_NULL;
        if (!aligned(ep->bn_scale, 4) || !aligned(ep->bn_shift, 4)) return RTN_ERR_ALIGN;
        d.ep.relu = ep->relu != 0;
        d.ep.bn_scale = ep->bn_scale;
        d.ep.bn_shift = ep->bn_shift;
    }
    d.a = (const int8_t*)a_codes;
    d.w = (const int8_t*)w_codes;
    d.Kp = pad64((int64_t)KH * KW);
    d.acc = acc_out;
    d.y = y_out;
    const hipError_t he = rtn::launch_dwconv(d, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_quaternary_pack(const float* x, int64_t rows, int64_t K, float t1, float t2, float t3,
                        rtn_code_format fmt, void* codes, void* stream)
{
    if (!x || !codes) return RTN_ERR_NULL;
    if (fmt != RTN_CODE_I8 && fmt != RTN_CODE_BITPLANE && fmt != RTN_CODE_FP4) return RTN_ERR_UNSUPPORTED;
    if (rows <= 0 || K <= 0 || rows > kMaxDim || K > kMaxK) return RTN_ERR_SHAPE;
    if (!(t1 <= t2 && t2 <= t3)) return RTN_ERR_SHAPE;
    if (!aligned(x, 4) || !aligned(codes, 16)) return RTN_ERR_ALIGN;
    rtn::QPackArgs a = {};
    a.x = x, a.rows = rows, a.K = K, a.Kpad = padk(fmt, K);
    a.t1 = t1, a.t2 = t2, a.t3 = t3;
    a.codes = codes;
    const hipError_t he = rtn::launch_pack_rows_q4(a, (int)fmt, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_quaternary_gemm(rtn_code_format fmt, rtn_path path, const void* a_codes, const void* w_codes, int64_t M,
                        int64_t N, int64_t K, int32_t* acc_out, void* stream)
{
    if (!a_codes || !w_codes || !acc_out) return RTN_ERR_NULL;
    if (fmt != RTN_CODE_I8 && fmt != RTN_CODE_BITPLANE && fmt != RTN_CODE_FP4) return RTN_ERR_UNSUPPORTED;
    const rtn_path want = fmt == RTN_CODE_I8 ? RTN_PATH_MFMA_I8 : (fmt == RTN_CODE_FP4 ? RTN_PATH_MFMA_FP4 : RTN_PATH_POPC);
    if (path != RTN_PATH_AUTO && path != want) return RTN_ERR_UNSUPPORTED;
    // 9 K must stay an exact int32 and, on the FP4 path, an exact fp32 integer
    if (M <= 0 || N <= 0 || K <= 0 || M > kMaxDim || N > kMaxDim || K > ((int64_t)1 << 20)) return RTN_ERR_SHAPE;
    if (!aligned(a_codes, 16) || !aligned(w_codes, 16) || !aligned(acc_out, 4)) return RTN_ERR_ALIGN;
    hipError_t he;
    if (fmt == RTN_CODE_BITPLANE) {
        rtn::QPopcArgs p = {};
        const int64_t words = pad64(K) / 64;
        p.a_hi = (const uint64_t*)a_codes, p.a_lo = p.a_hi + M * words;
        p.w_hi = (const uint64_t*)w_codes, p.w_lo = p.w_hi + N * words;
        p.M = M, p.N = N, p.words = words;
        p.acc = acc_out;
        he = rtn::launch_qgemm_popc(p, (hipStream_t)stream);
    } else {
        rtn::GemmArgs g = {};
        g.a = (const int8_t*)a_codes, g.w = (const int8_t*)w_codes;
        g.M = M, g.N = N, g.K = K, g.Kpad = padk(fmt, K);
        g.fp4 = fmt == RTN_CODE_FP4;
        g.acc = acc_out;
        he = rtn::launch_gemm_mfma(g, (hipStream_t)stream);
    }
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_epilogue_reparam(const int32_t* acc, int64_t M, int64_t N, int64_t K, const rtn_epilogue* ep,
                         float* y_out, void* stream)
{
    if (!acc || !y_out) return RTN_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0 || M > kMaxDim || N > kMaxDim || K > kMaxK) return RTN_ERR_SHAPE;
    if (!aligned(acc, 4) || !aligned(y_out, 4)) return RTN_ERR_ALIGN;
    rtn::EpiArgs e = {};
    const int rc = make_epilogue(ep, false, e);
    if (rc != RTN_OK) return rc;
    const hipError_t he = rtn::launch_epilogue_gemm(acc, M, N, K, e, y_out, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

int rtn_epilogue_reparam_conv2d(const int32_t* acc, int64_t Nb, int64_t C, int64_t H, int64_t W,
                                int64_t O, int KH, int KW, int stride, int pad, rtn_pad_mode pad_mode,
                                const rtn_epilogue* ep, float* y_out, void* stream)
{
    if (!acc || !y_out) return RTN_ERR_NULL;
    rtn::ConvGeom g = {};
    int rc = make_geom(Nb, C, H, W, O, KH, KW, stride, pad, pad_mode, g);
    if (rc != RTN_OK) return rc;
    if (!aligned(acc, 4) || !aligned(y_out, 4)) return RTN_ERR_ALIGN;
    rtn::EpiArgs e = {};
    if ((rc = make_epilogue(ep, true, e)) != RTN_OK) return rc;
    const hipError_t he = rtn::launch_epilogue_conv(acc, g, e, y_out, (hipStream_t)stream);
    return he == hipSuccess ? RTN_OK : hip_fail(he);
}

}  // extern "C"
