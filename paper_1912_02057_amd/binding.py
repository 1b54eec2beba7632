"""Thin Python binding of librtn's C ABI (see include/rtn.h).

Argument marshalling only: torch tensors supply device memory and the current
HIP stream; every step of the path runs in the library's kernels.  There is no
CPU fallback -- if librtn.so is missing or cannot be loaded this raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librtn.so")

RTN_OK = 0
RTN_ERR_NULL, RTN_ERR_SHAPE, RTN_ERR_ALIGN, RTN_ERR_UNSUPPORTED, RTN_ERR_WORKSPACE, RTN_ERR_HIP = \
    -1, -2, -3, -4, -5, -6
RTN_CODE_I8, RTN_CODE_BITPLANE, RTN_CODE_FP4 = 0, 1, 2
RTN_SCALAR, RTN_VECTOR = 0, 1
RTN_ROWS_K_CONTIG, RTN_NCHW = 0, 1
RTN_PAD_TRUE_ZERO, RTN_PAD_CODE_ZERO = 0, 1
RTN_PATH_AUTO, RTN_PATH_MFMA_I8, RTN_PATH_POPC, RTN_PATH_MFMA_FP4 = 0, 1, 2, 3

EXPORTS = ["rtn_status_string", "rtn_last_hip_error", "rtn_num_tile_configs", "rtn_set_tile_config", "rtn_padded_k", "rtn_padded_k_format",
           "rtn_codes_bytes",
           "rtn_ternarize_pack", "rtn_ternary_gemm", "rtn_conv2d_workspace_bytes",
           "rtn_conv2d_prepare_constants",
           "rtn_ternary_conv2d_implicit_gemm", "rtn_ternary_conv2d_ternarize",
           "rtn_weight_gemm_workspace_bytes", "rtn_ternary_weight_gemm",
           "rtn_weight_conv2d_workspace_bytes", "rtn_ternary_weight_conv2d",
           "rtn_weight_gemm_prepared_bytes", "rtn_weight_gemm_prepare", "rtn_ternary_weight_gemm_prepared",
           "rtn_weight_conv2d_prepared_bytes", "rtn_weight_conv2d_prepare", "rtn_ternary_weight_conv2d_prepared",
           "rtn_activation_backward_workspace_bytes", "rtn_activation_backward",
           "rtn_activation_backward_static_max_n", "rtn_activation_backward_static", "rtn_weight_backward",
           "rtn_epilogue_reparam",
           "rtn_epilogue_reparam_conv2d", "rtn_quaternary_pack", "rtn_quaternary_gemm",
           "rtn_ternary_depthwise_conv2d"]


class RtnEpilogue(C.Structure):
    _fields_ = [("alpha_a", C.c_void_p), ("beta_a", C.c_void_p), ("gran_a", C.c_int),
                ("alpha_w", C.c_void_p), ("beta_w", C.c_void_p), ("gran_w", C.c_int),
                ("sum_ta", C.c_void_p), ("sum_tw", C.c_void_p), ("relu", C.c_int),
                ("bn_scale", C.c_void_p), ("bn_shift", C.c_void_p)]


class RtnError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().rtn_status_string(status).decode()
        if status == RTN_ERR_HIP:
            msg += " [hipError %d]" % lib().rtn_last_hip_error()
        super().__init__("%s: %s (%d)" % (where, msg, status))


_lib = None


def lib():
    """Loads librtn.so (built by build.py).  Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("librtn.so not built: run `python -m paper_1912_02057_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        i64, vp, ci = C.c_int64, C.c_void_p, C.c_int
        L.rtn_status_string.restype = C.c_char_p
        L.rtn_status_string.argtypes = [ci]
        L.rtn_last_hip_error.restype = ci
        L.rtn_padded_k.restype = i64
        L.rtn_padded_k.argtypes = [i64]
        L.rtn_padded_k_format.restype = i64
        L.rtn_padded_k_format.argtypes = [ci, i64]
        L.rtn_codes_bytes.restype = C.c_size_t
        L.rtn_codes_bytes.argtypes = [ci, i64, i64]
        L.rtn_ternarize_pack.restype = ci
        L.rtn_ternarize_pack.argtypes = [vp, ci, i64, i64, i64, i64, vp, vp, ci, ci, vp, vp, vp]
        L.rtn_ternary_gemm.restype = ci
        L.rtn_ternary_gemm.argtypes = [ci, ci, vp, vp, i64, i64, i64, vp, vp, vp, vp, C.c_size_t, vp]
        L.rtn_conv2d_workspace_bytes.restype = C.c_size_t
        L.rtn_conv2d_workspace_bytes.argtypes = [i64, ci, ci, ci]
        L.rtn_conv2d_prepare_constants.restype = ci
        L.rtn_conv2d_prepare_constants.argtypes = [i64, i64, ci, ci, ci, vp, vp, C.c_size_t, vp]
        L.rtn_ternary_conv2d_implicit_gemm.restype = ci
        L.rtn_ternary_conv2d_implicit_gemm.argtypes = [ci, ci, vp, vp, i64, i64, i64, i64, i64, ci, ci,
                                                       ci, ci, ci, vp, vp, vp, vp, C.c_size_t, vp]
        L.rtn_ternary_conv2d_ternarize.restype = ci
        L.rtn_ternary_conv2d_ternarize.argtypes = [ci, ci, vp, vp, i64, i64, i64, i64, i64, ci, ci, ci, ci,
                                                   ci, vp, vp, ci, vp, vp, ci, vp, vp, vp, C.c_size_t, vp]
        L.rtn_weight_gemm_workspace_bytes.restype = C.c_size_t
        L.rtn_weight_gemm_workspace_bytes.argtypes = [i64, i64, i64]
        L.rtn_ternary_weight_gemm.restype = ci
        L.rtn_ternary_weight_gemm.argtypes = [vp, vp, i64, i64, i64, vp, ci, ci, vp, vp, vp, vp, C.c_size_t, vp]
        L.rtn_weight_gemm_prepared_bytes.restype = C.c_size_t
        L.rtn_weight_gemm_prepared_bytes.argtypes = [i64, i64]
        L.rtn_weight_gemm_prepare.restype = ci
        L.rtn_weight_gemm_prepare.argtypes = [vp, i64, i64, vp, C.c_size_t, vp]
        L.rtn_ternary_weight_gemm_prepared.restype = ci
        L.rtn_ternary_weight_gemm_prepared.argtypes = [vp, vp, i64, i64, i64, vp, ci, ci, vp, vp, vp, vp, C.c_size_t, vp]
        L.rtn_weight_conv2d_prepared_bytes.restype = C.c_size_t
        L.rtn_weight_conv2d_prepared_bytes.argtypes = [i64, i64, ci, ci, ci]
        L.rtn_weight_conv2d_prepare.restype = ci
        L.rtn_weight_conv2d_prepare.argtypes = [vp, i64, i64, ci, ci, ci, vp, ci, vp, vp, vp, C.c_size_t, vp]
        L.rtn_ternary_weight_conv2d_prepared.restype = ci
        L.rtn_ternary_weight_conv2d_prepared.argtypes = [vp, vp, i64, i64, i64, i64, i64, ci, ci, ci, ci, ci, vp, vp,
                                                         C.c_size_t, vp]
        L.rtn_weight_conv2d_workspace_bytes.restype = C.c_size_t
        L.rtn_weight_conv2d_workspace_bytes.argtypes = [i64, i64, i64, i64, i64, ci, ci, ci]
        L.rtn_ternary_weight_conv2d.restype = ci
        L.rtn_ternary_weight_conv2d.argtypes = [vp, vp, i64, i64, i64, i64, i64, ci, ci, ci, ci, vp, ci, ci, vp,
                                                vp, vp, vp, C.c_size_t, vp]
        L.rtn_activation_backward_workspace_bytes.restype = C.c_size_t
        L.rtn_activation_backward_workspace_bytes.argtypes = [i64]
        L.rtn_activation_backward.restype = ci
        L.rtn_activation_backward.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.rtn_activation_backward_static_max_n.restype = i64
        L.rtn_activation_backward_static_max_n.argtypes = []
        L.rtn_activation_backward_static.restype = ci
        L.rtn_activation_backward_static.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp, vp]
        L.rtn_weight_backward.restype = ci
        L.rtn_weight_backward.argtypes = [vp, vp, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp]
        L.rtn_ternary_depthwise_conv2d.restype = ci
        L.rtn_ternary_depthwise_conv2d.argtypes = [vp, vp, i64, i64, i64, i64, ci, ci, ci, ci, ci, vp, vp, vp, vp]
        L.rtn_quaternary_pack.restype = ci
        L.rtn_quaternary_pack.argtypes = [vp, i64, i64, C.c_float, C.c_float, C.c_float, ci, vp, vp]
        L.rtn_quaternary_gemm.restype = ci
        L.rtn_quaternary_gemm.argtypes = [ci, ci, vp, vp, i64, i64, i64, vp, vp]
        L.rtn_epilogue_reparam.restype = ci
        L.rtn_epilogue_reparam.argtypes = [vp, i64, i64, i64, vp, vp, vp]
        L.rtn_epilogue_reparam_conv2d.restype = ci
        L.rtn_epilogue_reparam_conv2d.argtypes = [vp, i64, i64, i64, i64, i64, ci, ci, ci, ci, ci, vp,
                                                  vp, vp]
        _lib = L
    return _lib


def _check(rc, where):
    if rc != RTN_OK:
        raise RtnError(rc, where)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype):
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), (t.device, t.dtype)
    return C.c_void_p(t.data_ptr())


class _Gran:
    """A scalar (python float -> host float) or a device float32 vector."""

    def __init__(self, v):
        self.keep = None
        if v is None:
            self.ptr, self.gran = None, None
        elif torch.is_tensor(v):
            self.ptr, self.gran = _dev(v, torch.float32), RTN_VECTOR
        else:
            self.keep = C.c_float(float(v))
            self.ptr, self.gran = C.cast(C.pointer(self.keep), C.c_void_p), RTN_SCALAR


def num_tile_configs():
    return lib().rtn_num_tile_configs()


def set_tile_config(index):
    _check(lib().rtn_set_tile_config(int(index)), "rtn_set_tile_config")


def padded_k(K, fmt=RTN_CODE_I8):
    return lib().rtn_padded_k_format(fmt, K)


def ternarize_pack(x, lo, hi, fmt=RTN_CODE_I8, layout=None, want_sum=True, codes=None, sum_t=None):
    """x: cuda float32 [rows,K] (RTN_ROWS_K_CONTIG) or [N,C,H,W] (RTN_NCHW).
    lo/hi: python floats, or cuda float32 vectors (per row / per leading index).
    Returns (codes, sum_t).  codes: int8 [rows,Kpad] / [N,H,W,Cpad]; for FP4 uint8
    [rows,Kpad/2] / [N,H,W,Cpad/2] (two nibbles per byte); for bit planes
    uint64-as-int64 [2, rows, Kpad/64] / [2, N,H,W, Cpad/64]."""
    if layout is None:
        layout = RTN_NCHW if x.dim() == 4 else RTN_ROWS_K_CONTIG
    if layout == RTN_ROWS_K_CONTIG:
        d = (x.shape[0], x.shape[1], 1, 1)
        lead = (x.shape[0],)
    else:
        d = tuple(x.shape)
        lead = (x.shape[0], x.shape[2], x.shape[3])
    kp = padded_k(d[1], fmt)
    cshape = {RTN_CODE_I8: lead + (kp,), RTN_CODE_FP4: lead + (kp // 2,),
              RTN_CODE_BITPLANE: (2,) + lead + (kp // 64,)}[fmt]
    cdtype = {RTN_CODE_I8: torch.int8, RTN_CODE_FP4: torch.uint8, RTN_CODE_BITPLANE: torch.int64}[fmt]
    if codes is not None:
        assert tuple(codes.shape) == cshape and codes.dtype == cdtype and codes.is_cuda and codes.is_contiguous()
    else:
        codes = torch.empty(cshape, dtype=cdtype, device=x.device)
    if sum_t is None and want_sum:
        sum_t = torch.empty(lead, dtype=torch.int32, device=x.device)
    glo, ghi = _Gran(lo), _Gran(hi)
    assert glo.gran == ghi.gran
    rc = lib().rtn_ternarize_pack(_dev(x, torch.float32), layout, d[0], d[1], d[2], d[3], glo.ptr,
                                  ghi.ptr, glo.gran, fmt, C.c_void_p(codes.data_ptr()),
                                  None if sum_t is None else _dev(sum_t, torch.int32), _stream())
    _check(rc, "rtn_ternarize_pack")
    return codes, sum_t


class Epilogue:
    """Owns the marshalled rtn_epilogue (keeps host scalars alive)."""

    def __init__(self, alpha_a, beta_a, alpha_w, beta_w, sum_ta, sum_tw, relu=False, bn_scale=None,
                 bn_shift=None):
        self._a, self._b = _Gran(alpha_a), _Gran(beta_a)
        self._c, self._d = _Gran(alpha_w), _Gran(beta_w)
        assert self._a.gran == self._b.gran
        assert self._d.gran is None or self._c.gran == self._d.gran
        self._tensors = (alpha_a, beta_a, alpha_w, beta_w, sum_ta, sum_tw, bn_scale, bn_shift)
        self.s = RtnEpilogue(self._a.ptr, self._b.ptr, self._a.gran, self._c.ptr, self._d.ptr,
                             self._c.gran, None if sum_ta is None else _dev(sum_ta, torch.int32),
                             None if sum_tw is None else _dev(sum_tw, torch.int32),
                             int(bool(relu)),
                             None if bn_scale is None else _dev(bn_scale, torch.float32),
                             None if bn_shift is None else _dev(bn_shift, torch.float32))

    def ref(self):
        return C.cast(C.pointer(self.s), C.c_void_p)


def ternary_gemm(a_codes, w_codes, M, N, K, fmt=RTN_CODE_I8, path=RTN_PATH_AUTO, ep=None,
                 want_acc=False, acc_out=None, y_out=None):
    """Returns (acc or None, y or None)."""
    dev = a_codes.device
    if fmt != RTN_CODE_BITPLANE:
        _check_codes(a_codes, M, K, fmt, "a_codes")
        _check_codes(w_codes, N, K, fmt, "w_codes")
    if want_acc and acc_out is None:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=dev)
    if ep is not None and y_out is None:
        y_out = torch.empty((M, N), dtype=torch.float32, device=dev)
    rc = lib().rtn_ternary_gemm(fmt, path, C.c_void_p(a_codes.data_ptr()), C.c_void_p(w_codes.data_ptr()),
                                M, N, K, None if acc_out is None else _dev(acc_out, torch.int32),
                                None if ep is None else ep.ref(),
                                None if y_out is None else _dev(y_out, torch.float32), None, 0, _stream())
    _check(rc, "rtn_ternary_gemm")
    return acc_out, y_out


def code_row_bytes(K, fmt=RTN_CODE_I8):
    """Bytes of one row of K codes (a pixel's channels, a GEMM row) in format fmt."""
    return lib().rtn_codes_bytes(fmt, 1, K) // (2 if fmt == RTN_CODE_BITPLANE else 1)


def _check_codes(t, rows, K, fmt, what):
    """The library takes raw pointers: make sure the tensor really holds `rows` rows of K codes in
    format fmt, so that a tensor packed in another format cannot be read out of bounds."""
    need = lib().rtn_codes_bytes(fmt, rows, K)
    have = t.numel() * t.element_size()
    if not (t.is_cuda and t.is_contiguous() and have >= need):
        raise ValueError("%s: %d bytes, but %d rows of %d codes in format %d need %d" % (what, have, rows, K, fmt, need))
    if fmt == RTN_CODE_FP4 and t.dtype != torch.uint8 or fmt == RTN_CODE_I8 and t.dtype != torch.int8:
        raise ValueError("%s: dtype %s does not match code format %d" % (what, t.dtype, fmt))


def conv2d_workspace_bytes(O, KH, KW, pad):
    return lib().rtn_conv2d_workspace_bytes(O, KH, KW, pad)


def conv2d_prepare_constants(Cc, O, KH, KW, pad, ep, workspace=None):
    """Offline: fills (and returns) the per-border-class constant table of a conv layer."""
    if workspace is None:
        workspace = torch.empty(conv2d_workspace_bytes(O, KH, KW, pad), dtype=torch.uint8,
                                device=torch.device("cuda", torch.cuda.current_device()))
    rc = lib().rtn_conv2d_prepare_constants(Cc, O, KH, KW, pad, ep.ref(), C.c_void_p(workspace.data_ptr()),
                                            workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "rtn_conv2d_prepare_constants")
    return workspace


def conv_out_hw(H, W, KH, KW, stride, pad):
    return (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1


def ternary_conv2d(a_codes, w_codes, Nb, Cc, H, W, O, KH, KW, stride, pad, pad_mode=RTN_PAD_TRUE_ZERO,
                   ep=None, want_acc=False, acc_out=None, y_out=None, workspace=None,
                   fmt=RTN_CODE_I8, path=RTN_PATH_AUTO):
    """a_codes: int8 [Nb,H,W,Cpad]; w_codes: int8 [O,KH,KW,Cpad].  Returns (acc, y) in NCHW."""
    dev = a_codes.device
    _check_codes(a_codes, Nb * H * W, Cc, fmt, "a_codes")
    _check_codes(w_codes, O * KH * KW, Cc, fmt, "w_codes")
    OH, OW = conv_out_hw(H, W, KH, KW, stride, pad)
    if want_acc and acc_out is None:
        acc_out = torch.empty((Nb, O, OH, OW), dtype=torch.int32, device=dev)
    if ep is not None and y_out is None:
        y_out = torch.empty((Nb, O, OH, OW), dtype=torch.float32, device=dev)
    if ep is not None and workspace is None:
        workspace = conv2d_prepare_constants(Cc, O, KH, KW, pad, ep)
    rc = lib().rtn_ternary_conv2d_implicit_gemm(
        fmt, path, C.c_void_p(a_codes.data_ptr()), C.c_void_p(w_codes.data_ptr()), Nb, Cc, H, W, O, KH, KW,
        stride, pad, pad_mode, None if acc_out is None else _dev(acc_out, torch.int32),
        None if ep is None else ep.ref(), None if y_out is None else _dev(y_out, torch.float32),
        None if workspace is None else C.c_void_p(workspace.data_ptr()),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "rtn_ternary_conv2d_implicit_gemm")
    return acc_out, y_out


def ternary_conv2d_ternarize(a_codes, w_codes, Nb, Cc, H, W, O, KH, KW, stride, pad, ep, lo, hi,
                             pad_mode=RTN_PAD_TRUE_ZERO, codes_out=None, workspace=None,
                             residual=None, relu_out=False, y_out=None,
                             fmt=RTN_CODE_I8, path=RTN_PATH_AUTO):
    """The conv with the ternarizing epilogue.  lo/hi: python floats or cuda float32
    vectors (one per output channel).  residual / relu_out / y_out: the block-tail
    form (fp32 NCHW tensors).  Returns int8 codes [Nb,OH,OW,padded_k(O)]."""
    OH, OW = conv_out_hw(H, W, KH, KW, stride, pad)
    _check_codes(a_codes, Nb * H * W, Cc, fmt, "a_codes")
    _check_codes(w_codes, O * KH * KW, Cc, fmt, "w_codes")
    if codes_out is not None:
        _check_codes(codes_out, Nb * OH * OW, O, fmt, "codes_out")
    if codes_out is None:
        codes_out = (torch.empty((Nb, OH, OW, padded_k(O)), dtype=torch.int8, device=a_codes.device)
                     if fmt == RTN_CODE_I8 else
                     torch.empty((Nb, OH, OW, padded_k(O, fmt) // 2), dtype=torch.uint8, device=a_codes.device))
    if workspace is None:
        workspace = conv2d_prepare_constants(Cc, O, KH, KW, pad, ep)
    glo, ghi = _Gran(lo), _Gran(hi)
    assert glo.gran == ghi.gran
    rc = lib().rtn_ternary_conv2d_ternarize(
        fmt, path, C.c_void_p(a_codes.data_ptr()), C.c_void_p(w_codes.data_ptr()), Nb, Cc, H, W, O, KH, KW,
        stride, pad, pad_mode, ep.ref(), None if residual is None else _dev(residual, torch.float32),
        int(bool(relu_out)), glo.ptr, ghi.ptr, glo.gran,
        None if y_out is None else _dev(y_out, torch.float32),
        _dev(codes_out, torch.int8 if fmt == RTN_CODE_I8 else torch.uint8),
        C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "rtn_ternary_conv2d_ternarize")
    return codes_out


def weight_gemm_prepare(w_codes, N, K):
    """Weight side of the weight-only GEMM, once per layer: returns the prepared buffer (cuda uint8)."""
    prepared = torch.empty(lib().rtn_weight_gemm_prepared_bytes(N, K), dtype=torch.uint8, device=w_codes.device)
    rc = lib().rtn_weight_gemm_prepare(C.c_void_p(w_codes.data_ptr()), N, K, C.c_void_p(prepared.data_ptr()),
                                       prepared.numel(), _stream())
    _check(rc, "rtn_weight_gemm_prepare")
    return prepared


def ternary_weight_gemm(x, w_codes, M, N, K, alpha_w, relu=False, bn_scale=None, bn_shift=None, y_out=None,
                        workspace=None, prepared=None):
    """Weight-only ternary GEMM: x cuda float32 [M,K], w_codes int8 [N,Kpad] (or None with
    prepared = weight_gemm_prepare(...)); alpha_w python float or cuda float32 [N].
    Returns y float32 [M,N]."""
    if y_out is None:
        y_out = torch.empty((M, N), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = torch.empty(lib().rtn_weight_gemm_workspace_bytes(M, N, K), dtype=torch.uint8,
                                device=x.device)
    ga = _Gran(alpha_w)
    fn = lib().rtn_ternary_weight_gemm if prepared is None else lib().rtn_ternary_weight_gemm_prepared
    wsrc = w_codes if prepared is None else prepared
    rc = fn(
        _dev(x, torch.float32), C.c_void_p(wsrc.data_ptr()), M, N, K, ga.ptr, ga.gran, int(bool(relu)),
        None if bn_scale is None else _dev(bn_scale, torch.float32),
        None if bn_shift is None else _dev(bn_shift, torch.float32), _dev(y_out, torch.float32),
        C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream())
    _check(rc, "rtn_ternary_weight_gemm")
    return y_out


def weight_conv2d_prepare(w_codes, Cc, O, KH, KW, pad, alpha_w, bn_scale=None, bn_shift=None):
    """Weight side of the weight-only conv, once per layer (bf16 weights + epilogue table)."""
    prepared = torch.empty(lib().rtn_weight_conv2d_prepared_bytes(Cc, O, KH, KW, pad), dtype=torch.uint8,
                           device=w_codes.device)
    ga = _Gran(alpha_w)
    rc = lib().rtn_weight_conv2d_prepare(
        C.c_void_p(w_codes.data_ptr()), Cc, O, KH, KW, pad, ga.ptr, ga.gran,
        None if bn_scale is None else _dev(bn_scale, torch.float32),
        None if bn_shift is None else _dev(bn_shift, torch.float32), C.c_void_p(prepared.data_ptr()),
        prepared.numel(), _stream())
    _check(rc, "rtn_weight_conv2d_prepare")
    return prepared


def ternary_weight_conv2d(x, w_codes, O, KH, KW, stride, pad, alpha_w=None, relu=False, bn_scale=None,
                          bn_shift=None, y_out=None, workspace=None, prepared=None):
    """conv form of the weight-only ternary layer: x cuda float32 [Nb,C,H,W], w_codes int8
    [O,KH,KW,Cpad]; or w_codes None and prepared = weight_conv2d_prepare(...), which already
    holds alpha_w and the BN affine.  Returns y float32 [Nb,O,OH,OW]."""
    Nb, Cc, H, W = x.shape
    OH, OW = conv_out_hw(H, W, KH, KW, stride, pad)
    if y_out is None:
        y_out = torch.empty((Nb, O, OH, OW), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = torch.empty(lib().rtn_weight_conv2d_workspace_bytes(Nb, Cc, H, W, O, KH, KW, pad),
                                dtype=torch.uint8, device=x.device)
    if prepared is not None:
        rc = lib().rtn_ternary_weight_conv2d_prepared(
            _dev(x, torch.float32), C.c_void_p(prepared.data_ptr()), Nb, Cc, H, W, O, KH, KW, stride, pad,
            int(bool(relu)), _dev(y_out, torch.float32), C.c_void_p(workspace.data_ptr()), workspace.numel(),
            _stream())
        _check(rc, "rtn_ternary_weight_conv2d_prepared")
        return y_out
    ga = _Gran(alpha_w)
    rc = lib().rtn_ternary_weight_conv2d(
        _dev(x, torch.float32), C.c_void_p(w_codes.data_ptr()), Nb, Cc, H, W, O, KH, KW, stride, pad, ga.ptr,
        ga.gran, int(bool(relu)), None if bn_scale is None else _dev(bn_scale, torch.float32),
        None if bn_shift is None else _dev(bn_shift, torch.float32), _dev(y_out, torch.float32),
        C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream())
    _check(rc, "rtn_ternary_weight_conv2d")
    return y_out


def activation_backward(a, grad_out, lo, hi, gamma, want_grad_in=True, grad_in=None, sums=None, workspace=None):
    """Backward of gamma*Q(a)+beta: returns (grad_in or None, sums) with sums a cuda float64 [2]
    tensor holding (dL/dgamma, dL/dbeta)."""
    n = a.numel()
    if want_grad_in and grad_in is None:
        grad_in = torch.empty_like(a)
    if sums is None:
        sums = torch.empty(2, dtype=torch.float64, device=a.device)
    if workspace is None:
        workspace = torch.empty(lib().rtn_activation_backward_workspace_bytes(n), dtype=torch.uint8,
                                device=a.device)
    glo, ghi, gg = _Gran(lo), _Gran(hi), _Gran(gamma)
    rc = lib().rtn_activation_backward(_dev(a, torch.float32), _dev(grad_out, torch.float32), n, glo.ptr, ghi.ptr,
                                       gg.ptr, None if grad_in is None else _dev(grad_in, torch.float32),
                                       _dev(sums, torch.float64), C.c_void_p(workspace.data_ptr()),
                                       workspace.numel(), _stream())
    _check(rc, "rtn_activation_backward")
    return grad_in, sums


def activation_backward_static(a, grad_out, lo, hi, gamma, grad_in, sums):
    """rtn_activation_backward_static: the caller passes every buffer (grad_in may be None);
    nothing is allocated here or in the library."""
    glo, ghi, gg = _Gran(lo), _Gran(hi), _Gran(gamma)
    rc = lib().rtn_activation_backward_static(_dev(a, torch.float32), _dev(grad_out, torch.float32), a.numel(),
                                              glo.ptr, ghi.ptr, gg.ptr,
                                              None if grad_in is None else _dev(grad_in, torch.float32),
                                              _dev(sums, torch.float64), _stream())
    _check(rc, "rtn_activation_backward_static")
    return grad_in, sums


def weight_backward(w, grad_out, lo, hi, k_w, b_w, alpha, want_grad_w=True, grad_w=None, sums=None):
    """Backward of alpha*Q(k_w*w + b_w) per filter: w, grad_out cuda float32 [O][K]; k_w, b_w, alpha cuda
    float32 [O].  Returns (grad_w or None, sums) with sums a cuda float64 [O][3] tensor holding
    (dL/dalpha, dL/dk_w, dL/db_w) per filter."""
    O, K = w.shape
    if want_grad_w and grad_w is None:
        grad_w = torch.empty_like(w)
    if sums is None:
        sums = torch.empty((O, 3), dtype=torch.float64, device=w.device)
    glo, ghi = _Gran(lo), _Gran(hi)
    rc = lib().rtn_weight_backward(_dev(w, torch.float32), _dev(grad_out, torch.float32), O, K, glo.ptr, ghi.ptr,
                                   _dev(k_w, torch.float32), _dev(b_w, torch.float32), _dev(alpha, torch.float32),
                                   None if grad_w is None else _dev(grad_w, torch.float32),
                                   _dev(sums, torch.float64), _stream())
    _check(rc, "rtn_weight_backward")
    return grad_w, sums


def epilogue_reparam(acc, K, ep, y_out=None):
    M, N = acc.shape
    if y_out is None:
        y_out = torch.empty((M, N), dtype=torch.float32, device=acc.device)
    rc = lib().rtn_epilogue_reparam(_dev(acc, torch.int32), M, N, K, ep.ref(), _dev(y_out, torch.float32),
                                    _stream())
    _check(rc, "rtn_epilogue_reparam")
    return y_out


def epilogue_reparam_conv2d(acc, Cc, H, W, KH, KW, stride, pad, pad_mode, ep, y_out=None):
    Nb, O, OH, OW = acc.shape
    if y_out is None:
        y_out = torch.empty_like(acc, dtype=torch.float32)
    rc = lib().rtn_epilogue_reparam_conv2d(_dev(acc, torch.int32), Nb, Cc, H, W, O, KH, KW, stride, pad,
                                           pad_mode, ep.ref(), _dev(y_out, torch.float32), _stream())
    _check(rc, "rtn_epilogue_reparam_conv2d")
    return y_out


def quaternary_pack(x, t1, t2, t3, fmt=RTN_CODE_I8):
    """x cuda float32 [rows, K] -> quaternary codes (values 0..3) in format fmt."""
    rows, K = x.shape
    kp = padded_k(K, fmt)
    if fmt == RTN_CODE_I8:
        codes = torch.empty((rows, kp), dtype=torch.int8, device=x.device)
    elif fmt == RTN_CODE_FP4:
        codes = torch.empty((rows, kp // 2), dtype=torch.uint8, device=x.device)
    else:
        codes = torch.empty((2, rows, kp // 64), dtype=torch.int64, device=x.device)
    rc = lib().rtn_quaternary_pack(_dev(x, torch.float32), rows, K, float(t1), float(t2), float(t3), fmt,
                                   C.c_void_p(codes.data_ptr()), _stream())
    _check(rc, "rtn_quaternary_pack")
    return codes


def quaternary_gemm(a_codes, w_codes, M, N, K, fmt=RTN_CODE_I8, path=RTN_PATH_AUTO, acc_out=None):
    """D[m][n] = sum_k qa*qw on quaternary codes; returns int32 [M, N]."""
    if fmt != RTN_CODE_BITPLANE:
        _check_codes(a_codes, M, K, fmt, "a_codes")
        _check_codes(w_codes, N, K, fmt, "w_codes")
    if acc_out is None:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=a_codes.device)
    rc = lib().rtn_quaternary_gemm(fmt, path, C.c_void_p(a_codes.data_ptr()), C.c_void_p(w_codes.data_ptr()), M, N, K,
                                   _dev(acc_out, torch.int32), _stream())
    _check(rc, "rtn_quaternary_gemm")
    return acc_out


def ternary_depthwise_conv2d(a_codes, w_codes, Nb, Cc, H, W, KH, KW, stride, pad, pad_mode=RTN_PAD_TRUE_ZERO, ep=None,
                             want_acc=False, acc_out=None, y_out=None):
    """a_codes int8 [Nb,H,W,Cpad]; w_codes int8 [C, padded_k(KH*KW)].  Returns (acc, y) in NCHW."""
    _check_codes(a_codes, Nb * H * W, Cc, RTN_CODE_I8, "a_codes")
    _check_codes(w_codes, Cc, KH * KW, RTN_CODE_I8, "w_codes")
    OH, OW = conv_out_hw(H, W, KH, KW, stride, pad)
    dev = a_codes.device
    if want_acc and acc_out is None:
        acc_out = torch.empty((Nb, Cc, OH, OW), dtype=torch.int32, device=dev)
    if ep is not None and y_out is None:
        y_out = torch.empty((Nb, Cc, OH, OW), dtype=torch.float32, device=dev)
    rc = lib().rtn_ternary_depthwise_conv2d(
        C.c_void_p(a_codes.data_ptr()), C.c_void_p(w_codes.data_ptr()), Nb, Cc, H, W, KH, KW, stride, pad, pad_mode,
        None if acc_out is None else _dev(acc_out, torch.int32), None if ep is None else ep.ref(),
        None if y_out is None else _dev(y_out, torch.float32), _stream())
    _check(rc, "rtn_ternary_depthwise_conv2d")
    return acc_out, y_out
