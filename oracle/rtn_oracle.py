"""ctypes wrapper around the C oracle (rtn_oracle.c) -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this.  It marshals numpy arrays to the C functions; all of the method's
arithmetic is in the C file.  Nothing here touches the HIP library.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rtn_oracle.c")
_LIB = os.path.join(_HERE, "librtn_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc -O2 (OpenMP on outermost loops only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_gemm_acc.restype = C.c_int
        _lib.orc_gemm_acc_rows.restype = C.c_int
        _lib.orc_conv_acc.restype = C.c_int
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    return None if a is None else np.ascontiguousarray(a, dtype=dt)


_i64 = C.c_int64
_f32 = C.c_float


def num_threads():
    return lib().orc_num_threads()


def ternarize(x, lo, hi):
    """O1.  x: float32 [..]; lo/hi scalars, or arrays with one entry per x.shape[0]."""
    x = _c(x, np.float32)
    lo = np.atleast_1d(np.asarray(lo, dtype=np.float32))
    hi = np.atleast_1d(np.asarray(hi, dtype=np.float32))
    per_row = int(lo.size > 1 or hi.size > 1)
    rows = x.shape[0] if per_row else 1
    if per_row:
        assert lo.size == rows and hi.size == rows
    cols = x.size // rows
    t = np.empty(x.shape, dtype=np.int8)
    lib().orc_ternarize(_p(x), _i64(rows), _i64(cols), _p(lo), _p(hi), C.c_int(per_row), _p(t))
    return t


def encode_2bit(t):
    t = _c(t, np.int8)
    v = np.empty(t.shape, dtype=np.uint8)
    lib().orc_encode_2bit(_p(t), _i64(t.size), _p(v))
    return v


def decode_2bit(v):
    v = _c(v, np.uint8)
    t = np.empty(v.shape, dtype=np.int8)
    lib().orc_decode_2bit(_p(v), _i64(v.size), _p(t))
    return t


def encode_planes(t, words=None):
    """t: int8 [rows, K] -> (mask, sign) uint64 [rows, words]."""
    t = _c(t, np.int8)
    rows, K = t.shape
    words = (K + 63) // 64 if words is None else words
    mask = np.empty((rows, words), dtype=np.uint64)
    sign = np.empty((rows, words), dtype=np.uint64)
    lib().orc_encode_planes(_p(t), _i64(rows), _i64(K), _i64(words), _p(mask), _p(sign))
    return mask, sign


def decode_planes(mask, sign, K):
    mask = _c(mask, np.uint64)
    sign = _c(sign, np.uint64)
    rows, words = mask.shape
    t = np.empty((rows, K), dtype=np.int8)
    lib().orc_decode_planes(_p(mask), _p(sign), _i64(rows), _i64(K), _i64(words), _p(t))
    return t


def e2m1_value(nibble):
    """O2b: value of an FP4 (E2M1) code point."""
    f = lib().orc_e2m1_value
    f.restype = C.c_double
    return f(C.c_int(int(nibble)))


def encode_fp4(t, Kpad=None):
    """O2b: t int8 [rows, K] -> uint8 [rows, Kpad/2], two E2M1 nibbles per byte (Kpad: K
    rounded up to a multiple of 128 unless given)."""
    t = _c(t, np.int8)
    rows, K = t.shape
    Kpad = (K + 127) // 128 * 128 if Kpad is None else Kpad
    out = np.empty((rows, Kpad // 2), dtype=np.uint8)
    lib().orc_encode_fp4(_p(t), _i64(rows), _i64(K), _i64(Kpad), _p(out))
    return out


def decode_fp4(codes, K):
    """O2b: uint8 [rows, Kpad/2] -> (t int8 [rows, K], count of nibbles that are not ternary)."""
    codes = _c(codes, np.uint8)
    rows, half = codes.shape
    t = np.empty((rows, K), dtype=np.int8)
    f = lib().orc_decode_fp4
    f.restype = C.c_int64
    bad = f(_p(codes), _i64(rows), _i64(K), _i64(2 * half), _p(t))
    return t, int(bad)


def pad_rows_i8(t, Kpad):
    t = _c(t, np.int8)
    rows, K = t.shape
    out = np.empty((rows, Kpad), dtype=np.int8)
    lib().orc_pad_rows_i8(_p(t), _i64(rows), _i64(K), _i64(Kpad), _p(out))
    return out


def nchw_to_nhwc_i8(t, Cpad):
    t = _c(t, np.int8)
    N, Cc, H, W = t.shape
    out = np.empty((N, H, W, Cpad), dtype=np.int8)
    lib().orc_nchw_to_nhwc_i8(_p(t), _i64(N), _i64(Cc), _i64(H), _i64(W), _i64(Cpad), _p(out))
    return out


def row_sums(t):
    t = _c(t, np.int8)
    rows, K = t.shape
    s = np.empty(rows, dtype=np.int32)
    lib().orc_row_sums(_p(t), _i64(rows), _i64(K), _p(s))
    return s


def pixel_sums(t):
    t = _c(t, np.int8)
    N, Cc, H, W = t.shape
    s = np.empty((N, H, W), dtype=np.int32)
    lib().orc_pixel_sums(_p(t), _i64(N), _i64(Cc), _i64(H), _i64(W), _p(s))
    return s


def gemm_acc(ta, tw):
    """O3.  ta: int8 [M,K], tw: int8 [N,K] -> int32 D [M,N]."""
    ta = _c(ta, np.int8)
    tw = _c(tw, np.int8)
    M, K = ta.shape
    N, K2 = tw.shape
    assert K == K2
    D = np.empty((M, N), dtype=np.int32)
    rc = lib().orc_gemm_acc(_p(ta), _p(tw), _i64(M), _i64(N), _i64(K), _p(D))
    assert rc == 0, "accumulator left [-K, K]"
    return D


def gemm_acc_rows(ta, tw, rows):
    ta = _c(ta, np.int8)
    tw = _c(tw, np.int8)
    rows = _c(rows, np.int64)
    M, K = ta.shape
    N = tw.shape[0]
    assert rows.size == 0 or (rows.min() >= 0 and rows.max() < M)
    D = np.empty((rows.size, N), dtype=np.int32)
    rc = lib().orc_gemm_acc_rows(_p(ta), _p(tw), _p(rows), _i64(rows.size), _i64(N), _i64(K), _p(D))
    assert rc == 0
    return D


def gemm_acc_popc(ma, sa, mw, sw):
    ma, sa, mw, sw = (_c(a, np.uint64) for a in (ma, sa, mw, sw))
    M, words = ma.shape
    N = mw.shape[0]
    D = np.empty((M, N), dtype=np.int32)
    lib().orc_gemm_acc_popc(_p(ma), _p(sa), _p(mw), _p(sw), _i64(M), _i64(N), _i64(words), _p(D))
    return D


def _gran(a, n):
    """scalar -> (array[1], stride 0); vector of n -> (array[n], stride 1)."""
    a = np.atleast_1d(np.asarray(a, dtype=np.float32))
    if a.size == 1:
        return np.ascontiguousarray(a), 0
    assert a.size == n
    return np.ascontiguousarray(a), 1


def gemm_epilogue(D, K, Sa, Sw, alpha_a, beta_a, alpha_w, beta_w=None, relu=False,
                  bn_scale=None, bn_shift=None):
    """O5.  D int32 [M,N]; Sa int32 [M]; Sw int32 [N] -> float32 y [M,N]."""
    D = _c(D, np.int32)
    M, N = D.shape
    Sa = _c(Sa, np.int32)
    Sw = _c(Sw, np.int32)
    aa, sa_ = _gran(alpha_a, M)
    ba, sb_ = _gran(beta_a, M)
    assert sa_ == sb_
    aw, sw_ = _gran(alpha_w, N)
    bw = None
    if beta_w is not None:
        bw, s2 = _gran(beta_w, N)
        assert s2 == sw_
    bs = _c(bn_scale, np.float32)
    bh = _c(bn_shift, np.float32)
    y = np.empty((M, N), dtype=np.float32)
    lib().orc_gemm_epilogue(_p(D), _i64(M), _i64(N), _i64(K), _p(Sa), _p(Sw), _p(aa), _p(ba),
                            C.c_int(sa_), _p(aw), _p(bw), C.c_int(sw_), C.c_int(int(relu)),
                            _p(bs), _p(bh), _p(y))
    return y


def gemm_direct(ta, tw, alpha_a, beta_a, alpha_w, beta_w=None):
    """O6.  float64 [M,N]."""
    ta = _c(ta, np.int8)
    tw = _c(tw, np.int8)
    M, K = ta.shape
    N = tw.shape[0]
    aa, sa_ = _gran(alpha_a, M)
    ba, _ = _gran(beta_a, M)
    aw, sw_ = _gran(alpha_w, N)
    bw = None if beta_w is None else _gran(beta_w, N)[0]
    y = np.empty((M, N), dtype=np.float64)
    lib().orc_gemm_direct(_p(ta), _p(tw), _i64(M), _i64(N), _i64(K), _p(aa), _p(ba), C.c_int(sa_),
                          _p(aw), _p(bw), C.c_int(sw_), _p(y))
    return y


def conv_out_shape(H, W, KH, KW, stride, pad):
    oh, ow = _i64(), _i64()
    lib().orc_conv_out_shape(_i64(H), _i64(W), _i64(KH), _i64(KW), _i64(stride), _i64(pad),
                             C.byref(oh), C.byref(ow))
    return oh.value, ow.value


def _geom(ta, tw):
    Nb, Cc, H, W = ta.shape
    O, C2, KH, KW = tw.shape
    assert Cc == C2
    return Nb, Cc, H, W, O, KH, KW


def conv_acc(ta, tw, stride, pad):
    """O3 for conv.  ta int8 [Nb,C,H,W], tw int8 [O,C,KH,KW] -> int32 [Nb,O,OH,OW]."""
    ta = _c(ta, np.int8)
    tw = _c(tw, np.int8)
    Nb, Cc, H, W, O, KH, KW = _geom(ta, tw)
    OH, OW = conv_out_shape(H, W, KH, KW, stride, pad)
    D = np.empty((Nb, O, OH, OW), dtype=np.int32)
    rc = lib().orc_conv_acc(_p(ta), _p(tw), _i64(Nb), _i64(Cc), _i64(H), _i64(W), _i64(O),
                            _i64(KH), _i64(KW), _i64(stride), _i64(pad), _p(D))
    assert rc == 0
    return D


def conv_sums(ta, tw, stride, pad, pad_true_zero=True):
    """O4 for conv -> Sa [Nb,OH,OW], Sw [O,OH,OW], Kv [OH,OW] (all int32)."""
    ta = _c(ta, np.int8)
    tw = _c(tw, np.int8)
    Nb, Cc, H, W, O, KH, KW = _geom(ta, tw)
    OH, OW = conv_out_shape(H, W, KH, KW, stride, pad)
    Sa = np.empty((Nb, OH, OW), dtype=np.int32)
    Sw = np.empty((O, OH, OW), dtype=np.int32)
    Kv = np.empty((OH, OW), dtype=np.int32)
    lib().orc_conv_sums(_p(ta), _p(tw), _i64(Nb), _i64(Cc), _i64(H), _i64(W), _i64(O), _i64(KH),
                        _i64(KW), _i64(stride), _i64(pad), C.c_int(int(pad_true_zero)),
                        _p(Sa), _p(Sw), _p(Kv))
    return Sa, Sw, Kv


def conv_epilogue(D, Sa, Sw, Kv, alpha_a, beta_a, alpha_w, beta_w=None, relu=False,
                  bn_scale=None, bn_shift=None):
    """O5 for conv.  alpha_a/beta_a scalars; alpha_w/beta_w scalar or per filter."""
    D = _c(D, np.int32)
    Nb, O, OH, OW = D.shape
    Sa, Sw, Kv = _c(Sa, np.int32), _c(Sw, np.int32), _c(Kv, np.int32)
    aw, sw_ = _gran(alpha_w, O)
    bw = None
    if beta_w is not None:
        bw, s2 = _gran(beta_w, O)
        assert s2 == sw_
    bs = _c(bn_scale, np.float32)
    bh = _c(bn_shift, np.float32)
    y = np.empty((Nb, O, OH, OW), dtype=np.float32)
    lib().orc_conv_epilogue(_p(D), _p(Sa), _p(Sw), _p(Kv), _i64(Nb), _i64(O), _i64(OH), _i64(OW),
                            _f32(float(alpha_a)), _f32(float(beta_a)), _p(aw), _p(bw), C.c_int(sw_),
                            C.c_int(int(relu)), _p(bs), _p(bh), _p(y))
    return y


def conv_direct(ta, tw, stride, pad, alpha_a, beta_a, alpha_w, beta_w=None, pad_true_zero=True):
    """O6 for conv.  float64 [Nb,O,OH,OW]."""
    ta = _c(ta, np.int8)
    tw = _c(tw, np.int8)
    Nb, Cc, H, W, O, KH, KW = _geom(ta, tw)
    OH, OW = conv_out_shape(H, W, KH, KW, stride, pad)
    aw, sw_ = _gran(alpha_w, O)
    bw = None if beta_w is None else _gran(beta_w, O)[0]
    y = np.empty((Nb, O, OH, OW), dtype=np.float64)
    lib().orc_conv_direct(_p(ta), _p(tw), _i64(Nb), _i64(Cc), _i64(H), _i64(W), _i64(O), _i64(KH),
                          _i64(KW), _i64(stride), _i64(pad), C.c_int(int(pad_true_zero)),
                          _f32(float(alpha_a)), _f32(float(beta_a)), _p(aw), _p(bw), C.c_int(sw_),
                          _p(y))
    return y


def ternarize_nchw(z, lo, hi):
    """O7.  z: float32 [Nb,O,OH,OW]; lo/hi scalars or one per channel -> int8 codes, same shape."""
    z = _c(z, np.float32)
    Nb, O = z.shape[0], z.shape[1]
    HW = z.size // (Nb * O)
    lo = np.atleast_1d(np.asarray(lo, dtype=np.float32))
    hi = np.atleast_1d(np.asarray(hi, dtype=np.float32))
    per_ch = int(lo.size > 1 or hi.size > 1)
    if per_ch:
        assert lo.size == O and hi.size == O
    t = np.empty(z.shape, dtype=np.int8)
    lib().orc_ternarize_nchw(_p(z), _i64(Nb), _i64(O), _i64(HW), _p(lo), _p(hi), C.c_int(per_ch), _p(t))
    return t


def conv_next_codes(D, Sa, Sw, Kv, alpha_a, beta_a, alpha_w, beta_w, relu, bn_scale, bn_shift,
                    lo, hi, Cpad):
    """O5 then O7 then the channel-innermost code layout of O2: the next ternary
    layer's input codes [Nb,OH,OW,Cpad] (int8, padding channels 0), and z itself."""
    z = conv_epilogue(D, Sa, Sw, Kv, alpha_a, beta_a, alpha_w, beta_w, relu, bn_scale, bn_shift)
    t = ternarize_nchw(z, lo, hi)
    return nchw_to_nhwc_i8(t, Cpad), z


def add_relu(z, r, relu=True):
    """O8.  One fp32 add of two fp32 tensors of the same shape, then ReLU if asked."""
    z, r = _c(z, np.float32), _c(r, np.float32)
    assert z.shape == r.shape
    out = np.empty(z.shape, dtype=np.float32)
    lib().orc_add_relu(_p(z), _p(r), _i64(z.size), C.c_int(int(relu)), _p(out))
    return out


def wgemm(x, tw, alpha_w, relu=False, bn_scale=None, bn_shift=None):
    """O9.  x: float32 [M,K]; tw: int8 [N,K]; alpha_w scalar or [N] -> float32 [M,N]."""
    x, tw = _c(x, np.float32), _c(tw, np.int8)
    M, K = x.shape
    N, K2 = tw.shape
    assert K == K2
    aw, sw_ = _gran(alpha_w, N)
    bs, bh = _c(bn_scale, np.float32), _c(bn_shift, np.float32)
    y = np.empty((M, N), dtype=np.float32)
    lib().orc_wgemm(_p(x), _p(tw), _i64(M), _i64(N), _i64(K), _p(aw), C.c_int(sw_), C.c_int(int(relu)),
                    _p(bs), _p(bh), _p(y))
    return y


def wconv(x, tw, stride, pad, alpha_w, relu=False, bn_scale=None, bn_shift=None):
    """Conv form of O9.  x: float32 [Nb,C,H,W]; tw: int8 [O,C,KH,KW] -> float32 [Nb,O,OH,OW]."""
    x, tw = _c(x, np.float32), _c(tw, np.int8)
    Nb, Cc, H, W, O, KH, KW = _geom(x, tw)
    OH, OW = conv_out_shape(H, W, KH, KW, stride, pad)
    aw, sw_ = _gran(alpha_w, O)
    bs, bh = _c(bn_scale, np.float32), _c(bn_shift, np.float32)
    y = np.empty((Nb, O, OH, OW), dtype=np.float32)
    lib().orc_wconv(_p(x), _p(tw), _i64(Nb), _i64(Cc), _i64(H), _i64(W), _i64(O), _i64(KH), _i64(KW),
                    _i64(stride), _i64(pad), _p(aw), C.c_int(sw_), C.c_int(int(relu)), _p(bs), _p(bh), _p(y))
    return y


def act_backward(a, g, lo, hi, gamma, want_da=True):
    """O10.  a, g: float32, same shape -> (da float32 or None, dgamma float, dbeta float)."""
    a, g = _c(a, np.float32), _c(g, np.float32)
    assert a.shape == g.shape
    da = np.empty(a.shape, dtype=np.float32) if want_da else None
    sums = np.zeros(2, dtype=np.float64)
    lib().orc_act_backward(_p(a), _p(g), _i64(a.size), _f32(float(lo)), _f32(float(hi)), _f32(float(gamma)),
                           _p(da), _p(sums))
    return da, float(sums[0]), float(sums[1])


def weight_backward(w, g, lo, hi, kw, bw, alpha, want_dw=True):
    """O11.  w, g: float32 [O][K]; kw, bw, alpha: float32 [O]
    -> (dw float32 [O][K] or None, sums float64 [O][3] = dalpha, dk_W, db_W per filter)."""
    w, g = _c(w, np.float32), _c(g, np.float32)
    assert w.ndim == 2 and w.shape == g.shape
    O, K = w.shape
    kw, bw, alpha = _c(kw, np.float32), _c(bw, np.float32), _c(alpha, np.float32)
    assert kw.shape == bw.shape == alpha.shape == (O,)
    dw = np.empty(w.shape, dtype=np.float32) if want_dw else None
    sums = np.zeros((O, 3), dtype=np.float64)
    lib().orc_weight_backward(_p(w), _p(g), _i64(O), _i64(K), _f32(float(lo)), _f32(float(hi)), _p(kw), _p(bw),
                              _p(alpha), _p(dw), _p(sums))
    return dw, sums


def quantize4(x, t1, t2, t3):
    """O12: q = (x > t1) + (x > t2) + (x > t3), int8 in {0,1,2,3}, same shape."""
    x = _c(x, np.float32)
    q = np.empty(x.shape, dtype=np.int8)
    lib().orc_quantize4(_p(x), _i64(x.size), _f32(float(t1)), _f32(float(t2)), _f32(float(t3)), _p(q))
    return q


def qgemm_acc(qa, qw):
    """O12: D[m][n] = sum_k qa[m][k] * qw[n][k] for quaternary codes."""
    qa, qw = _c(qa, np.int8), _c(qw, np.int8)
    M, K = qa.shape
    N = qw.shape[0]
    D = np.empty((M, N), dtype=np.int32)
    lib().orc_qgemm_acc.restype = C.c_int
    assert lib().orc_qgemm_acc(_p(qa), _p(qw), _i64(M), _i64(N), _i64(K), _p(D)) == 0
    return D


def encode_qplanes(q, words=None):
    """O12: int8 [rows, K] in {0..3} -> (hi, lo) uint64 [rows, words]."""
    q = _c(q, np.int8)
    rows, K = q.shape
    words = (K + 63) // 64 if words is None else words
    hi = np.empty((rows, words), dtype=np.uint64)
    lo = np.empty((rows, words), dtype=np.uint64)
    lib().orc_encode_qplanes(_p(q), _i64(rows), _i64(K), _i64(words), _p(hi), _p(lo))
    return hi, lo


def qgemm_bitserial(ah, al, wh, wl):
    """O12: Fig.3(b)'s pattern on the bit planes."""
    ah, al, wh, wl = (_c(a, np.uint64) for a in (ah, al, wh, wl))
    M, words = ah.shape
    N = wh.shape[0]
    D = np.empty((M, N), dtype=np.int32)
    lib().orc_qgemm_bitserial(_p(ah), _p(al), _p(wh), _p(wl), _i64(M), _i64(N), _i64(words), _p(D))
    return D


def decode_fp4_int(codes, K):
    """uint8 [rows, Kpad/2] -> (int8 [rows, K] values, count of non-integer code points)."""
    codes = _c(codes, np.uint8)
    rows, half = codes.shape
    v = np.empty((rows, K), dtype=np.int8)
    f = lib().orc_decode_fp4_int
    f.restype = C.c_int64
    bad = f(_p(codes), _i64(rows), _i64(K), _i64(2 * half), _p(v))
    return v, int(bad)


def dwconv(ta, tw, stride, pad, alpha_a, beta_a, alpha_w, beta_w=None, pad_true_zero=True, relu=False,
           bn_scale=None, bn_shift=None):
    """O13: depthwise ternary conv.  ta int8 [Nb,C,H,W], tw int8 [C,KH,KW] -> (D int32, y float32) [Nb,C,OH,OW]."""
    ta, tw = _c(ta, np.int8), _c(tw, np.int8)
    Nb, Cc, H, W = ta.shape
    KH, KW = tw.shape[1:]
    OH, OW = conv_out_shape(H, W, KH, KW, stride, pad)
    aw, sw_ = _gran(alpha_w, Cc)
    bw = None if beta_w is None else _gran(beta_w, Cc)[0]
    bs, bh = _c(bn_scale, np.float32), _c(bn_shift, np.float32)
    D = np.empty((Nb, Cc, OH, OW), dtype=np.int32)
    y = np.empty((Nb, Cc, OH, OW), dtype=np.float32)
    lib().orc_dwconv(_p(ta), _p(tw), _i64(Nb), _i64(Cc), _i64(H), _i64(W), _i64(KH), _i64(KW), _i64(stride),
                     _i64(pad), C.c_int(int(pad_true_zero)), _f32(float(alpha_a)), _f32(float(beta_a)), _p(aw),
                     _p(bw), C.c_int(sw_), C.c_int(int(relu)), _p(bs), _p(bh), _p(D), _p(y))
    return D, y
