"""Host-side checks of the C ABI (no GPU): the library loads, exports every
symbol the header declares, and rejects bad arguments with the documented
status before anything is launched."""
import ctypes as C
import os
import re

import pytest

from paper_1912_02057_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_1912_02057_amd.build import build_lib
        build_lib()
    return B.lib()


def _declared():
    txt = open(os.path.join(ROOT, "include", "rtn.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(rtn_[a-z0-9_]+)\s*\(", txt)))


def test_header_symbols_exported(L):
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_helpers(L):
    assert L.rtn_padded_k(1) == 64 and L.rtn_padded_k(64) == 64 and L.rtn_padded_k(65) == 128
    assert L.rtn_padded_k(0) == 0
    assert L.rtn_codes_bytes(B.RTN_CODE_I8, 3, 70) == 3 * 128
    assert L.rtn_codes_bytes(B.RTN_CODE_BITPLANE, 3, 70) == 3 * 2 * 8 * 2
    assert L.rtn_codes_bytes(7, 3, 70) == 0
    assert L.rtn_conv2d_workspace_bytes(64, 3, 3, 1) == 64 * 20 * 8
    assert L.rtn_conv2d_workspace_bytes(63, 3, 3, 1) == 64 * 20 * 8      # row pitch rounded up to even
    assert L.rtn_conv2d_workspace_bytes(64, 1, 1, 0) == 64 * 5 * 8
    assert L.rtn_conv2d_workspace_bytes(64, 5, 5, 2) == 64 * 85 * 8
    assert L.rtn_conv2d_workspace_bytes(64, 3, 3, 3) == 0                # pad >= kernel
    assert L.rtn_conv2d_workspace_bytes(64, 7, 7, 3) == 0                # pad above the supported 2
    assert L.rtn_status_string(0) == b"ok"
    for s in range(-6, 0):
        assert len(L.rtn_status_string(s)) > 3


FAKE = C.c_void_p(0x10000)       # never dereferenced: validation fails first
ODD = C.c_void_p(0x10002)


def _f(v):
    return C.cast(C.pointer(C.c_float(v)), C.c_void_p)


def test_ternarize_pack_rejects(L):
    lo, hi = _f(-0.5), _f(0.5)
    call = L.rtn_ternarize_pack
    ok_args = [FAKE, B.RTN_ROWS_K_CONTIG, 4, 64, 1, 1, lo, hi, B.RTN_SCALAR, B.RTN_CODE_I8, FAKE, None, None]

    def with_(i, v):
        a = list(ok_args)
        a[i] = v
        return call(*a)
    assert with_(0, None) == B.RTN_ERR_NULL
    assert with_(10, None) == B.RTN_ERR_NULL
    assert with_(6, None) == B.RTN_ERR_NULL
    assert with_(2, 0) == B.RTN_ERR_SHAPE
    assert with_(3, -5) == B.RTN_ERR_SHAPE
    assert with_(4, 2) == B.RTN_ERR_SHAPE            # rows layout needs d2 = d3 = 1
    assert with_(1, 9) == B.RTN_ERR_UNSUPPORTED
    assert with_(9, 5) == B.RTN_ERR_UNSUPPORTED
    assert with_(8, 3) == B.RTN_ERR_UNSUPPORTED
    assert with_(0, ODD) == B.RTN_ERR_ALIGN
    assert with_(10, ODD) == B.RTN_ERR_ALIGN
    assert with_(6, _f(0.7)) == B.RTN_ERR_SHAPE      # lo > hi


def _ep(gran_a=B.RTN_SCALAR, gran_w=B.RTN_SCALAR, sums=True):
    e = B.RtnEpilogue(_f(1.0), _f(0.0), gran_a, _f(1.0), None, gran_w,
                      FAKE if sums else None, FAKE if sums else None, 0, None, None)
    return e


def test_gemm_rejects(L):
    call = L.rtn_ternary_gemm
    ok = [B.RTN_CODE_I8, B.RTN_PATH_AUTO, FAKE, FAKE, 8, 8, 64, FAKE, None, None, None, 0, None]

    def with_(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return call(*a)
    assert with_(_2=None) == B.RTN_ERR_NULL
    assert with_(_7=None) == B.RTN_ERR_NULL                     # neither acc nor y
    e = _ep()
    assert with_(_8=C.byref(e)) == B.RTN_ERR_NULL               # ep without y_out
    assert with_(_4=0) == B.RTN_ERR_SHAPE
    assert with_(_6=(1 << 22) + 1) == B.RTN_ERR_SHAPE
    assert with_(_0=3) == B.RTN_ERR_UNSUPPORTED
    assert with_(_1=B.RTN_PATH_POPC) == B.RTN_ERR_UNSUPPORTED   # int8 codes on the popcount path
    assert with_(_0=B.RTN_CODE_BITPLANE, _1=B.RTN_PATH_MFMA_I8) == B.RTN_ERR_UNSUPPORTED
    assert with_(_2=ODD) == B.RTN_ERR_ALIGN
    e2 = _ep(sums=False)
    assert with_(_8=C.byref(e2), _9=FAKE) == B.RTN_ERR_NULL     # epilogue without side sums
    e3 = _ep(gran_a=5)
    assert with_(_8=C.byref(e3), _9=FAKE) == B.RTN_ERR_UNSUPPORTED


def test_conv_rejects(L):
    call = L.rtn_ternary_conv2d_implicit_gemm
    ok = [B.RTN_CODE_I8, B.RTN_PATH_AUTO, FAKE, FAKE, 1, 64, 8, 8, 64, 3, 3, 1, 1, B.RTN_PAD_TRUE_ZERO,
          FAKE, None, None, None, 0, None]

    def with_(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return call(*a)
    assert with_(_3=None) == B.RTN_ERR_NULL
    assert with_(_0=B.RTN_CODE_BITPLANE) == B.RTN_ERR_UNSUPPORTED
    assert with_(_9=8) == B.RTN_ERR_UNSUPPORTED                 # kernel size
    assert with_(_11=0) == B.RTN_ERR_UNSUPPORTED                # stride
    assert with_(_12=3) == B.RTN_ERR_UNSUPPORTED                # pad >= kernel
    assert with_(_13=4) == B.RTN_ERR_UNSUPPORTED
    assert with_(_4=0) == B.RTN_ERR_SHAPE
    assert with_(_6=1, _7=1, _12=0) == B.RTN_ERR_SHAPE          # image smaller than the kernel
    e = _ep()
    assert with_(_15=C.byref(e), _16=FAKE) == B.RTN_ERR_WORKSPACE
    assert with_(_15=C.byref(e), _16=FAKE, _17=FAKE, _18=16) == B.RTN_ERR_WORKSPACE
    ev = _ep(gran_a=B.RTN_VECTOR)
    assert with_(_15=C.byref(ev), _16=FAKE, _17=FAKE, _18=1 << 20) == B.RTN_ERR_UNSUPPORTED


def test_epilogue_rejects(L):
    e = _ep()
    assert L.rtn_epilogue_reparam(None, 4, 4, 64, C.byref(e), FAKE, None) == B.RTN_ERR_NULL
    assert L.rtn_epilogue_reparam(FAKE, 4, 4, 64, None, FAKE, None) == B.RTN_ERR_NULL
    assert L.rtn_epilogue_reparam(FAKE, 0, 4, 64, C.byref(e), FAKE, None) == B.RTN_ERR_SHAPE
    assert L.rtn_epilogue_reparam(FAKE, 4, 4, 64, C.byref(e), ODD, None) == B.RTN_ERR_ALIGN
    assert L.rtn_epilogue_reparam_conv2d(FAKE, 1, 64, 8, 8, 64, 3, 3, 1, 1, 0, None, FAKE, None) \
        == B.RTN_ERR_NULL
    assert L.rtn_epilogue_reparam_conv2d(FAKE, 1, 64, 8, 8, 64, 9, 3, 1, 1, 0, C.byref(e), FAKE, None) \
        == B.RTN_ERR_UNSUPPORTED


def test_binding_refuses_missing_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError):
        B.lib()


def test_prepare_constants_rejects(L):
    e = _ep()
    call = L.rtn_conv2d_prepare_constants
    assert call(64, 64, 3, 3, 1, None, FAKE, 1 << 20, None) == B.RTN_ERR_NULL
    assert call(64, 64, 3, 3, 1, C.byref(e), None, 1 << 20, None) == B.RTN_ERR_WORKSPACE
    assert call(64, 64, 3, 3, 1, C.byref(e), FAKE, 64 * 20 * 8 - 1, None) == B.RTN_ERR_WORKSPACE
    assert call(64, 64, 7, 7, 3, C.byref(e), FAKE, 1 << 20, None) == B.RTN_ERR_UNSUPPORTED   # pad above 2
    assert call(64, 64, 3, 3, 3, C.byref(e), FAKE, 1 << 20, None) == B.RTN_ERR_UNSUPPORTED   # pad >= kernel
    assert call(0, 64, 3, 3, 1, C.byref(e), FAKE, 1 << 20, None) == B.RTN_ERR_SHAPE
    assert call(64, 64, 3, 3, 1, C.byref(e), ODD, 1 << 20, None) == B.RTN_ERR_ALIGN


def test_conv_ternarize_rejects(L):
    call = L.rtn_ternary_conv2d_ternarize
    e = _ep()
    lo, hi = _f(-0.5), _f(0.5)
    ok = [B.RTN_CODE_I8, B.RTN_PATH_AUTO, FAKE, FAKE, 1, 64, 8, 8, 64, 3, 3, 1, 1, B.RTN_PAD_TRUE_ZERO,
          C.byref(e), None, 0, lo, hi, B.RTN_SCALAR, None, FAKE, FAKE, 1 << 20, None]

    def with_(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return call(*a)
    assert with_(_2=None) == B.RTN_ERR_NULL
    assert with_(_14=None) == B.RTN_ERR_NULL                    # the epilogue is not optional here
    assert with_(_17=None) == B.RTN_ERR_NULL                    # thresholds
    assert with_(_21=None) == B.RTN_ERR_NULL                    # codes_out
    assert with_(_21=ODD) == B.RTN_ERR_ALIGN
    assert with_(_15=ODD) == B.RTN_ERR_ALIGN                    # residual
    assert with_(_20=ODD) == B.RTN_ERR_ALIGN                    # y_out
    assert with_(_0=B.RTN_CODE_BITPLANE) == B.RTN_ERR_UNSUPPORTED
    assert with_(_1=B.RTN_PATH_POPC) == B.RTN_ERR_UNSUPPORTED
    assert with_(_12=3) == B.RTN_ERR_UNSUPPORTED                # pad >= kernel
    assert with_(_19=7) == B.RTN_ERR_UNSUPPORTED                # threshold granularity
    assert with_(_17=_f(0.5), _18=_f(-0.5)) == B.RTN_ERR_SHAPE  # lo > hi
    assert with_(_4=0) == B.RTN_ERR_SHAPE
    assert with_(_22=None) == B.RTN_ERR_WORKSPACE
    assert with_(_23=16) == B.RTN_ERR_WORKSPACE
    assert with_(_22=ODD) == B.RTN_ERR_ALIGN
    e2 = _ep(sums=False)
    assert with_(_14=C.byref(e2)) == B.RTN_ERR_NULL             # weight tap sums are required


def test_weight_gemm_rejects(L):
    call = L.rtn_ternary_weight_gemm
    a1 = _f(1.0)
    ok = [FAKE, FAKE, 8, 8, 64, a1, B.RTN_SCALAR, 0, None, None, FAKE, FAKE, 1 << 20, None]

    def with_(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return call(*a)
    assert L.rtn_weight_gemm_workspace_bytes(8, 8, 64) == (3 * 8 + 8) * 64 * 2
    assert L.rtn_weight_gemm_workspace_bytes(8, 8, 65) == (3 * 8 + 8) * 128 * 2
    assert L.rtn_weight_gemm_workspace_bytes(0, 8, 64) == 0
    assert with_(_0=None) == B.RTN_ERR_NULL
    assert with_(_5=None) == B.RTN_ERR_NULL                     # alpha_w
    assert with_(_10=None) == B.RTN_ERR_NULL                    # y_out
    assert with_(_9=FAKE) == B.RTN_ERR_NULL                     # bn_shift without bn_scale
    assert with_(_2=0) == B.RTN_ERR_SHAPE
    assert with_(_4=(1 << 22) + 1) == B.RTN_ERR_SHAPE
    assert with_(_1=ODD) == B.RTN_ERR_ALIGN
    assert with_(_6=5) == B.RTN_ERR_UNSUPPORTED
    assert with_(_11=None) == B.RTN_ERR_WORKSPACE
    assert with_(_12=100) == B.RTN_ERR_WORKSPACE
    assert with_(_11=ODD) == B.RTN_ERR_ALIGN


def test_weight_conv_rejects(L):
    call = L.rtn_ternary_weight_conv2d
    a1 = _f(1.0)
    ok = [FAKE, FAKE, 1, 64, 8, 8, 64, 3, 3, 1, 1, a1, B.RTN_SCALAR, 0, None, None, FAKE, FAKE, 1 << 24, None]

    def with_(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return call(*a)
    wsb = L.rtn_weight_conv2d_workspace_bytes
    assert wsb(1, 64, 8, 8, 64, 3, 3, 1) == 3 * 64 * 64 * 2 + 64 * 9 * 64 * 2 + 16 + 64 * 20 * 8
    assert wsb(1, 64, 8, 8, 64, 3, 3, 3) == 0
    assert with_(_0=None) == B.RTN_ERR_NULL
    assert with_(_11=None) == B.RTN_ERR_NULL                    # alpha_w
    assert with_(_16=None) == B.RTN_ERR_NULL                    # y_out
    assert with_(_15=FAKE) == B.RTN_ERR_NULL                    # bn_shift without bn_scale
    assert with_(_7=8) == B.RTN_ERR_UNSUPPORTED                 # kernel size
    assert with_(_10=3) == B.RTN_ERR_UNSUPPORTED                # pad >= kernel
    assert with_(_2=0) == B.RTN_ERR_SHAPE
    assert with_(_1=ODD) == B.RTN_ERR_ALIGN
    assert with_(_12=5) == B.RTN_ERR_UNSUPPORTED
    assert with_(_17=None) == B.RTN_ERR_WORKSPACE
    assert with_(_18=100) == B.RTN_ERR_WORKSPACE
    assert with_(_17=ODD) == B.RTN_ERR_ALIGN


def test_weight_prepare_rejects(L):
    a1 = _f(1.0)
    assert L.rtn_weight_gemm_prepared_bytes(8, 65) == 8 * 128 * 2
    assert L.rtn_weight_gemm_prepared_bytes(0, 64) == 0
    gp = L.rtn_weight_gemm_prepare
    assert gp(None, 8, 64, FAKE, 1 << 20, None) == B.RTN_ERR_NULL
    assert gp(FAKE, 8, 64, None, 1 << 20, None) == B.RTN_ERR_NULL
    assert gp(FAKE, 0, 64, FAKE, 1 << 20, None) == B.RTN_ERR_SHAPE
    assert gp(ODD, 8, 64, FAKE, 1 << 20, None) == B.RTN_ERR_ALIGN
    assert gp(FAKE, 8, 64, FAKE, 8 * 64 * 2 - 1, None) == B.RTN_ERR_WORKSPACE
    run = L.rtn_ternary_weight_gemm_prepared
    assert run(FAKE, None, 8, 8, 64, a1, B.RTN_SCALAR, 0, None, None, FAKE, FAKE, 1 << 20, None) == B.RTN_ERR_NULL
    assert run(FAKE, ODD, 8, 8, 64, a1, B.RTN_SCALAR, 0, None, None, FAKE, FAKE, 1 << 20, None) == B.RTN_ERR_ALIGN
    assert run(FAKE, FAKE, 8, 8, 64, a1, B.RTN_SCALAR, 0, None, None, FAKE, FAKE, 100, None) == B.RTN_ERR_WORKSPACE
    pb = L.rtn_weight_conv2d_prepared_bytes
    assert pb(64, 64, 3, 3, 1) == 64 * 9 * 64 * 2 + 16 + L.rtn_conv2d_workspace_bytes(64, 3, 3, 1)
    assert pb(64, 64, 3, 3, 3) == 0
    cp = L.rtn_weight_conv2d_prepare
    ok = [FAKE, 64, 64, 3, 3, 1, a1, B.RTN_SCALAR, None, None, FAKE, 1 << 24, None]

    def with_(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return cp(*a)
    assert with_(_0=None) == B.RTN_ERR_NULL
    assert with_(_6=None) == B.RTN_ERR_NULL                     # alpha_w
    assert with_(_10=None) == B.RTN_ERR_NULL
    assert with_(_9=FAKE) == B.RTN_ERR_NULL                     # bn_shift without bn_scale
    assert with_(_5=3) == B.RTN_ERR_UNSUPPORTED                 # pad >= kernel
    assert with_(_0=ODD) == B.RTN_ERR_ALIGN
    assert with_(_7=5) == B.RTN_ERR_UNSUPPORTED
    assert with_(_11=100) == B.RTN_ERR_WORKSPACE
    crun = L.rtn_ternary_weight_conv2d_prepared
    okr = [FAKE, FAKE, 1, 64, 8, 8, 64, 3, 3, 1, 1, 0, FAKE, FAKE, 1 << 24, None]
    assert crun(*okr[:1], None, *okr[2:]) == B.RTN_ERR_NULL
    assert crun(*okr[:12], None, *okr[13:]) == B.RTN_ERR_NULL   # y_out
    assert crun(*okr[:1], ODD, *okr[2:]) == B.RTN_ERR_ALIGN
    assert crun(*okr[:14], 100, None) == B.RTN_ERR_WORKSPACE


def test_weight_backward_rejects(L):
    call = L.rtn_weight_backward
    lo, hi = _f(-0.5), _f(0.5)
    ok = [FAKE, FAKE, 64, 576, lo, hi, FAKE, FAKE, FAKE, FAKE, FAKE, None]

    def with_(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return call(*a)
    for i in (0, 1, 4, 5, 6, 7, 8, 10):                         # everything but grad_w is required
        assert with_(**{"_%d" % i: None}) == B.RTN_ERR_NULL, i
    assert with_(_2=0) == B.RTN_ERR_SHAPE
    assert with_(_3=0) == B.RTN_ERR_SHAPE
    assert with_(_3=(1 << 22) + 1) == B.RTN_ERR_SHAPE
    assert with_(_4=_f(0.5), _5=_f(-0.5)) == B.RTN_ERR_SHAPE    # lo > hi
    assert with_(_4=_f(float("nan"))) == B.RTN_ERR_SHAPE
    assert with_(_9=ODD) == B.RTN_ERR_ALIGN
    assert with_(_10=C.c_void_p(0x10004)) == B.RTN_ERR_ALIGN    # doubles need 8-byte alignment


def test_activation_backward_rejects(L):
    call = L.rtn_activation_backward
    lo, hi, gm = _f(-0.5), _f(0.5), _f(1.0)
    ok = [FAKE, FAKE, 100, lo, hi, gm, FAKE, FAKE, FAKE, 1 << 10, None]

    def with_(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return call(*a)
    assert L.rtn_activation_backward_workspace_bytes(1) == 16
    assert L.rtn_activation_backward_workspace_bytes(16385) == 32
    assert L.rtn_activation_backward_workspace_bytes(0) == 0
    assert with_(_0=None) == B.RTN_ERR_NULL
    assert with_(_5=None) == B.RTN_ERR_NULL                     # gamma
    assert with_(_7=None) == B.RTN_ERR_NULL                     # the sums are not optional
    assert with_(_2=0) == B.RTN_ERR_SHAPE
    assert with_(_3=_f(0.5), _4=_f(-0.5)) == B.RTN_ERR_SHAPE    # lo > hi
    assert with_(_6=ODD) == B.RTN_ERR_ALIGN
    assert with_(_7=C.c_void_p(0x10004)) == B.RTN_ERR_ALIGN     # doubles need 8-byte alignment
    assert with_(_8=None) == B.RTN_ERR_WORKSPACE
    assert with_(_9=8) == B.RTN_ERR_WORKSPACE


def test_activation_backward_static_rejects(L):
    call = L.rtn_activation_backward_static
    lo, hi, gm = _f(-0.5), _f(0.5), _f(1.0)
    ok = [FAKE, FAKE, 100, lo, hi, gm, FAKE, FAKE, None]

    def with_(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return call(*a)
    nmax = L.rtn_activation_backward_static_max_n()
    assert nmax == 1 << 30
    assert with_(_0=None) == B.RTN_ERR_NULL
    assert with_(_7=None) == B.RTN_ERR_NULL
    assert with_(_2=0) == B.RTN_ERR_SHAPE
    assert with_(_2=nmax + 1) == B.RTN_ERR_SHAPE                # beyond the fixed array
    assert with_(_3=_f(0.5), _4=_f(-0.5)) == B.RTN_ERR_SHAPE
    assert with_(_6=ODD) == B.RTN_ERR_ALIGN
    assert with_(_7=C.c_void_p(0x10004)) == B.RTN_ERR_ALIGN


def test_quaternary_rejects(L):
    pack, gemm = L.rtn_quaternary_pack, L.rtn_quaternary_gemm
    f = C.c_float
    assert pack(None, 4, 100, f(0.1), f(0.5), f(0.9), B.RTN_CODE_I8, FAKE, None) == B.RTN_ERR_NULL
    assert pack(FAKE, 0, 100, f(0.1), f(0.5), f(0.9), B.RTN_CODE_I8, FAKE, None) == B.RTN_ERR_SHAPE
    assert pack(FAKE, 4, 100, f(0.6), f(0.5), f(0.9), B.RTN_CODE_I8, FAKE, None) == B.RTN_ERR_SHAPE     # t1 > t2
    assert pack(FAKE, 4, 100, f(0.1), f(0.5), f(0.9), 7, FAKE, None) == B.RTN_ERR_UNSUPPORTED
    assert pack(FAKE, 4, 100, f(0.1), f(0.5), f(0.9), B.RTN_CODE_I8, ODD, None) == B.RTN_ERR_ALIGN
    assert gemm(B.RTN_CODE_I8, B.RTN_PATH_AUTO, FAKE, FAKE, 8, 8, 64, None, None) == B.RTN_ERR_NULL
    assert gemm(B.RTN_CODE_I8, B.RTN_PATH_POPC, FAKE, FAKE, 8, 8, 64, FAKE, None) == B.RTN_ERR_UNSUPPORTED
    assert gemm(B.RTN_CODE_FP4, B.RTN_PATH_MFMA_I8, FAKE, FAKE, 8, 8, 64, FAKE, None) == B.RTN_ERR_UNSUPPORTED
    assert gemm(B.RTN_CODE_FP4, B.RTN_PATH_AUTO, FAKE, FAKE, 8, 8, (1 << 20) + 1, FAKE, None) == B.RTN_ERR_SHAPE
    assert gemm(B.RTN_CODE_BITPLANE, B.RTN_PATH_AUTO, FAKE, ODD, 8, 8, 64, FAKE, None) == B.RTN_ERR_ALIGN


def test_depthwise_rejects(L):
    call = L.rtn_ternary_depthwise_conv2d
    ok = [FAKE, FAKE, 2, 64, 8, 8, 3, 3, 1, 1, 0, FAKE, None, None, None]

    def with_(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return call(*a)
    assert with_(_0=None) == B.RTN_ERR_NULL
    assert with_(_11=None) == B.RTN_ERR_NULL                 # neither accumulators nor y
    assert with_(_13=FAKE) == B.RTN_ERR_NULL                 # y without an epilogue
    assert with_(_3=0) == B.RTN_ERR_SHAPE
    assert with_(_6=9) == B.RTN_ERR_UNSUPPORTED              # kernel size
    assert with_(_9=3) == B.RTN_ERR_UNSUPPORTED              # pad >= kernel size
    assert with_(_1=ODD) == B.RTN_ERR_ALIGN


def test_fp4_format_rejects(L):
    lo, hi = _f(-0.5), _f(0.5)
    assert L.rtn_padded_k_format(B.RTN_CODE_FP4, 1) == 128 and L.rtn_padded_k_format(B.RTN_CODE_I8, 65) == 128
    assert L.rtn_padded_k_format(5, 64) == 0
    assert L.rtn_codes_bytes(B.RTN_CODE_FP4, 3, 129) == 3 * 128
    # the path must match the code format
    assert L.rtn_ternary_gemm(B.RTN_CODE_FP4, B.RTN_PATH_MFMA_I8, FAKE, FAKE, 8, 8, 64, FAKE, None, None, None, 0,
                              None) == B.RTN_ERR_UNSUPPORTED
    assert L.rtn_ternary_gemm(B.RTN_CODE_I8, B.RTN_PATH_MFMA_FP4, FAKE, FAKE, 8, 8, 64, FAKE, None, None, None, 0,
                              None) == B.RTN_ERR_UNSUPPORTED
    assert L.rtn_ternary_conv2d_implicit_gemm(B.RTN_CODE_FP4, B.RTN_PATH_MFMA_I8, FAKE, FAKE, 1, 64, 8, 8, 64, 3, 3, 1, 1,
                                              0, FAKE, None, None, None, 0, None) == B.RTN_ERR_UNSUPPORTED
    assert L.rtn_ternary_conv2d_implicit_gemm(B.RTN_CODE_BITPLANE, B.RTN_PATH_AUTO, FAKE, FAKE, 1, 64, 8, 8, 64, 3, 3, 1,
                                              1, 0, FAKE, None, None, None, 0, None) == B.RTN_ERR_UNSUPPORTED
    # NCHW packing of FP4 codes has the same channel limit as int8
    assert L.rtn_ternarize_pack(FAKE, B.RTN_NCHW, 1, 4096, 4, 4, lo, hi, B.RTN_SCALAR, B.RTN_CODE_FP4, FAKE, None,
                                None) == B.RTN_ERR_UNSUPPORTED


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it exits with status 2 and says so, before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=300)
    assert r.returncode == 2
    assert "ONE GPU" in (r.stdout + r.stderr)
