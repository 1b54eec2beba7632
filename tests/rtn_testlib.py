"""Helpers shared by the GPU parity tests: run a workload through the oracle and
through the HIP library (via the C-ABI binding) and compare."""
import numpy as np
import torch

from oracle import rtn_oracle as orc
from paper_1912_02057_amd import binding as B

DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def thr_arg(v):
    """numpy scalar -> python float; numpy vector -> cuda tensor."""
    v = np.asarray(v, dtype=np.float32)
    return float(v) if v.ndim == 0 else dev(v)


def gran_arg(v):
    return None if v is None else thr_arg(v)


def planes_from_dev(codes):
    """[2, rows.., words] int64 device tensor -> (mask, sign) uint64 numpy [rows, words]."""
    c = codes.cpu().numpy().view(np.uint64)
    words = c.shape[-1]
    return c[0].reshape(-1, words), c[1].reshape(-1, words)


def fp4_rows(t, Kpad=None):
    """Oracle FP4 bytes of an int8 code tensor whose last axis is the row (any leading shape)."""
    t = np.ascontiguousarray(t)
    e = orc.encode_fp4(t.reshape(-1, t.shape[-1]), Kpad)
    return e.reshape(t.shape[:-1] + (e.shape[-1],))


def assert_y_close(y, yhat, what=""):
    """The stated bar: 1e-5 relative on the reparameterized outputs.  The HIP
    epilogue evaluates the four terms in fp64 and rounds once, so it sits within
    about one fp32 ulp of the oracle; the absolute floor (1e-9 of the largest
    output) only covers outputs where the four terms cancel to ~0."""
    y = np.asarray(y, dtype=np.float64)
    yhat = np.asarray(yhat, dtype=np.float64)
    assert y.shape == yhat.shape, (y.shape, yhat.shape)
    floor = 1e-9 * max(1.0, float(np.abs(yhat).max()))
    err = np.abs(y - yhat)
    bad = err > 1e-5 * np.abs(yhat) + floor
    assert not bad.any(), "%s: %d outputs off; worst abs err %g at yhat=%g" % (
        what, int(bad.sum()), float(err.max()), float(yhat.flat[int(err.argmax())]))


def oracle_gemm(case, relu=False, bn=None):
    """case from workloads.gemm_case*: returns dict of oracle results."""
    da, dw = case["delta_a"], case["delta_w"]
    ta = orc.ternarize(case["xa"], -da, da)
    tw = orc.ternarize(case["xw"], -dw, dw)
    D = orc.gemm_acc(ta, tw)
    Sa, Sw = orc.row_sums(ta), orc.row_sums(tw)
    y = orc.gemm_epilogue(D, case["K"], Sa, Sw, case["alpha_a"], case["beta_a"], case["alpha_w"],
                          case["beta_w"], relu=relu,
                          bn_scale=None if bn is None else bn[0], bn_shift=None if bn is None else bn[1])
    return dict(ta=ta, tw=tw, D=D, Sa=Sa, Sw=Sw, y=y)


def hip_gemm(case, fmt=B.RTN_CODE_I8, relu=False, bn=None, want_acc=True):
    da, dw = case["delta_a"], case["delta_w"]
    xa, xw = dev(case["xa"]), dev(case["xw"])
    ca, sa = B.ternarize_pack(xa, thr_arg(-da), thr_arg(da), fmt)
    cw, sw = B.ternarize_pack(xw, thr_arg(-dw), thr_arg(dw), fmt)
    ep = B.Epilogue(gran_arg(case["alpha_a"]), gran_arg(case["beta_a"]), gran_arg(case["alpha_w"]),
                    gran_arg(case["beta_w"]), sa, sw, relu=relu,
                    bn_scale=None if bn is None else dev(bn[0]), bn_shift=None if bn is None else dev(bn[1]))
    if want_acc == "separate":      # the two single-output launches (accumulators only, then y only)
        acc, _ = B.ternary_gemm(ca, cw, case["M"], case["N"], case["K"], fmt=fmt, ep=None, want_acc=True)
        _, y = B.ternary_gemm(ca, cw, case["M"], case["N"], case["K"], fmt=fmt, ep=ep, want_acc=False)
    else:
        acc, y = B.ternary_gemm(ca, cw, case["M"], case["N"], case["K"], fmt=fmt, ep=ep, want_acc=want_acc)
    torch.cuda.synchronize()
    return dict(ca=ca, cw=cw, Sa=sa, Sw=sw, D=acc, y=y, ep=ep)


def oracle_conv(case, pad_true_zero=True, relu=False, images=None):
    """Oracle on the whole batch, or on the listed images only."""
    sh = case["shape"]
    x = case["x"] if images is None else case["x"][images]
    da, dw = case["delta_a"], case["delta_w"]
    ta = orc.ternarize(x, -da, da)
    tw = orc.ternarize(case["w"], -np.asarray(dw), dw)
    D = orc.conv_acc(ta, tw, sh.stride, sh.pad)
    Sa, Sw, Kv = orc.conv_sums(ta, tw, sh.stride, sh.pad, pad_true_zero)
    y = orc.conv_epilogue(D, Sa, Sw, Kv, case["alpha_a"], case["beta_a"], case["alpha_w"], case["beta_w"],
                          relu=relu, bn_scale=case.get("bn_scale"), bn_shift=case.get("bn_shift"))
    return dict(ta=ta, tw=tw, D=D, y=y)


def hip_conv(case, pad_true_zero=True, relu=False, want_acc=True, fmt=B.RTN_CODE_I8):
    sh = case["shape"]
    da, dw = case["delta_a"], case["delta_w"]
    x, w = dev(case["x"]), dev(case["w"])
    ca, pa = B.ternarize_pack(x, thr_arg(-da), thr_arg(da), fmt)
    cw, pw = B.ternarize_pack(w, thr_arg(-np.asarray(dw)), thr_arg(dw), fmt)
    ep = B.Epilogue(gran_arg(case["alpha_a"]), gran_arg(case["beta_a"]), gran_arg(case["alpha_w"]),
                    gran_arg(case["beta_w"]), pa, pw, relu=relu,
                    bn_scale=None if "bn_scale" not in case else dev(case["bn_scale"]),
                    bn_shift=None if "bn_shift" not in case else dev(case["bn_shift"]))
    Nb, Cc, H, W = case["x"].shape
    pm = B.RTN_PAD_TRUE_ZERO if pad_true_zero else B.RTN_PAD_CODE_ZERO
    if want_acc == "separate":      # the two single-output launches (accumulators only, then y only)
        acc, _ = B.ternary_conv2d(ca, cw, Nb, Cc, H, W, sh.O, sh.k, sh.k, sh.stride, sh.pad, pm,
                                  ep=None, want_acc=True, fmt=fmt)
        _, y = B.ternary_conv2d(ca, cw, Nb, Cc, H, W, sh.O, sh.k, sh.k, sh.stride, sh.pad, pm,
                                ep=ep, want_acc=False, fmt=fmt)
    else:
        acc, y = B.ternary_conv2d(ca, cw, Nb, Cc, H, W, sh.O, sh.k, sh.k, sh.stride, sh.pad, pm,
                                  ep=ep, want_acc=want_acc, fmt=fmt)
    torch.cuda.synchronize()
    return dict(ca=ca, cw=cw, pa=pa, pw=pw, D=acc, y=y, ep=ep)


def oracle_next_codes(ref, lo, hi):
    """Oracle codes [Nb,OH,OW,Opad] of the next layer from an oracle_conv() result."""
    O = ref["y"].shape[1]
    return orc.nchw_to_nhwc_i8(orc.ternarize_nchw(ref["y"], lo, hi), (O + 63) // 64 * 64)


def codes_as_i8(codes, fmt, O):
    """Device code tensor [Nb,OH,OW,*] written by the ternarizing conv -> numpy int8 [Nb,OH,OW,pad64(O)].
    FP4 tensors are decoded with the oracle's decoder; every nibble must be a ternary code and
    every channel past O zero."""
    c = codes.cpu().numpy()
    if fmt == B.RTN_CODE_I8:
        return c
    assert c.dtype == np.uint8 and c.shape[-1] * 2 == (O + 127) // 128 * 128
    t, bad = orc.decode_fp4(c.reshape(-1, c.shape[-1]), c.shape[-1] * 2)
    assert bad == 0, "%d nibbles are not ternary codes" % bad
    t = t.reshape(c.shape[:-1] + (c.shape[-1] * 2,))
    assert (t[..., O:] == 0).all(), "padding channels must be code 0"
    return np.ascontiguousarray(t[..., :(O + 63) // 64 * 64])


def hip_conv_ternarize(case, lo, hi, pad_true_zero=True, relu=False, residual=None, relu_out=False,
                       want_y=False, fmt=B.RTN_CODE_I8):
    """pack -> conv with the ternarizing epilogue; returns the int8 code tensor (device),
    or (codes, y) with want_y (the block-tail form's fp32 output)."""
    sh = case["shape"]
    da, dw = case["delta_a"], case["delta_w"]
    x, w = dev(case["x"]), dev(case["w"])
    ca, _ = B.ternarize_pack(x, thr_arg(-da), thr_arg(da), fmt, want_sum=False)
    cw, pw = B.ternarize_pack(w, thr_arg(-np.asarray(dw)), thr_arg(dw), fmt)
    ep = B.Epilogue(gran_arg(case["alpha_a"]), gran_arg(case["beta_a"]), gran_arg(case["alpha_w"]),
                    gran_arg(case["beta_w"]), None, pw, relu=relu,
                    bn_scale=None if "bn_scale" not in case else dev(case["bn_scale"]),
                    bn_shift=None if "bn_shift" not in case else dev(case["bn_shift"]))
    Nb, Cc, H, W = case["x"].shape
    pm = B.RTN_PAD_TRUE_ZERO if pad_true_zero else B.RTN_PAD_CODE_ZERO
    # poison the output so that unwritten bytes (padding channels included) show
    OH, OW = B.conv_out_hw(H, W, sh.k, sh.k, sh.stride, sh.pad)
    if fmt == B.RTN_CODE_I8:
        out = torch.full((Nb, OH, OW, B.padded_k(sh.O)), 77, dtype=torch.int8, device=DEV)
    else:       # 0x77: both nibbles the code point 6.0, never a ternary code
        out = torch.full((Nb, OH, OW, B.padded_k(sh.O, fmt) // 2), 0x77, dtype=torch.uint8, device=DEV)
    y = torch.full((Nb, sh.O, OH, OW), float("nan"), dtype=torch.float32, device=DEV) if want_y else None
    codes = B.ternary_conv2d_ternarize(ca, cw, Nb, Cc, H, W, sh.O, sh.k, sh.k, sh.stride, sh.pad, ep,
                                       thr_arg(lo), thr_arg(hi), pad_mode=pm, codes_out=out,
                                       residual=None if residual is None else dev(residual),
                                       relu_out=relu_out, y_out=y, fmt=fmt)
    torch.cuda.synchronize()
    return (codes, y) if want_y else codes


def assert_codes_match(codes, want, z, lo, hi, what=""):
    """Codes decided by a floating-point comparison: both sides compare the fp32 value
    z with the fp32 thresholds.  The two sides may round z differently in its last
    bit (fp64 evaluation order), which can move a code only where z sits within a few
    fp32 ulps of a threshold; everywhere else the codes must be identical, and such
    elements must be rare.  z: oracle fp32 [Nb,O,OH,OW]; codes/want: [Nb,OH,OW,Opad]."""
    codes = np.asarray(codes)
    assert codes.shape == want.shape and codes.dtype == np.int8, (codes.shape, want.shape, codes.dtype)
    O = z.shape[1]
    assert (codes[..., O:] == 0).all(), what + ": padding channels must be code 0"
    bad = codes != want
    if not bad.any():
        return 0
    zz = z.transpose(0, 2, 3, 1).astype(np.float64)
    lo_b = np.broadcast_to(np.asarray(lo, np.float64), (O,))
    hi_b = np.broadcast_to(np.asarray(hi, np.float64), (O,))
    tol = 4e-7 * np.maximum(1.0, np.abs(zz))
    near = (np.abs(zz - lo_b) <= tol) | (np.abs(zz - hi_b) <= tol)
    badv = bad[..., :O]
    assert not (badv & ~near).any(), "%s: %d codes differ away from a threshold" % (what, int((badv & ~near).sum()))
    assert int(badv.sum()) <= 2 + zz.size // 1000000, "%s: %d codes differ at a threshold" % (what, int(badv.sum()))
    return int(badv.sum())
