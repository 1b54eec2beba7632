"""GPU parity: the HIP library (through the C ABI) against the CPU oracle on the
same seeded inputs.  Integer results (codes, side sums, accumulators) must be
bit-exact; reparameterized outputs within 1e-5 relative."""
import numpy as np
import pytest
import torch

from oracle import rtn_oracle as orc
from paper_1912_02057_amd import binding as B
from paper_1912_02057_amd import workloads as wl

import rtn_testlib as T

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)


def _sample_images(batch, n, seed):
    """n seeded images spread over the batch: first, last, the two in the middle and
    random ones between (tiles in the middle of the remapped grid included)."""
    fixed = [0, batch // 2 - 1, batch // 2, batch - 1]
    rest = np.random.default_rng(seed).choice(np.setdiff1d(np.arange(batch), fixed), n - len(fixed), replace=False)
    return sorted(set(fixed) | set(int(i) for i in rest))


def _sample_rows(M, n, seed):
    """n seeded rows of an M-row problem, first and last included, sorted."""
    rows = np.random.default_rng(seed).choice(np.arange(1, M - 1), n - 2, replace=False)
    return np.sort(np.concatenate([[0, M - 1], rows])).astype(np.int64)


# ------------------------------------------------------------ S1: pack ------
@pytest.mark.parametrize("rows,K", [(1, 1), (5, 63), (4, 64), (7, 65), (9, 200), (37, 1000), (3, 4096),
                                    (130, 258)])
@pytest.mark.parametrize("per_row", [False, True])
def test_pack_rows(rows, K, per_row):
    _say("pack_rows rows=%d K=%d per_row=%s" % (rows, K, per_row))
    rng = np.random.default_rng(rows * 1000 + K)
    x = rng.standard_normal((rows, K)).astype(np.float32)
    if per_row:
        hi = rng.uniform(0.1, 1.0, rows).astype(np.float32)
        lo = -rng.uniform(0.1, 1.0, rows).astype(np.float32)
        x[:, 0] = hi            # ties -> 0
        x[:, -1] = lo
    else:
        hi, lo = np.float32(0.62), np.float32(-0.31)   # asymmetric, as Eq.3 allows
        x.flat[:: max(1, x.size // 7)] = hi
    special = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0], np.float32)
    x.flat[1:1 + min(5, x.size - 1)] = special[: min(5, x.size - 1)]
    t = orc.ternarize(x, lo, hi)
    Kp = (K + 63) // 64 * 64
    xd = T.dev(x)
    codes, s = B.ternarize_pack(xd, T.thr_arg(lo), T.thr_arg(hi), B.RTN_CODE_I8)
    assert codes.shape == (rows, Kp)
    assert (codes.cpu().numpy() == orc.pad_rows_i8(t, Kp)).all()
    assert (s.cpu().numpy() == orc.row_sums(t)).all()
    planes, s2 = B.ternarize_pack(xd, T.thr_arg(lo), T.thr_arg(hi), B.RTN_CODE_BITPLANE)
    m, sg = T.planes_from_dev(planes)
    em, es = orc.encode_planes(t, Kp // 64)
    assert (m == em).all() and (sg == es).all()
    assert (s2.cpu().numpy() == orc.row_sums(t)).all()
    nibbles, s3 = B.ternarize_pack(xd, T.thr_arg(lo), T.thr_arg(hi), B.RTN_CODE_FP4)
    assert nibbles.shape == (rows, (K + 127) // 128 * 64)
    assert (nibbles.cpu().numpy() == orc.encode_fp4(t)).all()
    assert (s3.cpu().numpy() == orc.row_sums(t)).all()


def test_pack_rows_unaligned_base():
    # a view whose base is only 4-byte aligned takes the scalar-load variant
    _say("pack_rows unaligned base")
    rng = np.random.default_rng(5)
    buf = T.dev(rng.standard_normal(1 + 6 * 128).astype(np.float32))
    x = buf[1:].view(6, 128)
    t = orc.ternarize(x.cpu().numpy(), -0.5, 0.5)
    codes, s = B.ternarize_pack(x, -0.5, 0.5)
    assert (codes.cpu().numpy() == t).all() and (s.cpu().numpy() == orc.row_sums(t)).all()


@pytest.mark.parametrize("shape", [(2, 5, 7, 9), (3, 64, 8, 8), (2, 130, 5, 5), (1, 64, 56, 56),
                                   (8, 70, 3, 3), (4, 256, 1, 1),
                                   # 16-byte-load kernels: 128- and 256-byte output runs, channel
                                   # groups overhanging the padded row, ragged last pixel block
                                   (2, 130, 6, 6), (5, 128, 10, 10), (3, 300, 4, 4), (2, 512, 14, 14),
                                   # one-block-per-image kernel: H*W % 4 != 0, C*H*W % 4 == 0
                                   (4, 64, 7, 7), (3, 512, 7, 7), (2, 100, 3, 5)])
@pytest.mark.parametrize("per_lead", [False, True])
def test_pack_nchw(shape, per_lead):
    _say("pack_nchw %s per_lead=%s" % (shape, per_lead))
    rng = np.random.default_rng(sum(shape))
    x = rng.standard_normal(shape).astype(np.float32)
    if per_lead:
        hi = rng.uniform(0.1, 1.0, shape[0]).astype(np.float32)
        lo = -hi
        x[:, 0, 0, 0] = hi
    else:
        hi, lo = np.float32(0.4), np.float32(-0.9)
    x.flat[3] = np.nan
    t = orc.ternarize(x, lo, hi)
    Cp = (shape[1] + 63) // 64 * 64
    xd = T.dev(x)
    codes, s = B.ternarize_pack(xd, T.thr_arg(lo), T.thr_arg(hi), B.RTN_CODE_I8)
    assert tuple(codes.shape) == (shape[0], shape[2], shape[3], Cp)
    assert (codes.cpu().numpy() == orc.nchw_to_nhwc_i8(t, Cp)).all()
    assert (s.cpu().numpy() == orc.pixel_sums(t)).all()
    planes, s2 = B.ternarize_pack(xd, T.thr_arg(lo), T.thr_arg(hi), B.RTN_CODE_BITPLANE)
    m, sg = T.planes_from_dev(planes)
    em, es = orc.encode_planes(orc.nchw_to_nhwc_i8(t, shape[1]).reshape(-1, shape[1]), Cp // 64)
    assert (m == em).all() and (sg == es).all()
    assert (s2.cpu().numpy() == orc.pixel_sums(t)).all()
    nibbles, s3 = B.ternarize_pack(xd, T.thr_arg(lo), T.thr_arg(hi), B.RTN_CODE_FP4)
    assert tuple(nibbles.shape) == (shape[0], shape[2], shape[3], (shape[1] + 127) // 128 * 64)
    assert (nibbles.cpu().numpy() == T.fp4_rows(orc.nchw_to_nhwc_i8(t, shape[1]))).all()
    assert (s3.cpu().numpy() == orc.pixel_sums(t)).all()


@pytest.mark.parametrize("shape", [(3, 192, 12, 12), (2, 320, 8, 8), (6, 256, 6, 6), (2, 64, 30, 30),
                                   (7, 128, 2, 2), (1, 1024, 4, 4)])
def test_pack_nchw_straight_line_kernel(shape):
    """The NCHW pack's straight-line kernel (H*W % 4 == 0, C % 64 == 0) in its four forms: with and
    without the side sum, scalar (ordered) thresholds and per-image ones, one of which has lo > hi
    (x between them is then +1 and -1 at once, i.e. 0)."""
    _say("pack_nchw straight-line %s" % (shape,))
    rng = np.random.default_rng(11 + sum(shape))
    x = rng.standard_normal(shape).astype(np.float32)
    x.flat[5] = np.nan
    x.flat[6] = np.inf
    x.flat[7] = -np.inf
    hi_v = rng.uniform(0.1, 1.0, shape[0]).astype(np.float32)
    lo_v = -hi_v
    lo_v[-1], hi_v[-1] = np.float32(0.3), np.float32(-0.2)          # unordered pair on the last image
    x[:, 0, 0, 0] = hi_v
    xd = T.dev(x)
    for lo, hi in ((np.float32(-0.9), np.float32(0.4)), (lo_v, hi_v)):
        t = orc.ternarize(x, lo, hi)
        nhwc = orc.nchw_to_nhwc_i8(t, shape[1])
        for fmt in (B.RTN_CODE_FP4, B.RTN_CODE_I8):
            want = T.fp4_rows(nhwc) if fmt == B.RTN_CODE_FP4 else orc.nchw_to_nhwc_i8(t, (shape[1] + 63) // 64 * 64)
            codes, s = B.ternarize_pack(xd, T.thr_arg(lo), T.thr_arg(hi), fmt)
            assert (codes.cpu().numpy() == want).all()
            assert (s.cpu().numpy() == orc.pixel_sums(t)).all()
            codes2, s2 = B.ternarize_pack(xd, T.thr_arg(lo), T.thr_arg(hi), fmt, want_sum=False)
            assert s2 is None and (codes2.cpu().numpy() == want).all()


# ------------------------------------------------------ S2 + S4: GEMM -------
GEMM_SHAPES = [(1, 1, 1), (37, 19, 131), (64, 64, 64), (65, 33, 64), (300, 200, 576), (129, 257, 1000),
               (512, 384, 2048), (1024, 1024, 512)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_mfma_vs_oracle(M, N, K):
    _say("gemm_mfma M=%d N=%d K=%d" % (M, N, K))
    case = wl.gemm_case(M, N, K, p_zero=0.4, seed=M + N + K)
    ref = T.oracle_gemm(case)
    got = T.hip_gemm(case)
    assert (got["Sa"].cpu().numpy() == ref["Sa"]).all() and (got["Sw"].cpu().numpy() == ref["Sw"]).all()
    assert (got["D"].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "gemm y")
    # the accumulator equals sum t_a*t_w by an independent library route too
    assert (ref["D"] == ref["ta"].astype(np.int64) @ ref["tw"].astype(np.int64).T).all()


def test_gemm_real_inputs_relu_bn_scalar_params():
    _say("gemm real inputs, relu+bn, scalar/vector mixes")
    case = wl.gemm_case_real(200, 150, 700, seed=3)
    rng = np.random.default_rng(0)
    bn = (rng.uniform(0.5, 1.5, 150).astype(np.float32), rng.normal(0, 0.1, 150).astype(np.float32))
    ref = T.oracle_gemm(case, relu=True, bn=bn)
    got = T.hip_gemm(case, relu=True, bn=bn)
    assert (got["D"].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "gemm relu+bn")
    # scalar alpha/beta on both sides, beta_w = NULL (Eq.9 as printed)
    c2 = dict(case, alpha_a=np.float32(1.3), beta_a=np.float32(0.4), alpha_w=np.float32(0.8), beta_w=None)
    ref2, got2 = T.oracle_gemm(c2), T.hip_gemm(c2)
    T.assert_y_close(got2["y"].cpu().numpy(), ref2["y"], "gemm scalar params")
    # identity parameters return D itself
    c3 = dict(case, alpha_a=np.float32(1), beta_a=np.float32(0), alpha_w=np.float32(1), beta_w=np.float32(0))
    got3 = T.hip_gemm(c3)
    assert (got3["y"].cpu().numpy() == got3["D"].cpu().numpy().astype(np.float32)).all()


def test_gemm_acc_only_and_y_only_and_deterministic():
    _say("gemm acc-only / y-only / determinism")
    case = wl.gemm_case(260, 300, 640, seed=9)
    ref = T.oracle_gemm(case)
    g1 = T.hip_gemm(case)
    acc_only, none_y = B.ternary_gemm(g1["ca"], g1["cw"], 260, 300, 640, want_acc=True)
    assert none_y is None and (acc_only.cpu().numpy() == ref["D"]).all()
    none_acc, y_only = B.ternary_gemm(g1["ca"], g1["cw"], 260, 300, 640, ep=g1["ep"])
    assert none_acc is None
    assert torch.equal(y_only, g1["y"])
    g2 = T.hip_gemm(case)
    assert torch.equal(g1["D"], g2["D"]) and torch.equal(g1["y"], g2["y"])


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (37, 19, 131), (130, 70, 1000), (256, 256, 4096)])
def test_gemm_popc_vs_oracle(M, N, K):
    _say("gemm_popc M=%d N=%d K=%d" % (M, N, K))
    case = wl.gemm_case(M, N, K, p_zero=0.5, seed=M + K)
    ref = T.oracle_gemm(case)
    got = T.hip_gemm(case, fmt=B.RTN_CODE_BITPLANE)
    assert (got["D"].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "popc y")


def test_standalone_epilogue_gemm():
    _say("standalone epilogue (gemm form)")
    case = wl.gemm_case(100, 90, 300, seed=4, table4=True)
    ref = T.oracle_gemm(case, relu=True)
    got = T.hip_gemm(case, relu=True)
    y = B.epilogue_reparam(got["D"], 300, got["ep"])
    torch.cuda.synchronize()
    T.assert_y_close(y.cpu().numpy(), ref["y"], "standalone epilogue")
    assert torch.equal(y, got["y"])


# ------------------------------------------------- S3: implicit-GEMM conv ----
CONV_SHAPES = [
    wl.ConvShape("c3x3s1", 64, 12, 64, 3, 1, 1),
    wl.ConvShape("c3x3s2", 64, 14, 128, 3, 2, 1),
    wl.ConvShape("c1x1s2", 64, 14, 128, 1, 2, 0),
    wl.ConvShape("c1x1s1", 128, 7, 64, 1, 1, 0),
    wl.ConvShape("ragged_c", 5, 9, 7, 3, 1, 1),          # C and O far from tile sizes
    wl.ConvShape("c130", 130, 6, 70, 3, 1, 1),           # C pads to 192
    wl.ConvShape("tiny", 3, 2, 2, 3, 1, 1),              # image smaller than the kernel
    wl.ConvShape("nopad", 64, 9, 32, 3, 1, 0),
    wl.ConvShape("k5", 16, 11, 24, 5, 2, 2),
    wl.ConvShape("wide_o", 64, 7, 320, 3, 1, 1),
]


@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("true_zero", [True, False])
def test_conv_vs_oracle(shape, true_zero):
    _say("conv %s true_zero=%s" % (shape, true_zero))
    case = wl.conv_case(shape, batch=3, seed=len(shape.name), per_channel=True, bn=True)
    ref = T.oracle_conv(case, true_zero, relu=True)
    got = T.hip_conv(case, true_zero, relu=True)
    Cp = (shape.C + 63) // 64 * 64
    assert (got["ca"].cpu().numpy() == orc.nchw_to_nhwc_i8(ref["ta"], Cp)).all()
    assert (got["cw"].cpu().numpy() == orc.nchw_to_nhwc_i8(ref["tw"], Cp)).all()
    assert (got["D"].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "conv y")
    y2 = B.epilogue_reparam_conv2d(got["D"], shape.C, case["H"], case["W"], shape.k, shape.k, shape.stride,
                                   shape.pad, B.RTN_PAD_TRUE_ZERO if true_zero else B.RTN_PAD_CODE_ZERO,
                                   got["ep"])
    torch.cuda.synchronize()
    assert torch.equal(y2, got["y"])


def test_conv_rectangular_image():
    _say("conv rectangular image 10x23")
    shape = wl.ConvShape("rect", 64, 10, 96, 3, 1, 1)
    case = wl.conv_case(shape, batch=2, seed=77, Hx=10, Wx=23)
    ref, got = T.oracle_conv(case), T.hip_conv(case)
    assert (got["D"].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "rect conv")


def test_config1_single_layer():
    """3x3 s1 p1, batch 1, 64->64 @ 56x56, Delta_a = 0.5, per-layer scalars."""
    _say("config 1")
    case = wl.config1_case()
    ref, got = T.oracle_conv(case), T.hip_conv(case)
    assert (got["D"].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "config1")
    # direct float conv of the reparameterized values (zero padding)
    direct = orc.conv_direct(ref["ta"], ref["tw"], 1, 1, case["alpha_a"], case["beta_a"], case["alpha_w"],
                             case["beta_w"], True)
    assert np.abs(got["y"].cpu().numpy() - direct).max() <= 1e-5 * np.abs(direct).max()


def test_conv_beta_w_null_is_eq9():
    _say("conv beta_w = NULL")
    shape = wl.ConvShape("eq9", 64, 8, 64, 3, 1, 1)
    case = dict(wl.conv_case(shape, batch=2, seed=5), beta_w=None)
    ref, got = T.oracle_conv(case, False, relu=True), T.hip_conv(case, False, relu=True)
    T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "eq9")
    # Eq.9 as printed: z = relu(alpha*gamma*D + alpha*beta*sum(t_w)), code-zero padding
    Sw = ref["tw"].reshape(shape.O, -1).sum(1).astype(np.float64)
    aw = np.asarray(case["alpha_w"], np.float64)
    z = np.maximum(0.0, float(case["alpha_a"]) * aw[None, :, None, None] * ref["D"] +
                   (aw * float(case["beta_a"]) * Sw)[None, :, None, None])
    assert np.abs(got["y"].cpu().numpy() - z).max() <= 1e-5 * np.abs(z).max()


# ------------------------------------------ every tile configuration ---------
@pytest.fixture
def tile_reset():
    yield
    B.set_tile_config(-1)


@pytest.mark.parametrize("cfg", range(20))
def test_all_tile_configs_gemm_and_conv(cfg, tile_reset):
    _say("tile config %d" % cfg)
    assert B.num_tile_configs() == 20
    B.set_tile_config(cfg)
    case = wl.gemm_case(300, 530, 320, seed=cfg)          # several tiles + ragged tails in M and N
    ref, got = T.oracle_gemm(case), T.hip_gemm(case)
    assert (got["D"].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "gemm cfg %d" % cfg)
    shape = wl.ConvShape("t", 64, 13, 200, 3, 2, 1)
    ccase = wl.conv_case(shape, batch=7, seed=cfg)         # 7*49 = 343 pixels, O = 200
    cref, cgot = T.oracle_conv(ccase, True, relu=True), T.hip_conv(ccase, True, relu=True)
    assert (cgot["D"].cpu().numpy() == cref["D"]).all()
    T.assert_y_close(cgot["y"].cpu().numpy(), cref["y"], "conv cfg %d" % cfg)


@pytest.mark.parametrize("cfg", range(20))
def test_all_tile_configs_single_output_launches(cfg, tile_reset):
    """Accumulators only and y only, on shapes whose rows can be written 16 bytes
    at a time (N % 4 == 0, OH*OW % 4 == 0) and that have full tiles as well as
    ragged ones: the staged wide-store path of every tile configuration."""
    _say("tile config %d, single-output launches" % cfg)
    B.set_tile_config(cfg)
    case = wl.gemm_case(300, 528, 320, seed=50 + cfg)
    ref, got = T.oracle_gemm(case), T.hip_gemm(case, want_acc="separate")
    assert (got["D"].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "gemm cfg %d" % cfg)
    shape = wl.ConvShape("t", 64, 16, 264, 3, 1, 1)
    ccase = wl.conv_case(shape, batch=3, seed=50 + cfg, bn=True)    # 3*256 pixels, O = 264
    cref = T.oracle_conv(ccase, True, relu=True)
    cgot = T.hip_conv(ccase, True, relu=True, want_acc="separate")
    assert (cgot["D"].cpu().numpy() == cref["D"]).all()
    T.assert_y_close(cgot["y"].cpu().numpy(), cref["y"], "conv cfg %d" % cfg)


HALO_SHAPES = [
    # name, C, H, O, k, stride, pad, batch, W (None = H)
    ("h64", 64, 16, 72, 3, 1, 1, 3, None),          # Cpad 64: tile straddles images
    ("h64r", 50, 9, 64, 3, 1, 1, 5, 11),            # C padded to 64, non-square, ragged pixel tail
    ("h64k5", 64, 12, 40, 5, 1, 2, 2, None),        # 5x5 window, pad 2
    ("h128", 128, 12, 136, 3, 1, 1, 3, None),       # Cpad 128: two K-steps per tap
    ("h128r", 100, 7, 130, 3, 1, 1, 9, 10),         # C padded to 128, ragged in O and pixels
    ("h128k1", 128, 8, 64, 1, 1, 0, 4, None),       # 1x1: the run is the tile itself
]


@pytest.mark.parametrize("cfg", range(14, 20))
@pytest.mark.parametrize("hs", HALO_SHAPES, ids=[h[0] for h in HALO_SHAPES])
def test_halo_variants(cfg, hs, tile_reset):
    """The conv variants that hold the input pixel run of a tile in LDS (stride 1,
    centred window, Cpad 64 or 128), in the combined and in the single-output
    launches; a configuration that does not cover a shape falls back to its
    plain tile, which must give the same result."""
    name, Cc, H, O, k, stride, pad, batch, W = hs
    _say("halo cfg %d shape %s" % (cfg, name))
    B.set_tile_config(cfg)
    shape = wl.ConvShape(name, Cc, H, O, k, stride, pad)
    case = wl.conv_case(shape, batch=batch, seed=300 + cfg, bn=True, Wx=W)
    for tz in (True, False):
        ref = T.oracle_conv(case, tz, relu=True)
        for mode in (True, "separate"):
            got = T.hip_conv(case, tz, relu=True, want_acc=mode)
            assert (got["D"].cpu().numpy() == ref["D"]).all(), (name, tz, mode)
            T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "%s cfg %d" % (name, cfg))


# --------------- the FP4 matrix path (codes stored as E2M1 nibbles) ---------------
FP4 = B.RTN_CODE_FP4


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES + [(200, 136, 129), (70, 300, 4096)])
def test_gemm_fp4_vs_oracle(M, N, K):
    _say("gemm fp4 M=%d N=%d K=%d" % (M, N, K))
    case = wl.gemm_case(M, N, K, p_zero=0.4, seed=M + N + K + 1)
    ref = T.oracle_gemm(case)
    for mode in (True, "separate"):
        got = T.hip_gemm(case, fmt=FP4, want_acc=mode)
        assert (got["ca"].cpu().numpy() == orc.encode_fp4(ref["ta"])).all()
        assert (got["Sa"].cpu().numpy() == ref["Sa"]).all() and (got["Sw"].cpu().numpy() == ref["Sw"]).all()
        assert (got["D"].cpu().numpy() == ref["D"]).all()
        T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "gemm fp4 y")


def test_gemm_fp4_extreme_sums_are_exact():
    """All-ones rows against all-ones and all-minus-ones rows: |D| = K at the largest K the
    sweep uses, the case where fp32 accumulation has the least headroom."""
    _say("gemm fp4, |D| = K = 8192")
    K = 8192
    xa = np.ones((96, K), np.float32)
    xw = np.ones((80, K), np.float32)
    xw[1::2] = -1.0
    xw[5, 17] = 0.0
    case = dict(xa=xa, xw=xw, delta_a=np.float32(0.5), delta_w=np.float32(0.5), alpha_a=np.float32(1.0),
                beta_a=np.float32(0.0), alpha_w=np.float32(1.0), beta_w=np.float32(0.0), M=96, N=80, K=K)
    ref, got = T.oracle_gemm(case), T.hip_gemm(case, fmt=FP4)
    assert int(np.abs(ref["D"]).max()) == K
    assert (got["D"].cpu().numpy() == ref["D"]).all()
    assert (got["y"].cpu().numpy() == ref["D"].astype(np.float32)).all()


@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("true_zero", [True, False])
def test_conv_fp4_vs_oracle(shape, true_zero):
    _say("conv fp4 %s true_zero=%s" % (shape, true_zero))
    case = wl.conv_case(shape, batch=3, seed=len(shape.name) + 9, per_channel=True, bn=True)
    ref = T.oracle_conv(case, true_zero, relu=True)
    got = T.hip_conv(case, true_zero, relu=True, fmt=FP4)
    assert (got["ca"].cpu().numpy() == T.fp4_rows(orc.nchw_to_nhwc_i8(ref["ta"], shape.C))).all()
    assert (got["cw"].cpu().numpy() == T.fp4_rows(orc.nchw_to_nhwc_i8(ref["tw"], shape.C))).all()
    assert (got["D"].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "conv fp4 y")


@pytest.mark.parametrize("cfg", range(20))
def test_all_tile_configs_fp4(cfg, tile_reset):
    _say("tile config %d, fp4" % cfg)
    B.set_tile_config(cfg)
    case = wl.gemm_case(300, 530, 700, seed=cfg + 3)
    ref = T.oracle_gemm(case)
    for mode in (True, "separate"):
        got = T.hip_gemm(case, fmt=FP4, want_acc=mode)
        assert (got["D"].cpu().numpy() == ref["D"]).all()
        T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "gemm fp4 cfg %d" % cfg)
    for shape, batch in [(wl.ConvShape("t", 64, 13, 200, 3, 2, 1), 7), (wl.ConvShape("u", 192, 16, 264, 3, 1, 1), 3)]:
        ccase = wl.conv_case(shape, batch=batch, seed=cfg + 5, bn=True)
        cref = T.oracle_conv(ccase, True, relu=True)
        for mode in (True, "separate"):
            cgot = T.hip_conv(ccase, True, relu=True, want_acc=mode, fmt=FP4)
            assert (cgot["D"].cpu().numpy() == cref["D"]).all()
            T.assert_y_close(cgot["y"].cpu().numpy(), cref["y"], "conv fp4 cfg %d" % cfg)


FP4_HALO_SHAPES = HALO_SHAPES + [
    ("h256", 256, 10, 136, 3, 1, 1, 3, None),      # 128 bytes per pixel: two K-steps per tap
    ("h200r", 200, 7, 130, 3, 1, 1, 9, 10),        # C padded to 256, ragged in O and pixels
]


@pytest.mark.parametrize("cfg", range(14, 20))
@pytest.mark.parametrize("hs", FP4_HALO_SHAPES, ids=[h[0] for h in FP4_HALO_SHAPES])
def test_halo_variants_fp4(cfg, hs, tile_reset):
    """The pixel-run-in-LDS variants on FP4 codes: 64 bytes per pixel are up to 128 channels,
    128 bytes up to 256."""
    name, Cc, H, O, k, stride, pad, batch, W = hs
    _say("halo fp4 cfg %d shape %s" % (cfg, name))
    B.set_tile_config(cfg)
    shape = wl.ConvShape(name, Cc, H, O, k, stride, pad)
    case = wl.conv_case(shape, batch=batch, seed=310 + cfg, bn=True, Wx=W)
    for tz in (True, False):
        ref = T.oracle_conv(case, tz, relu=True)
        got = T.hip_conv(case, tz, relu=True, fmt=FP4)
        assert (got["D"].cpu().numpy() == ref["D"]).all(), (name, tz)
        T.assert_y_close(got["y"].cpu().numpy(), ref["y"], "%s fp4 cfg %d" % (name, cfg))


def test_binding_rejects_code_tensors_of_another_format():
    """The C ABI takes raw pointers; the binding refuses, before any launch, a code tensor whose
    size or dtype does not fit the format the call names (an FP4 tensor is half the bytes of
    an int8 one, so the int8 kernels would read past its end)."""
    _say("binding: code tensor / format mismatch is refused")
    shape = wl.ConvShape("m", 128, 8, 64, 3, 1, 1)
    case = wl.conv_case(shape, batch=2, seed=1)
    x, w = T.dev(case["x"]), T.dev(case["w"])
    ca4, _ = B.ternarize_pack(x, -0.5, 0.5, FP4)
    cw4, _ = B.ternarize_pack(w, -0.05, 0.05, FP4)
    ca8, _ = B.ternarize_pack(x, -0.5, 0.5)
    cw8, _ = B.ternarize_pack(w, -0.05, 0.05)
    for a, wt, fmt in [(ca4, cw4, B.RTN_CODE_I8), (ca8, cw4, B.RTN_CODE_I8), (ca8, cw8, FP4), (ca4, cw8, FP4)]:
        with pytest.raises(ValueError):
            B.ternary_conv2d(a, wt, 2, 128, 8, 8, 64, 3, 3, 1, 1, want_acc=True, fmt=fmt)
    g4, _ = B.ternarize_pack(T.dev(case["x"].reshape(2 * 128, 64)), -0.5, 0.5, FP4)
    with pytest.raises(ValueError):
        B.ternary_gemm(g4, g4, 256, 256, 64, want_acc=True)


@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("kind", ["scalar", "vector"])
def test_conv_ternarize_fp4_vs_oracle(shape, kind):
    """The ternarizing epilogue and its block-tail form on FP4 codes in, FP4 codes out."""
    _say("conv+ternarize fp4 %s thresholds=%s" % (shape, kind))
    true_zero = kind == "scalar"
    relu = kind == "vector"
    case = wl.conv_case(shape, batch=3, seed=41 + len(shape.name), per_channel=True, bn=(kind == "scalar"))
    lo, hi = _thresholds(kind, case, shape.O, 6)
    ref = T.oracle_conv(case, true_zero, relu=relu)
    got = T.codes_as_i8(T.hip_conv_ternarize(case, lo, hi, true_zero, relu=relu, fmt=FP4), FP4, shape.O)
    T.assert_codes_match(got, T.oracle_next_codes(ref, lo, hi), ref["y"], lo, hi, shape.name)
    rng = np.random.default_rng(8)
    res = rng.standard_normal(ref["y"].shape).astype(np.float32)
    codes, y = T.hip_conv_ternarize(case, lo, hi, true_zero, relu=relu, residual=res, relu_out=True, want_y=True,
                                    fmt=FP4)
    s = orc.add_relu(ref["y"], res, True)
    want = orc.nchw_to_nhwc_i8(orc.ternarize_nchw(s, lo, hi), (shape.O + 63) // 64 * 64)
    T.assert_codes_match(T.codes_as_i8(codes, FP4, shape.O), want, s, lo, hi, shape.name + " tail")
    tol = 1e-5 * np.abs(ref["y"]) + 1e-9 * max(1.0, float(np.abs(ref["y"]).max())) + 1e-6 * np.abs(res)
    assert (np.abs(y.cpu().numpy().astype(np.float64) - s) <= tol).all()


@pytest.mark.parametrize("cfg", range(20))
def test_all_tile_configs_conv_ternarize_fp4(cfg, tile_reset):
    _say("tile config %d, ternarizing epilogues, fp4" % cfg)
    B.set_tile_config(cfg)
    for shape, batch in [(wl.ConvShape("t", 64, 13, 200, 3, 2, 1), 7),       # ragged in O and pixels
                         (wl.ConvShape("u", 64, 16, 64, 3, 1, 1), 3),        # O = 64: half a 128-code row
                         (wl.ConvShape("v", 192, 12, 136, 3, 1, 1), 3)]:
        case = wl.conv_case(shape, batch=batch, seed=290 + cfg, bn=True)
        lo, hi = _thresholds("scalar", case, shape.O, cfg)
        ref = T.oracle_conv(case, True, relu=True)
        got = T.codes_as_i8(T.hip_conv_ternarize(case, lo, hi, True, relu=True, fmt=FP4), FP4, shape.O)
        T.assert_codes_match(got, T.oracle_next_codes(ref, lo, hi), ref["y"], lo, hi, "cfg %d %s" % (cfg, shape.name))
        res = np.random.default_rng(cfg).standard_normal(ref["y"].shape).astype(np.float32)
        codes, y = T.hip_conv_ternarize(case, lo, hi, True, relu=True, residual=res, relu_out=True, want_y=True,
                                        fmt=FP4)
        s = orc.add_relu(ref["y"], res, True)
        want = orc.nchw_to_nhwc_i8(orc.ternarize_nchw(s, lo, hi), (shape.O + 63) // 64 * 64)
        T.assert_codes_match(T.codes_as_i8(codes, FP4, shape.O), want, s, lo, hi, "cfg %d %s tail" % (cfg, shape.name))
        T.assert_y_close(y.cpu().numpy(), s, "cfg %d %s tail y" % (cfg, shape.name))


# ---------------------- conv with the ternarizing epilogue (next layer's codes) ----
def _thresholds(kind, case, O, seed):
    """scalar: one Delta for the layer; vector: Eq.3's BN-folded pair per channel."""
    if kind == "scalar":
        return np.float32(-0.4), np.float32(0.6)
    rng = np.random.default_rng(seed)
    k = rng.uniform(0.5, 1.5, O)
    b = rng.normal(0.0, 0.3, O)
    return (-(0.5 + b) / k).astype(np.float32), ((0.5 - b) / k).astype(np.float32)


@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("kind", ["scalar", "vector"])
def test_conv_ternarize_vs_oracle(shape, kind):
    _say("conv+ternarize %s thresholds=%s" % (shape, kind))
    true_zero = kind == "scalar"
    relu = kind == "vector"
    case = wl.conv_case(shape, batch=3, seed=40 + len(shape.name), per_channel=True, bn=(kind == "scalar"))
    lo, hi = _thresholds(kind, case, shape.O, 5)
    ref = T.oracle_conv(case, true_zero, relu=relu)
    want = T.oracle_next_codes(ref, lo, hi)
    got = T.hip_conv_ternarize(case, lo, hi, true_zero, relu=relu).cpu().numpy()
    T.assert_codes_match(got, want, ref["y"], lo, hi, shape.name)
    assert {0, 1} <= set(np.unique(want))          # the case decides something


@pytest.mark.parametrize("cfg", range(20))
def test_all_tile_configs_conv_ternarize(cfg, tile_reset):
    _say("tile config %d, ternarizing epilogue" % cfg)
    B.set_tile_config(cfg)
    for shape, batch in [(wl.ConvShape("t", 64, 13, 200, 3, 2, 1), 7),       # ragged in O and pixels
                         (wl.ConvShape("u", 64, 16, 256, 3, 1, 1), 3)]:      # full tiles only
        case = wl.conv_case(shape, batch=batch, seed=90 + cfg, bn=True)
        lo, hi = _thresholds("vector", case, shape.O, cfg)
        ref = T.oracle_conv(case, True, relu=True)
        want = T.oracle_next_codes(ref, lo, hi)
        got = T.hip_conv_ternarize(case, lo, hi, True, relu=True).cpu().numpy()
        T.assert_codes_match(got, want, ref["y"], lo, hi, "cfg %d %s" % (cfg, shape.name))
        assert {-1, 0, 1} <= set(np.unique(want))


@pytest.mark.parametrize("cfg", range(14, 20))
@pytest.mark.parametrize("hs", HALO_SHAPES, ids=[h[0] for h in HALO_SHAPES])
def test_halo_variants_conv_ternarize(cfg, hs, tile_reset):
    name, Cc, H, O, k, stride, pad, batch, W = hs
    _say("halo cfg %d shape %s, ternarizing epilogue" % (cfg, name))
    B.set_tile_config(cfg)
    shape = wl.ConvShape(name, Cc, H, O, k, stride, pad)
    case = wl.conv_case(shape, batch=batch, seed=400 + cfg, bn=True, Wx=W)
    lo, hi = _thresholds("scalar", case, O, 0)
    ref = T.oracle_conv(case, True, relu=True)
    got = T.hip_conv_ternarize(case, lo, hi, True, relu=True).cpu().numpy()
    T.assert_codes_match(got, T.oracle_next_codes(ref, lo, hi), ref["y"], lo, hi, "%s cfg %d" % (name, cfg))


def test_conv_ternarize_equals_pack_of_conv_output():
    """The fused epilogue against the library's own two-step route (fp32 y, then
    rtn_ternarize_pack): the same codes, and Eq.3's fold -- BN applied and one
    threshold pair of +-0.5, against no BN and per-channel thresholds -- agrees away
    from ties."""
    _say("conv+ternarize vs pack(conv)")
    shape = wl.ConvShape("f", 64, 14, 128, 3, 1, 1)
    case = wl.conv_case(shape, batch=4, seed=61, bn=True)
    case["bn_scale"] = np.abs(case["bn_scale"]) + np.float32(0.25)          # k > 0
    fused = T.hip_conv_ternarize(case, np.float32(-0.5), np.float32(0.5), True, relu=True)
    two = T.hip_conv(case, True, relu=True, want_acc=False)
    packed, _ = B.ternarize_pack(two["y"], -0.5, 0.5, want_sum=False)
    torch.cuda.synchronize()
    assert torch.equal(fused, packed)
    k, b = case["bn_scale"].astype(np.float64), case["bn_shift"].astype(np.float64)
    lo, hi = (-(0.5 + b) / k).astype(np.float32), ((0.5 - b) / k).astype(np.float32)
    nobn = {kk: v for kk, v in case.items() if kk not in ("bn_scale", "bn_shift")}
    folded = T.hip_conv_ternarize(nobn, lo, hi, True, relu=True)
    diff = (folded != fused)
    z = two["y"].permute(0, 2, 3, 1)                        # bn(relu(.)) as stored
    near = (z.abs() - 0.5).abs() < 1e-5
    assert not bool((diff & ~near).any())
    assert int(diff.sum()) < 20


def _block_tail_check(case, shape, true_zero, lo, hi, use_res, relu_out, want_y, what):
    """conv -> (BN) -> + residual -> ReLU -> ternarize, fused, against the oracle's steps."""
    ref = T.oracle_conv(case, true_zero, relu=False)
    rng = np.random.default_rng(len(what))
    res = rng.standard_normal(ref["y"].shape).astype(np.float32) if use_res else None
    s = ref["y"]
    if use_res:
        s = orc.add_relu(s, res, relu_out)
    elif relu_out:
        s = orc.add_relu(s, np.zeros_like(s), True)
    want = orc.nchw_to_nhwc_i8(orc.ternarize_nchw(s, lo, hi), (shape.O + 63) // 64 * 64)
    got = T.hip_conv_ternarize(case, lo, hi, true_zero, relu=False, residual=res, relu_out=relu_out,
                               want_y=want_y)
    codes, y = got if want_y else (got, None)
    T.assert_codes_match(codes.cpu().numpy(), want, s, lo, hi, what)
    if want_y:
        # the stored fp32 value: the oracle's z within the fp32 tolerance, then the same fp32 add
        yh = y.cpu().numpy()
        assert not np.isnan(yh).any(), what + ": unwritten outputs"
        floor = 1e-9 * max(1.0, float(np.abs(ref["y"]).max()))
        tol = 1e-5 * np.abs(ref["y"]) + floor + 1e-6 * (np.abs(res) if use_res else 0.0)
        assert (np.abs(yh.astype(np.float64) - s) <= tol).all(), what


@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("mode", ["res_relu_y", "res_only", "y_only", "relu_only"])
def test_conv_block_tail_vs_oracle(shape, mode):
    _say("conv block tail %s %s" % (shape, mode))
    case = wl.conv_case(shape, batch=3, seed=70 + len(shape.name), per_channel=True, bn=True)
    lo, hi = _thresholds("vector" if mode == "res_only" else "scalar", case, shape.O, 9)
    _block_tail_check(case, shape, mode != "y_only", lo, hi,
                      use_res=mode in ("res_relu_y", "res_only"),
                      relu_out=mode in ("res_relu_y", "relu_only"),
                      want_y=mode in ("res_relu_y", "y_only"), what="%s %s" % (shape.name, mode))


@pytest.mark.parametrize("cfg", range(20))
def test_all_tile_configs_conv_block_tail(cfg, tile_reset):
    _say("tile config %d, block-tail epilogue" % cfg)
    B.set_tile_config(cfg)
    for shape, batch in [(wl.ConvShape("t", 64, 13, 200, 3, 2, 1), 7),       # ragged in O and pixels
                         (wl.ConvShape("u", 64, 16, 256, 3, 1, 1), 3),       # full tiles only
                         (wl.ConvShape("v", 128, 12, 136, 3, 1, 1), 3)]:     # Cpad 128 (halo-eligible)
        case = wl.conv_case(shape, batch=batch, seed=190 + cfg, bn=True)
        lo, hi = _thresholds("scalar", case, shape.O, cfg)
        _block_tail_check(case, shape, True, lo, hi, True, True, True, "cfg %d %s" % (cfg, shape.name))


CONV2_OF_BLOCK = [1, 3, 5, 8, 10, 13, 15, 18]


@pytest.mark.parametrize("idx", CONV2_OF_BLOCK)
def test_resnet18_conv2_layers_batch256_block_tail_sampled_images(idx):
    """The last conv of each ResNet-18 block at batch 256 with the block-tail epilogue
    (residual add, ReLU, fp32 output and the next block's codes), in the launch
    configuration of the benchmark's trunk forward; the oracle recomputes eight images spread over the batch."""
    shape = wl.resnet18_ternary_layers()[idx]
    _say("resnet18 b256 block tail %s" % (shape,))
    case = wl.conv_case(shape, batch=256, seed=600 + idx, per_channel=True, bn=True)
    lo, hi = np.float32(-0.5), np.float32(0.5)
    rng = np.random.default_rng(idx)
    res = rng.standard_normal((256, shape.O, shape.OH, shape.OH)).astype(np.float32)
    codes, y = T.hip_conv_ternarize(case, lo, hi, True, relu=False, residual=res, relu_out=True, want_y=True)
    imgs = _sample_images(256, 8, 600 + idx)
    ref = T.oracle_conv(case, True, relu=False, images=imgs)
    s = orc.add_relu(ref["y"], res[imgs], True)
    want = orc.nchw_to_nhwc_i8(orc.ternarize_nchw(s, lo, hi), (shape.O + 63) // 64 * 64)
    T.assert_codes_match(codes[imgs].cpu().numpy(), want, s, lo, hi, shape.name)
    T.assert_y_close(y[imgs].cpu().numpy(), s, shape.name + " block output")
    assert not bool(torch.isnan(y).any())
    assert float(y.min()) >= 0.0 and int(codes.abs().max()) == 1


CONV1_OF_BLOCK = [0, 2, 4, 7, 9, 12, 14, 17]


@pytest.mark.parametrize("idx", CONV1_OF_BLOCK)
def test_resnet18_conv1_layers_batch256_ternarize_sampled_images(idx):
    """The first conv of each ResNet-18 block at batch 256 (the shapes whose output
    feeds another ternary conv), ternarizing epilogue, launch configuration as the
    benchmark's fused workload; the oracle recomputes eight whole images spread over the batch."""
    shape = wl.resnet18_ternary_layers()[idx]
    _say("resnet18 b256 conv+ternarize %s" % (shape,))
    case = wl.conv_case(shape, batch=256, seed=500 + idx, per_channel=True, bn=True)
    lo, hi = np.float32(-0.5), np.float32(0.5)
    got = T.hip_conv_ternarize(case, lo, hi, True, relu=True)
    imgs = _sample_images(256, 8, 500 + idx)
    ref = T.oracle_conv(case, True, relu=True, images=imgs)
    T.assert_codes_match(got[imgs].cpu().numpy(), T.oracle_next_codes(ref, lo, hi), ref["y"], lo, hi, shape.name)
    # properties at any size: only codes, zero padding channels, a plausible mix
    assert int(got.abs().max()) == 1
    frac = got.float().abs().mean().item()
    assert 0.02 < frac < 0.98


# ----------------------------------------------------- full-size checks ------
def test_config2_gemm_4096_sampled_rows():
    """M = N = K = 4096 in the launch configuration the benchmark times; the
    oracle computes 1024 sampled rows (all columns) plus every code and side sum."""
    _say("config 2: 4096^3, sampled rows")
    case = wl.gemm_case(4096, 4096, 4096, p_zero=0.4, seed=1)
    got = T.hip_gemm(case, want_acc="separate")
    ta = orc.ternarize(case["xa"], -0.5, 0.5)
    tw = orc.ternarize(case["xw"], -0.5, 0.5)
    assert (got["ca"].cpu().numpy() == ta).all() and (got["cw"].cpu().numpy() == tw).all()
    Sa, Sw = orc.row_sums(ta), orc.row_sums(tw)
    assert (got["Sa"].cpu().numpy() == Sa).all() and (got["Sw"].cpu().numpy() == Sw).all()
    rows = _sample_rows(4096, 1024, 0)
    D = orc.gemm_acc_rows(ta, tw, rows)
    assert (got["D"].cpu().numpy()[rows] == D).all()
    y = orc.gemm_epilogue(D, 4096, Sa[rows], Sw, case["alpha_a"][rows], case["beta_a"][rows],
                          case["alpha_w"], case["beta_w"])
    T.assert_y_close(got["y"].cpu().numpy()[rows], y, "config2 y")
    # statistics the i.i.d. P(0) = 0.4 draw fixes: E[D] = 0, Var[D] = 0.36 K
    Dall = got["D"].double()
    assert abs(float(Dall.mean())) < 0.05
    assert abs(float(Dall.var()) / (0.36 * 4096) - 1) < 0.01


@pytest.mark.parametrize("idx", range(19))
def test_resnet18_layers_batch256_sampled_images(idx):
    """Each ternary ResNet-18 layer at batch 256 (the benchmark's shape and launch
    configuration); the oracle recomputes eight whole images spread over the batch."""
    shape = wl.resnet18_ternary_layers()[idx]
    _say("resnet18 b256 %s" % (shape,))
    case = wl.conv_case(shape, batch=256, seed=100 + idx, per_channel=True, bn=True)
    got = T.hip_conv(case, True, relu=True, want_acc="separate")
    imgs = _sample_images(256, 8, 100 + idx)
    ref = T.oracle_conv(case, True, relu=True, images=imgs)
    assert (got["D"][imgs].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"][imgs].cpu().numpy(), ref["y"], shape.name)
    # properties that hold at any size: |D| <= K, D has the parity pattern of an integer sum
    assert int(got["D"].abs().max()) <= shape.K


@pytest.mark.parametrize("idx", range(19))
def test_resnet18_layers_batch256_fp4_sampled_images(idx):
    """The same layers on the FP4 matrix path (the launch configuration the benchmark
    times): all activation codes of the sampled images, accumulators and outputs."""
    shape = wl.resnet18_ternary_layers()[idx]
    _say("resnet18 b256 fp4 %s" % (shape,))
    case = wl.conv_case(shape, batch=256, seed=100 + idx, per_channel=True, bn=True)
    got = T.hip_conv(case, True, relu=True, want_acc="separate", fmt=FP4)
    imgs = _sample_images(256, 8, 100 + idx)
    ref = T.oracle_conv(case, True, relu=True, images=imgs)
    assert (got["ca"][imgs].cpu().numpy() == T.fp4_rows(orc.nchw_to_nhwc_i8(ref["ta"], shape.C))).all()
    assert (got["D"][imgs].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"][imgs].cpu().numpy(), ref["y"], shape.name)
    assert int(got["D"].abs().max()) <= shape.K


def test_config2_gemm_4096_fp4_sampled_rows():
    _say("config 2 on the FP4 path: 4096^3, 1024 sampled rows")
    case = wl.gemm_case(4096, 4096, 4096, p_zero=0.4, seed=1)
    got = T.hip_gemm(case, fmt=FP4, want_acc="separate")
    ta = orc.ternarize(case["xa"], -0.5, 0.5)
    tw = orc.ternarize(case["xw"], -0.5, 0.5)
    assert (got["ca"].cpu().numpy() == orc.encode_fp4(ta)).all() and (got["cw"].cpu().numpy() == orc.encode_fp4(tw)).all()
    Sa, Sw = orc.row_sums(ta), orc.row_sums(tw)
    assert (got["Sa"].cpu().numpy() == Sa).all() and (got["Sw"].cpu().numpy() == Sw).all()
    rows = _sample_rows(4096, 1024, 2)
    D = orc.gemm_acc_rows(ta, tw, rows)
    assert (got["D"].cpu().numpy()[rows] == D).all()
    y = orc.gemm_epilogue(D, 4096, Sa[rows], Sw, case["alpha_a"][rows], case["beta_a"][rows],
                          case["alpha_w"], case["beta_w"])
    T.assert_y_close(got["y"].cpu().numpy()[rows], y, "config2 fp4 y")


# ------------------------------------ config 3: the conv stack at batch 64 ------
@pytest.mark.parametrize("idx", range(19))
def test_resnet18_layers_batch64_sampled_images(idx):
    """The 19 ternary ResNet-18 layer shapes at batch 64, each standalone, per-filter
    thresholds and scales, one activation threshold per tensor; single-output launches
    as the benchmark issues them.  The oracle recomputes six whole images spread over the batch."""
    shape = wl.resnet18_ternary_layers()[idx]
    _say("resnet18 b64 %s" % (shape,))
    case = wl.conv_case(shape, batch=64, seed=400 + idx, per_channel=True)
    got = T.hip_conv(case, True, want_acc="separate")
    imgs = _sample_images(64, 6, 400 + idx)
    ref = T.oracle_conv(case, True, images=imgs)
    assert (got["ca"][imgs].cpu().numpy() == orc.nchw_to_nhwc_i8(ref["ta"], got["ca"].shape[-1])).all()
    assert (got["D"][imgs].cpu().numpy() == ref["D"]).all()
    T.assert_y_close(got["y"][imgs].cpu().numpy(), ref["y"], shape.name)
    assert int(got["D"].abs().max()) <= shape.K


@pytest.mark.parametrize("idx", range(19))
def test_resnet18_layers_table4_parameters(idx):
    """Each ternary ResNet-18 layer with the activation scale gamma, offset beta and
    (mean) weight scale alpha the paper prints for it in Table 4, no weight offset
    (Eq.9 as printed, ReLU included), batch 3, both pad modes."""
    from golden_io import table4_params
    name, gamma, beta, alpha = table4_params()[idx]
    shape = wl.resnet18_ternary_layers()[idx]
    assert shape.name == name
    _say("resnet18 Table 4 parameters %s gamma=%g beta=%g alpha=%g" % (name, gamma, beta, alpha))
    case = wl.conv_case(shape, batch=3, seed=800 + idx, per_channel=False)
    case.update(alpha_a=np.float32(gamma), beta_a=np.float32(beta), alpha_w=np.float32(alpha), beta_w=None)
    for true_zero in (True, False):
        ref = T.oracle_conv(case, true_zero, relu=True)
        got = T.hip_conv(case, true_zero, relu=True)
        assert (got["D"].cpu().numpy() == ref["D"]).all()
        T.assert_y_close(got["y"].cpu().numpy(), ref["y"], name)


# ------------------------------------ config 5: the large GEMM sweep -------------
SWEEP = [(M, NK, p0) for M in (8192, 16384) for NK in (4096, 8192) for p0 in (0.2, 0.5, 0.8)]


def _sweep_check(M, NK, p0, fmt, seed):
    case = wl.gemm_case(M, NK, NK, p_zero=p0, seed=seed)
    got = T.hip_gemm(case, fmt=fmt, want_acc="separate")
    rows = _sample_rows(M, 1024, seed)
    ta = orc.ternarize(case["xa"][rows], -0.5, 0.5)
    tw = orc.ternarize(case["xw"], -0.5, 0.5)
    Sa, Sw = orc.row_sums(ta), orc.row_sums(tw)
    assert (got["Sa"].cpu().numpy()[rows] == Sa).all() and (got["Sw"].cpu().numpy() == Sw).all()
    if fmt == B.RTN_CODE_I8:
        assert (got["ca"][torch.as_tensor(rows)].cpu().numpy() == ta).all()
        assert (got["cw"].cpu().numpy() == tw).all()
    if fmt == B.RTN_CODE_FP4:
        assert (got["ca"][torch.as_tensor(rows)].cpu().numpy() == orc.encode_fp4(ta)).all()
        assert (got["cw"].cpu().numpy() == orc.encode_fp4(tw)).all()
    D = orc.gemm_acc_rows(ta, tw, np.arange(rows.size, dtype=np.int64))
    assert (got["D"].cpu().numpy()[rows] == D).all()
    y = orc.gemm_epilogue(D, NK, Sa, Sw, case["alpha_a"][rows], case["beta_a"][rows],
                          case["alpha_w"], case["beta_w"])
    T.assert_y_close(got["y"].cpu().numpy()[rows], y, "sweep %d %d %.1f" % (M, NK, p0))
    # the draw fixes E[D] = 0 and Var[D] = K (1 - p0)^2
    Dall = got["D"][:: max(1, M // 512)].double()
    assert abs(float(Dall.mean())) < 0.2
    assert abs(float(Dall.var()) / (NK * (1 - p0) ** 2) - 1) < 0.02


@pytest.mark.parametrize("M,NK,p0", SWEEP)
def test_config5_gemm_sweep_mfma(M, NK, p0):
    """Large ternary GEMMs at three sparsities on the matrix-core path: 1024 sampled
    rows (all columns) against the oracle, all side sums, all weight codes."""
    _say("sweep mfma M=%d N=K=%d P(0)=%.1f" % (M, NK, p0))
    _sweep_check(M, NK, p0, B.RTN_CODE_I8, seed=int(1000 * p0) + M // 1024 + NK // 512)


@pytest.mark.parametrize("M,NK,p0", SWEEP)
def test_config5_gemm_sweep_fp4(M, NK, p0):
    """The same sweep, all twelve points, on the FP4 matrix path."""
    _say("sweep fp4 M=%d N=K=%d P(0)=%.1f" % (M, NK, p0))
    _sweep_check(M, NK, p0, B.RTN_CODE_FP4, seed=int(1000 * p0) + M // 1024 + NK // 512 + 1)


@pytest.mark.parametrize("M,NK,p0", SWEEP)
def test_config5_gemm_sweep_popcount(M, NK, p0):
    """The same sweep, all twelve points, on the bit-plane popcount path (Eq.8)."""
    _say("sweep popc M=%d N=K=%d P(0)=%.1f" % (M, NK, p0))
    _sweep_check(M, NK, p0, B.RTN_CODE_BITPLANE, seed=int(1000 * p0) + 7)


# ------------------------------------ config 4: the chained ternary stack --------
def _chain_params(batch, seed):
    """Per-layer weights and parameters of the chained stack (generators only)."""
    P = []
    for i, sh in enumerate(wl.resnet18_ternary_layers()):
        c = wl.conv_case(sh, batch=1, seed=seed + i, per_channel=True, bn=True)
        P.append(dict(sh=sh, w=c["w"], dw=c["delta_w"], aa=c["alpha_a"], ba=c["beta_a"], aw=c["alpha_w"],
                      bw=c["beta_w"], bs=c["bn_scale"], bh=c["bn_shift"]))
    return P


def _chain_topology():
    """(conv1, conv2, downsample or None) layer indices of the 8 residual blocks."""
    blocks = [(0, 1, None), (2, 3, None)]
    for s in range(3):
        b = 4 + 5 * s
        blocks += [(b, b + 1, b + 2), (b + 3, b + 4, None)]
    return blocks


DELTA_CHAIN = np.float32(0.5)     # Eq.1's threshold, the same fixed input on both sides


def test_config4_chained_blocks_small_batch():
    """The ternary part of ResNet-18 chained as residual blocks,
        out = relu(bn2(tconv2(T(bn1(relu(tconv1(T(x))))))) + shortcut(x)),
    shortcut = identity or the ternary 1x1/stride-2 conv of T(x); T ternarizes at
    Delta = 0.5; adds and the last ReLU are plain fp32.  The paper's figure of the
    block is missing, so this topology is this repository's reading: parity of the
    chain is unpinned by the paper, the per-layer results it is made of are not.
    Both sides run the same definition from the same input; codes entering every
    conv must agree exactly, outputs within the fp32 tolerance."""
    _say("config 4: chained blocks, batch 2")
    P = _chain_params(2, 700)
    rng = np.random.default_rng(77)
    x0 = rng.standard_normal((2, 64, 56, 56)).astype(np.float32)

    def oracle_layer(x, p, relu):
        sh = p["sh"]
        ta = orc.ternarize(x, -DELTA_CHAIN, DELTA_CHAIN)
        tw = orc.ternarize(p["w"], -np.asarray(p["dw"]), p["dw"])
        D = orc.conv_acc(ta, tw, sh.stride, sh.pad)
        Sa, Sw, Kv = orc.conv_sums(ta, tw, sh.stride, sh.pad, True)
        y = orc.conv_epilogue(D, Sa, Sw, Kv, p["aa"], p["ba"], p["aw"], p["bw"], relu=relu,
                              bn_scale=p["bs"], bn_shift=p["bh"])
        return ta, y

    def hip_layer(xd, p, relu):
        sh = p["sh"]
        ca, pa = B.ternarize_pack(xd, T.thr_arg(-DELTA_CHAIN), T.thr_arg(DELTA_CHAIN))
        cw, pw = B.ternarize_pack(T.dev(p["w"]), T.thr_arg(-np.asarray(p["dw"])), T.thr_arg(p["dw"]))
        ep = B.Epilogue(T.gran_arg(p["aa"]), T.gran_arg(p["ba"]), T.gran_arg(p["aw"]), T.gran_arg(p["bw"]),
                        pa, pw, relu=relu, bn_scale=T.dev(p["bs"]), bn_shift=T.dev(p["bh"]))
        Nb, Cc, H, W = xd.shape
        _, y = B.ternary_conv2d(ca, cw, Nb, Cc, H, W, sh.O, sh.k, sh.k, sh.stride, sh.pad,
                                B.RTN_PAD_TRUE_ZERO, ep=ep, want_acc=False)
        return ca, y

    xo, xh = x0, T.dev(x0)
    for bi, (i1, i2, ids) in enumerate(_chain_topology()):
        # oracle side
        ta1, y1 = oracle_layer(xo, P[i1], True)
        ta2, y2 = oracle_layer(y1, P[i2], False)
        sc = xo if ids is None else oracle_layer(xo, P[ids], False)[1]
        xo_next = np.maximum(y2 + sc, np.float32(0)).astype(np.float32)
        # HIP side
        ca1, h1 = hip_layer(xh, P[i1], True)
        ca2, h2 = hip_layer(h1, P[i2], False)
        sh_ = xh if ids is None else hip_layer(xh, P[ids], False)[1]
        xh_next = torch.clamp_min(h2 + sh_, 0.0)
        torch.cuda.synchronize()
        Cp1, Cp2 = ca1.shape[-1], ca2.shape[-1]
        assert (ca1.cpu().numpy() == orc.nchw_to_nhwc_i8(ta1, Cp1)).all(), "block %d conv1 codes" % bi
        assert (ca2.cpu().numpy() == orc.nchw_to_nhwc_i8(ta2, Cp2)).all(), "block %d conv2 codes" % bi
        T.assert_y_close(h1.cpu().numpy(), y1, "block %d y1" % bi)
        T.assert_y_close(xh_next.cpu().numpy(), xo_next, "block %d out" % bi)
        xo, xh = xo_next, xh_next
    assert xo.shape == (2, 512, 7, 7)


def test_config4_chained_blocks_ternarizing_epilogue():
    """The chained stack of test_config4_chained_blocks_small_batch with the first conv
    of every block handing its output to the second as codes (ternarizing epilogue),
    and the block input packed once for conv1 and the downsample conv.  The oracle
    runs the two-step definition (fp32 activation, then Eq.1); codes entering every
    conv and the block outputs must agree."""
    _say("config 4: chained blocks with the ternarizing epilogue, batch 2")
    P = _chain_params(2, 700)
    rng = np.random.default_rng(77)
    x0 = rng.standard_normal((2, 64, 56, 56)).astype(np.float32)
    lo, hi = -DELTA_CHAIN, DELTA_CHAIN

    def weights(p):
        cw, pw = B.ternarize_pack(T.dev(p["w"]), T.thr_arg(-np.asarray(p["dw"])), T.thr_arg(p["dw"]))
        ep = B.Epilogue(T.gran_arg(p["aa"]), T.gran_arg(p["ba"]), T.gran_arg(p["aw"]), T.gran_arg(p["bw"]),
                        None, pw, relu=p["relu"], bn_scale=T.dev(p["bs"]), bn_shift=T.dev(p["bh"]))
        return cw, ep

    def oracle_layer(ta, p, relu):
        sh = p["sh"]
        tw = orc.ternarize(p["w"], -np.asarray(p["dw"]), p["dw"])
        D = orc.conv_acc(ta, tw, sh.stride, sh.pad)
        Sa, Sw, Kv = orc.conv_sums(ta, tw, sh.stride, sh.pad, True)
        return orc.conv_epilogue(D, Sa, Sw, Kv, p["aa"], p["ba"], p["aw"], p["bw"], relu=relu,
                                 bn_scale=p["bs"], bn_shift=p["bh"])

    xo, xh = x0, T.dev(x0)
    for bi, (i1, i2, ids) in enumerate(_chain_topology()):
        p1, p2 = dict(P[i1], relu=True), dict(P[i2], relu=False)
        sh1, sh2 = p1["sh"], p2["sh"]
        # oracle: T(x) -> conv1 -> relu -> bn -> T -> conv2 -> bn ; shortcut ; add ; relu
        ta1 = orc.ternarize(xo, lo, hi)
        y1 = oracle_layer(ta1, p1, True)
        ta2 = orc.ternarize_nchw(y1, lo, hi)
        y2 = oracle_layer(ta2, p2, False)
        sc = xo if ids is None else oracle_layer(ta1, P[ids], False)
        xo_next = np.maximum(y2 + sc, np.float32(0)).astype(np.float32)
        # HIP: one pack, conv1 with the ternarizing epilogue, conv2 (and downsample) to fp32
        Nb, Cc, H, W = xh.shape
        ca1, _ = B.ternarize_pack(xh, float(lo), float(hi), want_sum=False)
        cw1, ep1 = weights(p1)
        ca2 = B.ternary_conv2d_ternarize(ca1, cw1, Nb, Cc, H, W, sh1.O, sh1.k, sh1.k, sh1.stride, sh1.pad,
                                         ep1, float(lo), float(hi))
        cw2, ep2 = weights(p2)
        _, h2 = B.ternary_conv2d(ca2, cw2, Nb, sh2.C, sh2.H, sh2.H, sh2.O, sh2.k, sh2.k, sh2.stride, sh2.pad,
                                 ep=ep2)
        if ids is None:
            sh_ = xh
        else:
            pd = dict(P[ids], relu=False)
            cwd, epd = weights(pd)
            s3 = pd["sh"]
            _, sh_ = B.ternary_conv2d(ca1, cwd, Nb, Cc, H, W, s3.O, s3.k, s3.k, s3.stride, s3.pad, ep=epd)
        xh_next = torch.clamp_min(h2 + sh_, 0.0)
        torch.cuda.synchronize()
        assert (ca1.cpu().numpy() == orc.nchw_to_nhwc_i8(ta1, ca1.shape[-1])).all(), "block %d conv1 codes" % bi
        T.assert_codes_match(ca2.cpu().numpy(), orc.nchw_to_nhwc_i8(ta2, ca2.shape[-1]), y1, lo, hi,
                             "block %d conv2 codes" % bi)
        assert (ca2.cpu().numpy() == orc.nchw_to_nhwc_i8(ta2, ca2.shape[-1])).all(), "block %d conv2 codes" % bi
        T.assert_y_close(xh_next.cpu().numpy(), xo_next, "block %d out" % bi)
        xo, xh = xo_next, xh_next
    assert xo.shape == (2, 512, 7, 7)


def test_config4_trunk_forward_fully_fused():
    """The chained stack with every hand-over fused: one pack of the trunk input, then
    per block conv1 with the ternarizing epilogue and conv2 with the block-tail epilogue
    (shortcut add, ReLU, fp32 output for the next shortcut, codes for the next block);
    the downsample conv reads the same codes as conv1.  20 launches for 19 convs.
    The oracle runs the step-by-step definition."""
    _say("config 4: trunk forward, fully fused, batch 2")
    P = _chain_params(2, 700)
    rng = np.random.default_rng(78)
    x0 = rng.standard_normal((2, 64, 56, 56)).astype(np.float32)
    lo, hi = -DELTA_CHAIN, DELTA_CHAIN

    def weights(p, relu):
        cw, pw = B.ternarize_pack(T.dev(p["w"]), T.thr_arg(-np.asarray(p["dw"])), T.thr_arg(p["dw"]))
        ep = B.Epilogue(T.gran_arg(p["aa"]), T.gran_arg(p["ba"]), T.gran_arg(p["aw"]), T.gran_arg(p["bw"]),
                        None, pw, relu=relu, bn_scale=T.dev(p["bs"]), bn_shift=T.dev(p["bh"]))
        return cw, ep

    def oracle_layer(ta, p, relu):
        sh = p["sh"]
        tw = orc.ternarize(p["w"], -np.asarray(p["dw"]), p["dw"])
        D = orc.conv_acc(ta, tw, sh.stride, sh.pad)
        Sa, Sw, Kv = orc.conv_sums(ta, tw, sh.stride, sh.pad, True)
        return orc.conv_epilogue(D, Sa, Sw, Kv, p["aa"], p["ba"], p["aw"], p["bw"], relu=relu,
                                 bn_scale=p["bs"], bn_shift=p["bh"])

    xo = x0
    ta_o = orc.ternarize(xo, lo, hi)
    xh = T.dev(x0)
    ca, _ = B.ternarize_pack(xh, float(lo), float(hi), want_sum=False)
    torch.cuda.synchronize()
    assert (ca.cpu().numpy() == orc.nchw_to_nhwc_i8(ta_o, ca.shape[-1])).all()
    for bi, (i1, i2, ids) in enumerate(_chain_topology()):
        p1, p2 = P[i1], P[i2]
        sh1, sh2 = p1["sh"], p2["sh"]
        # oracle
        y1 = oracle_layer(ta_o, p1, True)
        ta2 = orc.ternarize_nchw(y1, lo, hi)
        y2 = oracle_layer(ta2, p2, False)
        sc = xo if ids is None else oracle_layer(ta_o, P[ids], False)
        xo = orc.add_relu(y2, sc, True)
        ta_o = orc.ternarize_nchw(xo, lo, hi)
        # HIP
        Nb, Cc, H, W = xh.shape
        cw1, ep1 = weights(p1, True)
        ca2 = B.ternary_conv2d_ternarize(ca, cw1, Nb, Cc, H, W, sh1.O, sh1.k, sh1.k, sh1.stride, sh1.pad,
                                         ep1, float(lo), float(hi))
        if ids is None:
            res = xh
        else:
            s3 = P[ids]["sh"]
            cwd, epd = weights(P[ids], False)
            _, res = B.ternary_conv2d(ca, cwd, Nb, Cc, H, W, s3.O, s3.k, s3.k, s3.stride, s3.pad, ep=epd)
        cw2, ep2 = weights(p2, False)
        out = torch.empty((Nb, sh2.O, sh2.OH, sh2.OH), dtype=torch.float32, device=T.DEV)
        ca = B.ternary_conv2d_ternarize(ca2, cw2, Nb, sh2.C, sh2.H, sh2.H, sh2.O, sh2.k, sh2.k, sh2.stride,
                                        sh2.pad, ep2, float(lo), float(hi), residual=res, relu_out=True,
                                        y_out=out)
        torch.cuda.synchronize()
        T.assert_codes_match(ca2.cpu().numpy(), orc.nchw_to_nhwc_i8(ta2, ca2.shape[-1]), y1, lo, hi,
                             "block %d conv2 input codes" % bi)
        T.assert_y_close(out.cpu().numpy(), xo, "block %d output" % bi)
        T.assert_codes_match(ca.cpu().numpy(), orc.nchw_to_nhwc_i8(ta_o, ca.shape[-1]), xo, lo, hi,
                             "block %d output codes" % bi)
        # the chain stays comparable only while the codes agree exactly
        assert (ca.cpu().numpy() == orc.nchw_to_nhwc_i8(ta_o, ca.shape[-1])).all(), "block %d" % bi
        xh = out
    assert xo.shape == (2, 512, 7, 7)


@pytest.mark.parametrize("fmt", [B.RTN_CODE_FP4, B.RTN_CODE_I8], ids=["fp4", "i8"])
def test_config4_full_forward_batch256_sampled_images(fmt):
    """The full-network configuration at its stated size: 256 images of 3x224x224, fp32
    stem and classifier (torch, outside the ternary library), the 8 residual blocks of 19
    ternary convs through the C ABI with every hand-over fused (1 pack + 19 convs).  Images
    are independent, so the oracle runs the step-by-step chain on six images spread over
    the batch, starting from the trunk input the stem produced, and every block's input
    codes, hand-over codes and fp32 output are compared.  The block topology is this
    repository's reading (the paper's figure is not in its text): chain parity is
    unpinned by the paper, the per-layer arithmetic it is made of is pinned."""
    from paper_1912_02057_amd.resnet18 import TernaryResNet18
    _say("config 4: full forward, batch 256, six sampled images, code format %d" % fmt)
    prm = wl.resnet18_network_params(seed=4)
    rng = np.random.Generator(np.random.PCG64(44))
    images = rng.standard_normal((256, 3, 224, 224), dtype=np.float32)
    net = TernaryResNet18(prm, 256, T.DEV, fmt)
    x0 = net.stem(T.dev(images))
    assert tuple(x0.shape) == (256, 64, 56, 56)
    keep = []
    out = net.trunk(x0, keep)
    logits = net.head(out)
    torch.cuda.synchronize()
    assert tuple(out.shape) == (256, 512, 7, 7) and tuple(logits.shape) == (256, 1000)
    assert bool(torch.isfinite(logits).all())
    imgs = _sample_images(256, 6, 4)
    lo, hi = -prm["delta_a"], prm["delta_a"]

    def oracle_layer(ta, p, relu):
        sh = p["sh"]
        tw = orc.ternarize(p["w"], -np.asarray(p["dw"]), p["dw"])
        D = orc.conv_acc(ta, tw, sh.stride, sh.pad)
        Sa, Sw, Kv = orc.conv_sums(ta, tw, sh.stride, sh.pad, True)
        return orc.conv_epilogue(D, Sa, Sw, Kv, p["aa"], p["ba"], p["aw"], p["bw"], relu=relu,
                                 bn_scale=p["bs"], bn_shift=p["bh"])

    P = prm["layers"]
    xo = x0[imgs].cpu().numpy()
    ta_o = orc.ternarize(xo, lo, hi)
    for bi, (i1, i2, ids) in enumerate(wl.resnet18_block_topology()):
        sh1, sh2 = P[i1]["sh"], P[i2]["sh"]
        c1 = T.codes_as_i8(keep[bi][0][imgs], fmt, sh1.C)
        c2 = T.codes_as_i8(keep[bi][1][imgs], fmt, sh2.C)
        yb = keep[bi][2][imgs].cpu().numpy()
        assert (c1 == orc.nchw_to_nhwc_i8(ta_o, c1.shape[-1])).all(), "block %d input codes" % bi
        y1 = oracle_layer(ta_o, P[i1], True)
        ta2 = orc.ternarize_nchw(y1, lo, hi)
        T.assert_codes_match(c2, orc.nchw_to_nhwc_i8(ta2, c2.shape[-1]), y1, lo, hi, "block %d hand-over codes" % bi)
        assert (c2 == orc.nchw_to_nhwc_i8(ta2, c2.shape[-1])).all(), "block %d hand-over codes" % bi
        y2 = oracle_layer(ta2, P[i2], False)
        sc = xo if ids is None else oracle_layer(ta_o, P[ids], False)
        xo = orc.add_relu(y2, sc, True)
        T.assert_y_close(yb, xo, "block %d output" % bi)
        ta_o = orc.ternarize_nchw(xo, lo, hi)
    last = T.codes_as_i8(net.last_codes[imgs], fmt, 512)
    T.assert_codes_match(last, orc.nchw_to_nhwc_i8(ta_o, 512), xo, lo, hi, "trunk output codes")
    # the fp32 head on the oracle's trunk output (plain numpy): average pool + FC
    want = xo.astype(np.float64).mean(axis=(2, 3)) @ prm["fc_w"].astype(np.float64).T + prm["fc_b"]
    got = logits[imgs].cpu().numpy()
    assert np.abs(got - want).max() <= 1e-4 * max(1.0, np.abs(want).max())


# ------------------------- weight-only ternary GEMM (fp32 activations) ----------
def _wgemm_check(M, N, K, seed, vector_alpha=True, relu=False, bn=False, rows=None, what=""):
    """HIP weight-only GEMM against the oracle.  The kernel sums 3K exact bf16 products
    in fp32 (order fixed by the matrix core), the oracle in double: the difference is
    fp32 accumulation error, bounded by 3K * 2^-24 * alpha * sum|x| in the worst case.
    Asserted here: the random-walk size of it, (4 sqrt(3K) + 8) * 2^-24 * alpha * sum|x|,
    plus one fp32 rounding of y."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[0, 0] = 0.0
    if M > 1 and K > 1:
        x[1, 1] = np.float32(1e-20)           # tiny and huge magnitudes in one row
        x[1, 0] = np.float32(3e4)
    w = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    dw = wl.twn_threshold(w, axis=0)
    aw = rng.uniform(0.5, 1.5, N).astype(np.float32) if vector_alpha else np.float32(0.8)
    bs = rng.uniform(0.5, 1.5, N).astype(np.float32) if bn else None
    bh = rng.normal(0, 0.1, N).astype(np.float32) if bn else None
    tw = orc.ternarize(w, -dw, dw)
    cw, _ = B.ternarize_pack(T.dev(w), T.thr_arg(-dw), T.thr_arg(dw), want_sum=False)
    y = B.ternary_weight_gemm(T.dev(x), cw, M, N, K, T.thr_arg(aw), relu=relu,
                              bn_scale=None if bs is None else T.dev(bs),
                              bn_shift=None if bh is None else T.dev(bh))
    # the same call with the weight side prepared ahead of time: same kernels, same bits
    y2 = B.ternary_weight_gemm(T.dev(x), None, M, N, K, T.thr_arg(aw), relu=relu,
                               bn_scale=None if bs is None else T.dev(bs),
                               bn_shift=None if bh is None else T.dev(bh), prepared=B.weight_gemm_prepare(cw, N, K))
    torch.cuda.synchronize()
    assert torch.equal(y, y2), "prepared weight-only GEMM differs from the one-call form"
    y = y.cpu().numpy()
    sel = np.arange(M) if rows is None else rows
    ref = orc.wgemm(x[sel], tw, aw, relu=relu, bn_scale=bs, bn_shift=bh).astype(np.float64)
    scale = np.abs(x[sel].astype(np.float64)).sum(1)[:, None] * np.abs(np.asarray(aw, np.float64))[None, ...]
    if bn:
        scale = scale * np.abs(bs.astype(np.float64))[None, :]
    tol = (4.0 * np.sqrt(3.0 * K) + 8.0) * 2.0 ** -24 * scale + 1.2e-7 * np.abs(ref) + 1e-30
    err = np.abs(y[sel].astype(np.float64) - ref)
    _report_rel(err, ref, scale, tol, what)
    assert (err <= tol).all(), "%s: worst err/tol %.3g" % (what, float((err / tol).max()))
    return float((err / tol).max())


def _report_rel(err, ref, scale, tol, what):
    """Prints what the weight-only path achieved next to its bound: the largest error
    relative to the output over the outputs that are not cancelled (|y| above 1 % of
    alpha * sum|x|), relative to alpha * sum|x| over all outputs, and the worst
    err / bound."""
    big = np.abs(ref) > 1e-2 * np.broadcast_to(scale, ref.shape)
    rel_y = float((err[big] / np.abs(ref[big])).max()) if big.any() else 0.0
    rel_s = float((err / np.maximum(np.broadcast_to(scale, ref.shape), 1e-300)).max())
    print("[weight-only] %s: max |err|/|y| %.3g (uncancelled outputs), max |err|/(alpha*sum|x|) %.3g, "
          "worst err/bound %.3g" % (what, rel_y, rel_s, float((err / tol).max())), flush=True)
    # the bar of the main path, where it is attainable: 1e-5 relative on every output that is not a
    # near-cancellation (measured: at most 4e-6, and at most 0.08 of the accumulation bound)
    assert rel_y <= 1e-5, "%s: relative error %.3g on an uncancelled output" % (what, rel_y)


WGEMM_SHAPES = [(1, 1, 1), (37, 19, 131), (64, 64, 64), (65, 33, 64), (300, 200, 576), (129, 257, 1000),
                (512, 384, 2304)]


@pytest.mark.parametrize("M,N,K", WGEMM_SHAPES)
def test_weight_gemm_vs_oracle(M, N, K):
    _say("weight-only gemm %dx%dx%d" % (M, N, K))
    _wgemm_check(M, N, K, seed=M + N + K, vector_alpha=True, what="wgemm")
    _wgemm_check(M, N, K, seed=M + N + K + 1, vector_alpha=False, relu=True, bn=True, what="wgemm relu bn")


@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_weight_gemm_tile_configs(cfg, tile_reset):
    _say("weight-only gemm, tile config %d" % cfg)
    B.set_tile_config(cfg)
    _wgemm_check(300, 530, 320, seed=cfg, what="wgemm cfg %d" % cfg)


def test_weight_gemm_exact_on_ternary_activations():
    """Activations that are themselves -1/0/+1 (exact in bf16, zero middle and low terms):
    the result must equal the integer contraction exactly."""
    _say("weight-only gemm on ternary activations")
    case = wl.gemm_case(200, 136, 448, seed=9)
    ref = T.oracle_gemm(case)
    cw, _ = B.ternarize_pack(T.dev(case["xw"]), -0.5, 0.5, want_sum=False)
    y = B.ternary_weight_gemm(T.dev(case["xa"]), cw, 200, 136, 448, 1.0)
    torch.cuda.synchronize()
    assert (y.cpu().numpy() == ref["D"].astype(np.float32)).all()


def test_weight_gemm_4096_sampled_rows():
    _say("weight-only gemm 4096^3, sampled rows")
    rows = np.sort(np.random.default_rng(1).choice(4096, 24, replace=False))
    rows[0], rows[-1] = 0, 4095
    worst = _wgemm_check(4096, 4096, 4096, seed=5, rows=rows, what="wgemm 4096")
    assert worst < 1.0


def _wconv_check(shape, batch, seed, relu=False, bn=False, Wx=None, images=None, what=""):
    """conv form of the weight-only layer against the oracle; tolerance as for the GEMM
    form, with the sum of |x| taken over each output's window (a conv of |x| with ones)."""
    rng = np.random.default_rng(seed)
    H, W = shape.H, (shape.H if Wx is None else Wx)
    x = rng.standard_normal((batch, shape.C, H, W)).astype(np.float32)
    w = (rng.standard_normal((shape.O, shape.C, shape.k, shape.k)) * 0.05).astype(np.float32)
    dw = wl.twn_threshold(w, axis=0)
    aw = rng.uniform(0.5, 1.5, shape.O).astype(np.float32)
    bs = rng.uniform(0.5, 1.5, shape.O).astype(np.float32) if bn else None
    bh = rng.normal(0, 0.1, shape.O).astype(np.float32) if bn else None
    tw = orc.ternarize(w, -dw, dw)
    cw, _ = B.ternarize_pack(T.dev(w), T.thr_arg(-dw), T.thr_arg(dw), want_sum=False)
    y = B.ternary_weight_conv2d(T.dev(x), cw, shape.O, shape.k, shape.k, shape.stride, shape.pad, T.dev(aw),
                                relu=relu, bn_scale=None if bs is None else T.dev(bs),
                                bn_shift=None if bh is None else T.dev(bh))
    prep = B.weight_conv2d_prepare(cw, shape.C, shape.O, shape.k, shape.k, shape.pad, T.dev(aw),
                                   bn_scale=None if bs is None else T.dev(bs),
                                   bn_shift=None if bh is None else T.dev(bh))
    y2 = B.ternary_weight_conv2d(T.dev(x), None, shape.O, shape.k, shape.k, shape.stride, shape.pad, relu=relu,
                                 prepared=prep)
    torch.cuda.synchronize()
    assert torch.equal(y, y2), "prepared weight-only conv differs from the one-call form"
    y = y.cpu().numpy()
    sel = list(range(batch)) if images is None else images
    ref = orc.wconv(x[sel], tw, shape.stride, shape.pad, aw, relu=relu, bn_scale=bs, bn_shift=bh).astype(np.float64)
    absum = torch.nn.functional.conv2d(torch.from_numpy(np.abs(x[sel]).astype(np.float64)),
                                       torch.ones(1, shape.C, shape.k, shape.k, dtype=torch.float64),
                                       stride=shape.stride, padding=shape.pad).numpy()       # [n,1,OH,OW]
    scale = absum * np.abs(aw.astype(np.float64))[None, :, None, None]
    if bn:
        scale = scale * np.abs(bs.astype(np.float64))[None, :, None, None]
    K = shape.C * shape.k * shape.k
    tol = (4.0 * np.sqrt(3.0 * K) + 8.0) * 2.0 ** -24 * scale + 1.2e-7 * np.abs(ref) + 1e-30
    err = np.abs(y[sel].astype(np.float64) - ref)
    assert y.shape[1:] == ref.shape[1:]
    _report_rel(err, ref, scale, tol, what)
    assert (err <= tol).all(), "%s: worst err/tol %.3g" % (what, float((err / tol).max()))


@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: s.name)
def test_weight_conv_vs_oracle(shape):
    _say("weight-only conv %s" % (shape,))
    _wconv_check(shape, 3, seed=len(shape.name), what=shape.name)
    _wconv_check(shape, 2, seed=len(shape.name) + 50, relu=True, bn=True, what=shape.name + " relu bn")


@pytest.mark.parametrize("cfg", [0, 1, 7, 13])
def test_weight_conv_tile_configs(cfg, tile_reset):
    _say("weight-only conv, tile config %d" % cfg)
    B.set_tile_config(cfg)
    _wconv_check(wl.ConvShape("t", 64, 13, 200, 3, 2, 1), 7, seed=cfg, what="wconv cfg %d" % cfg)
    _wconv_check(wl.ConvShape("u", 128, 12, 136, 3, 1, 1), 3, seed=cfg + 9, Wx=10, what="wconv cfg %d rect" % cfg)


def test_weight_conv_exact_on_ternary_activations():
    _say("weight-only conv on ternary activations")
    shape = wl.ConvShape("e", 64, 10, 96, 3, 1, 1)
    rng = np.random.default_rng(3)
    ta = rng.integers(-1, 2, size=(2, 64, 10, 10)).astype(np.int8)
    w = (rng.standard_normal((96, 64, 3, 3)) * 0.05).astype(np.float32)
    dw = wl.twn_threshold(w, axis=0)
    tw = orc.ternarize(w, -dw, dw)
    cw, _ = B.ternarize_pack(T.dev(w), T.thr_arg(-dw), T.thr_arg(dw), want_sum=False)
    y = B.ternary_weight_conv2d(T.dev(ta.astype(np.float32)), cw, 96, 3, 3, 1, 1, 1.0)
    torch.cuda.synchronize()
    assert (y.cpu().numpy() == orc.conv_acc(ta, tw, 1, 1).astype(np.float32)).all()


@pytest.mark.parametrize("idx", [0, 4, 6, 10, 15])
def test_weight_conv_resnet18_layers_batch64_sampled_images(idx):
    shape = wl.resnet18_ternary_layers()[idx]
    _say("weight-only conv, resnet18 b64 %s" % (shape,))
    _wconv_check(shape, 64, seed=800 + idx, relu=True, bn=True, images=[0, 63], what=shape.name)


# ------------------ backward of the reparameterized ternary activation ---------
def _act_bwd_check(n, seed, offset=0, want_da=True):
    rng = np.random.default_rng(seed)
    a = (rng.standard_normal(n + offset) * 0.8).astype(np.float32)
    g = rng.standard_normal(n + offset).astype(np.float32)
    if n >= 8:
        a[offset:offset + 6] = [1.0, -1.0, 0.5, -0.5, np.nan, 2.0]     # inclusive clip, threshold ties, NaN
    lo, hi, gamma = np.float32(-0.5), np.float32(0.5), np.float32(1.37)
    ad, gd = T.dev(a)[offset:], T.dev(g)[offset:]                       # offset != 0: unaligned views
    out = torch.full((n + offset,), 7.0, dtype=torch.float32, device=T.DEV)[offset:] if want_da else None
    da, sums = B.activation_backward(ad, gd, float(lo), float(hi), float(gamma), want_grad_in=want_da, grad_in=out)
    torch.cuda.synchronize()
    rda, rg, rb = orc.act_backward(a[offset:], g[offset:], lo, hi, gamma, want_da)
    s = sums.cpu().numpy()
    scale = float(np.abs(g[offset:]).astype(np.float64).sum()) + 1e-30
    assert abs(s[0] - rg) <= 1e-12 * scale and abs(s[1] - rb) <= 1e-12 * scale, (s, rg, rb)
    if want_da:
        assert (da.cpu().numpy() == rda).all()                          # bit-exact


@pytest.mark.parametrize("n", [1, 5, 255, 4095, 16384, 16385, 100003, 1 << 20])
def test_activation_backward_vs_oracle(n):
    _say("activation backward n=%d" % n)
    _act_bwd_check(n, seed=n)
    _act_bwd_check(n, seed=n + 1, offset=1)           # 4-byte-aligned pointers: the scalar path
    _act_bwd_check(n, seed=n + 2, want_da=False)


def test_activation_backward_layer1_tensor_and_reproducible():
    """The largest activation tensor of the ResNet-18 stack at batch 256 (51.4 M elements);
    the sums must also be identical run to run."""
    _say("activation backward, 256x64x56x56")
    n = 256 * 64 * 56 * 56
    rng = np.random.default_rng(5)
    a = rng.standard_normal(n, dtype=np.float32)
    g = rng.standard_normal(n, dtype=np.float32)
    ad, gd = T.dev(a), T.dev(g)
    da, s1 = B.activation_backward(ad, gd, -0.5, 0.5, 0.9)
    _, s2 = B.activation_backward(ad, gd, -0.5, 0.5, 0.9, want_grad_in=False)
    torch.cuda.synchronize()
    rda, rg, rb = orc.act_backward(a, g, -0.5, 0.5, 0.9)
    assert torch.equal(s1, s2)
    s = s1.cpu().numpy()
    scale = float(np.abs(g).astype(np.float64).sum())
    assert abs(s[0] - rg) <= 1e-12 * scale and abs(s[1] - rb) <= 1e-12 * scale
    assert (da.cpu().numpy() == rda).all()


# ------------------ backward of the reparameterized ternary weights -------------
def _weight_bwd_check(O, K, seed, want_dw=True):
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((O, K)) * 0.6).astype(np.float32)
    g = rng.standard_normal((O, K)).astype(np.float32)
    kw = (0.7 + rng.random(O)).astype(np.float32)
    bw = (rng.standard_normal(O) * 0.1).astype(np.float32)
    al = (0.2 + rng.random(O)).astype(np.float32)
    if K >= 8:                                         # inclusive clip, threshold ties, NaN: k = 1, b = 0 in filter 0
        kw[0], bw[0] = 1.0, 0.0
        w[0, :6] = [1.0, -1.0, 0.5, -0.5, np.nan, 2.0]
    out = torch.full((O, K), 7.0, dtype=torch.float32, device=T.DEV) if want_dw else None
    dw, sums = B.weight_backward(T.dev(w), T.dev(g), -0.5, 0.5, T.dev(kw), T.dev(bw), T.dev(al),
                                 want_grad_w=want_dw, grad_w=out)
    torch.cuda.synchronize()
    rdw, rs = orc.weight_backward(w, g, -0.5, 0.5, kw, bw, al, want_dw)
    s = sums.cpu().numpy()
    ok = ~np.isnan(w)
    gabs = np.where(ok, np.abs(g), 0).astype(np.float64)
    scale_a = gabs.sum(axis=1) + 1e-30
    scale_b = al.astype(np.float64) * scale_a
    scale_k = (np.where(ok, np.abs(w), 0) * gabs).sum(axis=1) * al + 1e-30
    for col, scale in ((0, scale_a), (1, scale_k), (2, scale_b)):
        assert (np.abs(s[:, col] - rs[:, col]) <= 1e-12 * scale).all(), (col, O, K)
    if want_dw:
        assert (dw.cpu().numpy() == rdw).all()                          # bit-exact
    return sums


@pytest.mark.parametrize("O,K", [(1, 1), (3, 7), (2, 255), (5, 257), (64, 576), (130, 1153), (512, 4608),
                                 (3, 70001)])
def test_weight_backward_vs_oracle(O, K):
    _say("weight backward O=%d K=%d" % (O, K))
    s1 = _weight_bwd_check(O, K, seed=O * 7 + K)
    s2 = _weight_bwd_check(O, K, seed=O * 7 + K, want_dw=False)
    assert torch.equal(s1, s2)                                          # reproducible, with or without dW


def test_weight_backward_all_resnet18_ternary_filters():
    for i, shape in enumerate(wl.resnet18_ternary_layers()):
        _say("weight backward %s" % (shape,))
        _weight_bwd_check(shape.O, shape.C * shape.k * shape.k, seed=900 + i)



# ------------------- the comparison system: quaternary (2-bit) codes and dot product -------
QT = (np.float32(1 / 6), np.float32(0.5), np.float32(5 / 6))


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (37, 19, 131), (64, 64, 64), (65, 33, 200), (300, 200, 576),
                                   (129, 257, 1000), (1024, 1024, 4096)])
def test_quaternary_pack_and_gemm_vs_oracle(M, N, K):
    """Quantize + pack in the three storage forms and the dot product on the three paths
    (bit-serial AND/popcount on planes, int8 matrix cores, FP4 matrix cores): codes and
    accumulators bit-exact against the oracle's plain sum of products."""
    _say("quaternary M=%d N=%d K=%d" % (M, N, K))
    rng = np.random.default_rng(M + N + K)
    xa = rng.uniform(-0.2, 1.2, (M, K)).astype(np.float32)
    xw = rng.uniform(-0.2, 1.2, (N, K)).astype(np.float32)
    xa.flat[:: max(1, xa.size // 11)] = QT[1]              # exact ties stay below the threshold
    if xa.size > 1:
        xa.flat[1] = np.nan
    qa, qw = orc.quantize4(xa, *QT), orc.quantize4(xw, *QT)
    D = orc.qgemm_acc(qa, qw)
    xad, xwd = T.dev(xa), T.dev(xw)
    for fmt in (B.RTN_CODE_I8, B.RTN_CODE_FP4, B.RTN_CODE_BITPLANE):
        ca, cw = B.quaternary_pack(xad, *QT, fmt), B.quaternary_pack(xwd, *QT, fmt)
        if fmt == B.RTN_CODE_I8:
            assert (ca.cpu().numpy() == orc.pad_rows_i8(qa, ca.shape[1])).all()
        elif fmt == B.RTN_CODE_FP4:
            assert (ca.cpu().numpy() == orc.encode_fp4(qa)).all()
        else:
            hi, lo = T.planes_from_dev(ca)
            eh, el = orc.encode_qplanes(qa, ca.shape[-1])
            assert (hi == eh).all() and (lo == el).all()
        got = B.quaternary_gemm(ca, cw, M, N, K, fmt)
        torch.cuda.synchronize()
        assert (got.cpu().numpy() == D).all(), "format %d" % fmt


def test_quaternary_extreme_sum_is_exact_on_the_fp4_path():
    _say("quaternary all threes, K = 65536")
    K = 65536
    x = np.ones((64, K), np.float32)
    c = B.quaternary_pack(T.dev(x), *QT, B.RTN_CODE_FP4)
    got = B.quaternary_gemm(c, c, 64, 64, K, B.RTN_CODE_FP4)
    torch.cuda.synchronize()
    assert (got.cpu().numpy() == 9 * K).all()


@pytest.mark.parametrize("fmt", [B.RTN_CODE_FP4, B.RTN_CODE_I8], ids=["fp4", "i8"])
def test_gemm_extreme_sums_at_the_maximum_k(fmt):
    """K = 2^22, the largest the library accepts: accumulators of +-K, the largest magnitude there
    is (on the FP4 path an fp32 sum of integers that must stay exact), and of 0 from full
    cancellation.  Expected values are closed forms; the four-term output is compared with the
    oracle's epilogue on those accumulators."""
    _say("gemm at K = 2^22, fmt %d" % fmt)
    K, M, N = 1 << 22, 64, 64
    xa = torch.ones((M, K), dtype=torch.float32, device=T.DEV)
    xa[1].fill_(-1.0)
    xa[2, ::2] = -1.0                                    # alternating: sums to 0 against ones
    xw = torch.ones((N, K), dtype=torch.float32, device=T.DEV)
    xw[3].fill_(-1.0)
    xw[5, 1::2] = 0.0                                    # every other weight zero
    ca, sa = B.ternarize_pack(xa, -0.5, 0.5, fmt)
    cw, sw = B.ternarize_pack(xw, -0.5, 0.5, fmt)
    ra = np.full(M, K, np.int64); ra[1] = -K; ra[2] = 0                 # row sums of t_a
    rw = np.full(N, K, np.int64); rw[3] = -K; rw[5] = K // 2            # row sums of t_w
    assert (sa.cpu().numpy() == ra).all() and (sw.cpu().numpy() == rw).all()
    D = np.empty((M, N), np.int64)
    for m in range(M):
        for n in range(N):
            if m == 2:
                # alternating signs cancel, except against the filter that keeps only the even taps
                D[m, n] = -(K // 2) if n == 5 else 0
            else:
                base = K if n != 5 else K // 2
                D[m, n] = base * (-1 if m == 1 else 1) * (-1 if n == 3 else 1)
    aa, ba, aw, bw = np.float32(0.75), np.float32(-0.1), np.float32(1.25), np.float32(0.05)
    ep = B.Epilogue(float(aa), float(ba), float(aw), float(bw), sa, sw)
    acc = torch.empty((M, N), dtype=torch.int32, device=T.DEV)
    y = torch.empty((M, N), dtype=torch.float32, device=T.DEV)
    B.ternary_gemm(ca, cw, M, N, K, fmt=fmt, ep=ep, acc_out=acc, y_out=y)
    torch.cuda.synchronize()
    assert (acc.cpu().numpy() == D).all()
    ref = orc.gemm_epilogue(D.astype(np.int32), K, ra.astype(np.int32), rw.astype(np.int32), aa, ba, aw, bw)
    T.assert_y_close(y.cpu().numpy(), ref, "y at K = 2^22")


# ------------------- other networks' layer shapes (MobileNet, AlexNet, NIN) -------------------
def _dw_check(C, H, k, stride, pad, batch, seed, true_zero=True, W=None):
    rng = np.random.default_rng(seed)
    W = H if W is None else W
    x = rng.standard_normal((batch, C, H, W)).astype(np.float32)
    w = (rng.standard_normal((C, k * k)) * 0.3).astype(np.float32)
    dw = wl.twn_threshold(w, axis=0)
    da = wl.twn_threshold(x)
    aw = rng.uniform(0.5, 1.5, C).astype(np.float32)
    bw = rng.uniform(-0.2, 0.2, C).astype(np.float32)
    bs = rng.uniform(0.5, 1.5, C).astype(np.float32)
    bh = rng.normal(0, 0.1, C).astype(np.float32)
    aa, ba = np.float32(1.2), np.float32(0.15)
    ta = orc.ternarize(x, -da, da)
    tw = orc.ternarize(w, -dw, dw)
    D, y = orc.dwconv(ta, tw.reshape(C, k, k), stride, pad, aa, ba, aw, bw, true_zero, relu=True, bn_scale=bs, bn_shift=bh)
    ca, _ = B.ternarize_pack(T.dev(x), float(-da), float(da), want_sum=False)
    cw, _ = B.ternarize_pack(T.dev(w), T.dev(-dw), T.dev(dw), want_sum=False)      # rows: one filter per row
    ep = B.Epilogue(float(aa), float(ba), T.dev(aw), T.dev(bw), None, None, relu=True, bn_scale=T.dev(bs), bn_shift=T.dev(bh))
    pm = B.RTN_PAD_TRUE_ZERO if true_zero else B.RTN_PAD_CODE_ZERO
    acc = torch.full(D.shape, -7777, dtype=torch.int32, device=T.DEV)
    yy = torch.full(D.shape, float("nan"), dtype=torch.float32, device=T.DEV)
    B.ternary_depthwise_conv2d(ca, cw, batch, C, H, W, k, k, stride, pad, pm, ep=ep, acc_out=acc, y_out=yy)
    torch.cuda.synchronize()
    assert (acc.cpu().numpy() == D).all()
    T.assert_y_close(yy.cpu().numpy(), y, "depthwise y")
    # one output at a time (the kernel then keeps one tile instead of two): same bits
    acc2 = torch.full(D.shape, -7777, dtype=torch.int32, device=T.DEV)
    y2 = torch.full(D.shape, float("nan"), dtype=torch.float32, device=T.DEV)
    B.ternary_depthwise_conv2d(ca, cw, batch, C, H, W, k, k, stride, pad, pm, acc_out=acc2)
    B.ternary_depthwise_conv2d(ca, cw, batch, C, H, W, k, k, stride, pad, pm, ep=ep, y_out=y2)
    torch.cuda.synchronize()
    assert torch.equal(acc, acc2) and torch.equal(yy, y2)


@pytest.mark.parametrize("C,H,k,stride,pad,batch", [(5, 9, 3, 1, 1, 2), (64, 12, 3, 1, 1, 3), (66, 11, 3, 2, 1, 3),
                                                     (130, 7, 3, 1, 1, 5), (32, 10, 5, 1, 2, 2), (16, 6, 1, 1, 0, 4),
                                                     (3, 2, 3, 1, 1, 1)])
def test_depthwise_conv_vs_oracle(C, H, k, stride, pad, batch):
    _say("depthwise conv C=%d H=%d k=%d s=%d p=%d" % (C, H, k, stride, pad))
    _dw_check(C, H, k, stride, pad, batch, seed=C + H, true_zero=True)
    _dw_check(C, H, k, stride, pad, batch, seed=C + H + 1, true_zero=False, W=H + 3)


@pytest.mark.parametrize("C,H,stride", [(32, 112, 1), (64, 112, 2), (128, 56, 1), (256, 28, 2), (512, 14, 1), (1024, 7, 1)])
def test_mobilenet_depthwise_layers(C, H, stride):
    """MobileNet's 3x3 depthwise layer shapes (batch 4 here)."""
    _say("mobilenet depthwise %d@%d s%d" % (C, H, stride))
    _dw_check(C, H, 3, stride, 1, 4, seed=C)


@pytest.mark.parametrize("C,H,stride,batch", [(512, 14, 1, 256), (128, 56, 1, 96), (32, 112, 1, 40)])
def test_depthwise_layers_at_bench_sizes(C, H, stride, batch):
    """Sizes at which a block of the 3x3 kernel walks several pixel tiles and, for the two
    larger ones, the fp32 output is stored with the non-temporal hint (above 128 MiB)."""
    _say("depthwise at size %d@%d s%d batch %d" % (C, H, stride, batch))
    _dw_check(C, H, 3, stride, 1, batch, seed=C + batch)


OTHER_NET_CONVS = [
    # MobileNet pointwise (1x1) layers, AlexNet's 5x5 and 3x3 layers (first layer stays fp32), NIN's 5x5 / 1x1
    wl.ConvShape("mobilenet.pw.64x128@56", 64, 56, 128, 1, 1, 0),
    wl.ConvShape("mobilenet.pw.512x512@14", 512, 14, 512, 1, 1, 0),
    wl.ConvShape("mobilenet.pw.1024x1024@7", 1024, 7, 1024, 1, 1, 0),
    wl.ConvShape("alexnet.conv2.5x5", 96, 27, 256, 5, 1, 2),
    wl.ConvShape("alexnet.conv3.3x3", 256, 13, 384, 3, 1, 1),
    wl.ConvShape("alexnet.conv4.3x3", 384, 13, 384, 3, 1, 1),
    wl.ConvShape("nin.conv2.5x5", 96, 16, 192, 5, 1, 2),
    wl.ConvShape("nin.cccp.1x1", 192, 16, 160, 1, 1, 0),
    wl.ConvShape("nin.conv3.3x3", 192, 8, 192, 3, 1, 1),
]


@pytest.mark.parametrize("shape", OTHER_NET_CONVS, ids=lambda s: s.name)
def test_other_networks_conv_layers(shape):
    """Layer shapes of the other networks of the paper's tables through the ternary conv, on
    both matrix paths (batch 4)."""
    _say("other nets %s" % (shape,))
    case = wl.conv_case(shape, batch=4, seed=len(shape.name), per_channel=True, bn=True)
    ref = T.oracle_conv(case, True, relu=True)
    for fmt in (B.RTN_CODE_FP4, B.RTN_CODE_I8):
        got = T.hip_conv(case, True, relu=True, fmt=fmt)
        assert (got["D"].cpu().numpy() == ref["D"]).all()
        T.assert_y_close(got["y"].cpu().numpy(), ref["y"], shape.name)


# ------------------------------------------ guard bytes around every output buffer ------
def test_outputs_stay_inside_their_buffers():
    """Ragged problems with every output carved out of a larger poisoned allocation: the guard
    regions before and after each output must be untouched (pack, GEMM, conv on both matrix
    paths, ternarizing conv, depthwise conv)."""
    _say("guard regions around outputs")
    G = 4096

    def carve(shape, dtype, fill):
        n = int(np.prod(shape))
        esz = torch.empty(0, dtype=dtype).element_size()
        raw = torch.full((n * esz + 2 * G,), 0x5A, dtype=torch.uint8, device=T.DEV)
        view = raw[G:G + n * esz].view(dtype).view(*shape)
        view.fill_(fill)
        return raw, view

    def check(raw, what):
        r = raw.cpu().numpy()
        assert (r[:G] == 0x5A).all() and (r[-G:] == 0x5A).all(), what + ": wrote outside its buffer"

    shape = wl.ConvShape("g", 70, 9, 77, 3, 1, 1)
    case = wl.conv_case(shape, batch=3, seed=5, bn=True, Wx=11)
    x, w = T.dev(case["x"]), T.dev(case["w"])
    dw = np.asarray(case["delta_w"])
    for fmt in (B.RTN_CODE_FP4, B.RTN_CODE_I8):
        rowb = B.padded_k(70, fmt) // (2 if fmt == B.RTN_CODE_FP4 else 1)
        cdt = torch.uint8 if fmt == B.RTN_CODE_FP4 else torch.int8
        rc, codes = carve((3, 9, 11, rowb), cdt, 0)
        rs, sums = carve((3, 9, 11), torch.int32, 0)
        B.ternarize_pack(x, -float(case["delta_a"]), float(case["delta_a"]), fmt, codes=codes, sum_t=sums)
        cw, pw = B.ternarize_pack(w, T.thr_arg(-dw), T.thr_arg(dw), fmt)
        ep = B.Epilogue(T.gran_arg(case["alpha_a"]), T.gran_arg(case["beta_a"]), T.gran_arg(case["alpha_w"]),
                        T.gran_arg(case["beta_w"]), sums, pw, relu=True, bn_scale=T.dev(case["bn_scale"]),
                        bn_shift=T.dev(case["bn_shift"]))
        ra, acc = carve((3, 77, 9, 11), torch.int32, 0)
        ry, y = carve((3, 77, 9, 11), torch.float32, 0.0)
        B.ternary_conv2d(codes, cw, 3, 70, 9, 11, 77, 3, 3, 1, 1, ep=ep, acc_out=acc, want_acc=True, y_out=y, fmt=fmt)
        orow = B.padded_k(77, fmt) // (2 if fmt == B.RTN_CODE_FP4 else 1)
        rz, zc = carve((3, 9, 11, orow), cdt, 0)
        ry2, y2 = carve((3, 77, 9, 11), torch.float32, 0.0)
        B.ternary_conv2d_ternarize(codes, cw, 3, 70, 9, 11, 77, 3, 3, 1, 1, ep, -0.4, 0.6, codes_out=zc, residual=y,
                                   relu_out=True, y_out=y2, fmt=fmt)
        torch.cuda.synchronize()
        for raw, what in ((rc, "pack codes"), (rs, "pack sums"), (ra, "conv acc"), (ry, "conv y"), (rz, "codes out"),
                          (ry2, "block-tail y")):
            check(raw, "%s (format %d)" % (what, fmt))
        g = wl.gemm_case(131, 77, 200, seed=3)
        ca, sa = B.ternarize_pack(T.dev(g["xa"]), -0.5, 0.5, fmt)
        cb, sb = B.ternarize_pack(T.dev(g["xw"]), -0.5, 0.5, fmt)
        epg = B.Epilogue(T.dev(g["alpha_a"]), T.dev(g["beta_a"]), T.dev(g["alpha_w"]), T.dev(g["beta_w"]), sa, sb)
        rga, gacc = carve((131, 77), torch.int32, 0)
        rgy, gy = carve((131, 77), torch.float32, 0.0)
        B.ternary_gemm(ca, cb, 131, 77, 200, fmt=fmt, ep=epg, acc_out=gacc, want_acc=True, y_out=gy)
        torch.cuda.synchronize()
        check(rga, "gemm acc"), check(rgy, "gemm y")
    ca8, _ = B.ternarize_pack(x, -0.5, 0.5, want_sum=False)
    wd = T.dev((np.random.default_rng(1).standard_normal((70, 9)) * 0.3).astype(np.float32))
    cwd, _ = B.ternarize_pack(wd, -0.2, 0.2, want_sum=False)
    rd, dacc = carve((3, 70, 9, 11), torch.int32, 0)
    rdy, dy = carve((3, 70, 9, 11), torch.float32, 0.0)
    epd = B.Epilogue(1.0, 0.1, 1.2, None, None, None)
    B.ternary_depthwise_conv2d(ca8, cwd, 3, 70, 9, 11, 3, 3, 1, 1, ep=epd, acc_out=dacc, y_out=dy)
    torch.cuda.synchronize()
    check(rd, "depthwise acc"), check(rdy, "depthwise y")
