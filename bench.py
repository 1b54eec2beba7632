"""Benchmark of the RTN ternary conv/GEMM hot path on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic input:
for each of the 19 ternary conv layers of ResNet-18 at batch 256 (weights
pre-packed offline, S0), ternarize+pack the fp32 NCHW input (S1), run the
implicit-GEMM ternary convolution on the int8 matrix cores (S2+S3) with the
fused four-term reparameterization + ReLU + BN epilogue (S4) writing fp32 NCHW.
Inputs are resident in HBM before the timed region.

Prints ONE JSON line: metric / value / unit / ms_per_step and the run parameters,
`roofline` (the dominant kernel's achieved rate against the MI355X peak that bounds
it, from HIP events on the launch stream), `cpu_baseline` (the CPU oracle timed on a
bounded sample of the same workload), `fused_blocks` (the same convs with the
ternarizing epilogue, and the trunk as one chained forward pass) and `layers`
(per-layer times).  Other workloads: --workload gemm4096 | gemm_sweep | wgemm4096 |
resnet18_weight_only_convs | act_backward | weight_backward.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0   # MI355X dense int8 MFMA, TOP/s (2 ops per MAC)
FP4_PEAK_TFLOPS = 10100.0  # MI355X dense FP4 MFMA (the path the FP4 code storage runs on)
BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
HBM_PEAK_GBS = 8000.0
# HBM bytes per k_tmm launch of the default run (FP4 codes, batch 256): rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE passes summarised in profiles/k_tmm_conv_resnet18_b256.md, (2 * FETCH_SIZE + WRITE_SIZE) KiB
# averaged over the 19 launches of a step.  Measured 2026-11-28 on the kernels of commit 6a61329 (the
# conv's loads and stores have not changed since); a constant, not a live reading: the counters need the
# profiler.  It only applies to the default format, batch and tile choice.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = 109.3e6
MEASURED_TRAFFIC_STAMP = "rocprofv3 FETCH_SIZE/WRITE_SIZE, 2026-11-28, kernels of commit 6a61329"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=15)
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--workload", default="resnet18_ternary_convs",
                    choices=["resnet18_ternary_convs", "gemm4096", "wgemm4096", "resnet18_weight_only_convs",
                             "act_backward", "weight_backward", "gemm_sweep", "peaks", "config1",
                             "resnet18_full_forward", "quaternary_gemm", "mobilenet_layers"])
    ap.add_argument("--tile", type=int, default=-1, help="force an MFMA tile configuration (tuning)")
    ap.add_argument("--format", default="fp4", choices=["fp4", "i8"],
                    help="storage of the ternary codes on the matrix-core path: FP4 (E2M1) nibbles on the FP4 "
                         "matrix cores (default), or int8 on the int8 matrix cores")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-images", type=int, default=128,
                    help="images per layer the oracle is timed on (cpu_baseline sample)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "re-run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1912_02057_amd import binding as B
    from paper_1912_02057_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()  # raises if the HIP library is missing: there is no fallback
    if args.tile >= 0:
        B.set_tile_config(args.tile)
    dev = "cuda:0"
    torch.cuda.set_device(0)

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    def garg(v):
        v = np.asarray(v, dtype=np.float32)
        return float(v) if v.ndim == 0 else to_dev(v)

    ev = torch.cuda.Event
    FMT = B.RTN_CODE_FP4 if args.format == "fp4" else B.RTN_CODE_I8

    def code_row_bytes(channels):
        return B.padded_k(channels, FMT) // (2 if FMT == B.RTN_CODE_FP4 else 1)

    def code_tensor(n, hw, channels):
        return torch.empty((n, hw, hw, code_row_bytes(channels)),
                           dtype=torch.uint8 if FMT == B.RTN_CODE_FP4 else torch.int8, device=dev)

    def timed(fn, reps, warm=2):
        """Average milliseconds of fn() over reps launches, HIP events on the current stream."""
        for _ in range(warm):
            fn()
        e0, e1 = ev(enable_timing=True), ev(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    if args.workload == "peaks":
        # The ceilings a kernel can reach on this machine, measured: register-only loops of the two
        # matrix-core instructions the contraction uses, and plain streaming kernels.
        import ctypes as C
        PL = C.CDLL(os.path.join(ROOT, "paper_1912_02057_amd", "librtn_peaks.so"))
        PL.rtn_peaks_mfma.restype = C.c_double
        PL.rtn_peaks_mfma.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        PL.rtn_peaks_stream.restype = C.c_int
        PL.rtn_peaks_stream.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        opnd = torch.full((8192,), 0x22, dtype=torch.uint8, device=dev)
        blocks, iters = 256 * 8, 10000
        sink = torch.empty(blocks * 256, dtype=torch.float32, device=dev)
        res = {}
        for kind, name in ((0, "mfma_i32_32x32x32_i8"), (1, "mfma_f32_32x32x64_fp4")):
            macs = []

            def go():
                macs.append(PL.rtn_peaks_mfma(kind, blocks, iters, opnd.data_ptr(), sink.data_ptr(), st))
            ms = timed(go, 5)
            assert macs[-1] > 0
            res[name] = dict(pmacs=round(macs[-1] / ms / 1e12, 3), pops=round(2 * macs[-1] / ms / 1e12, 3),
                             implied_clock_ghz=round(macs[-1] / ms / 1e6 / (256 * 4 * (1024 if kind == 0 else 2048)), 3))
        streams = {}
        for mb in (64, 256, 1024):
            nbytes = mb << 20
            a = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(1)
            b = torch.empty(nbytes, dtype=torch.uint8, device=dev)
            row = {}
            for kind, name, moved in ((1, "read", 1), (2, "write", 1), (0, "copy", 2)):
                ms = timed(lambda: PL.rtn_peaks_stream(kind, b.data_ptr(), a.data_ptr(), nbytes, st), 10)
                row[name + "_gbs"] = round(moved * nbytes / ms / 1e6, 0)
            streams["%d MiB" % mb] = row
            del a, b
        fp4 = res["mfma_f32_32x32x64_fp4"]
        print(json.dumps({
            "metric": "achievable ceilings on this machine: register-only matrix-core loops and streaming kernels",
            "value": round(fp4["pmacs"] * 1e3, 1), "unit": "TMAC/s", "n_gpus": 1, "steps": 5, "warmup": 2,
            "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp4",
            "data": "synthetic", "config": {"workload": "peaks: MFMA-only loops (int8, FP4) and stream read/write/copy"},
            "roofline": {"bound": "mfma", "kernel": "k_mfma_loop<fp4> (no memory traffic)", "achieved": round(2 * fp4["pmacs"] * 1e3, 1),
                         "peak": FP4_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(2 * fp4["pmacs"] * 1e3 / FP4_PEAK_TFLOPS, 4),
                         "traffic": None},
            "cpu_baseline": None, "mfma": res, "stream": streams}))
        return

    if args.workload == "config1":
        # the single-layer configuration: 3x3, stride 1, pad 1, batch 1, 64 -> 64 channels at 56x56.
        # 0.116 GMAC and 1.8 MB: two dependent launches, bound by launch and memory latency, so the
        # figure that matters is the latency in microseconds.
        case = wl.config1_case()
        sh = case["shape"]
        x, w = to_dev(case["x"]), to_dev(case["w"])
        dw, da = float(case["delta_w"]), float(case["delta_a"])
        cw, pw = B.ternarize_pack(w, -dw, dw, FMT)
        ca = code_tensor(1, sh.H, sh.C)
        pa = torch.empty((1, sh.H, sh.H), dtype=torch.int32, device=dev)
        y = torch.empty((1, sh.O, sh.OH, sh.OH), dtype=torch.float32, device=dev)
        ep = B.Epilogue(garg(case["alpha_a"]), garg(case["beta_a"]), garg(case["alpha_w"]), garg(case["beta_w"]), pa, pw)
        ws = B.conv2d_prepare_constants(sh.C, sh.O, sh.k, sh.k, sh.pad, ep)

        def one():
            B.ternarize_pack(x, -da, da, FMT, codes=ca, sum_t=pa)
            B.ternary_conv2d(ca, cw, 1, sh.C, sh.H, sh.H, sh.O, sh.k, sh.k, sh.stride, sh.pad, ep=ep, y_out=y,
                             workspace=ws, fmt=FMT)
        ms = timed(one, max(args.steps, 50), warm=max(args.warmup, 5))
        ms_conv = timed(lambda: B.ternary_conv2d(ca, cw, 1, sh.C, sh.H, sh.H, sh.O, sh.k, sh.k, sh.stride, sh.pad, ep=ep,
                                                 y_out=y, workspace=ws, fmt=FMT), 50, warm=5)
        # with the operands evicted between calls: a 512 MiB fill in between, its own time taken off
        junk = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
        ms_fill = timed(lambda: junk.fill_(3), 10)
        ms_cold = timed(lambda: (junk.fill_(3), one()), 10) - ms_fill
        macs = sh.macs(1)
        cpu = None
        if not args.no_cpu_baseline:
            from oracle import rtn_oracle as orc
            c0 = time.perf_counter()
            for _ in range(20):
                ta = orc.ternarize(case["x"], -case["delta_a"], case["delta_a"])
                tw = orc.ternarize(case["w"], -case["delta_w"], case["delta_w"])
                D = orc.conv_acc(ta, tw, sh.stride, sh.pad)
                Sa, Sw, Kv = orc.conv_sums(ta, tw, sh.stride, sh.pad, True)
                orc.conv_epilogue(D, Sa, Sw, Kv, case["alpha_a"], case["beta_a"], case["alpha_w"], case["beta_w"])
            t_cpu = (time.perf_counter() - c0) / 20
            cpu = dict(value=round(macs / t_cpu / 1e12, 6), unit="TMAC/s", cores=orc.num_threads(), kind="oracle",
                       sample="the whole configuration, 20 repetitions", seconds=round(20 * t_cpu, 2))
        print(json.dumps({
            "metric": "effective ternary MAC/s, single 3x3 conv at batch 1 (pack + conv); latency-bound: see latency_us",
            "value": round(macs / (ms * 1e-3) / 1e12, 3), "unit": "TMAC/s", "n_gpus": 1, "steps": max(args.steps, 50),
            "warmup": max(args.warmup, 5), "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": args.format, "data": "synthetic",
            "config": {"workload": "config 1: 3x3 s1 p1, batch 1, 64->64 @ 56x56, per-layer scalars", "format": args.format},
            "latency_us": {"pack_plus_conv": round(ms * 1e3, 2), "conv_only": round(ms_conv * 1e3, 2),
                           "pack_plus_conv_operands_evicted": round(ms_cold * 1e3, 2),
                           "note": "two dependent launches of a few microseconds each; bound by launch and memory "
                                   "latency, not by a roofline"},
            "roofline": {"bound": "hbm", "kernel": "k_tmm conv (latency-bound at this size)",
                         "achieved": round((sh.C * sh.H * sh.H * 5 + sh.O * sh.OH * sh.OH * 4) / (ms * 1e-3) / 1e9, 1),
                         "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round((sh.C * sh.H * sh.H * 5 + sh.O * sh.OH * sh.OH * 4) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 5),
                         "traffic": None},
            "cpu_baseline": cpu}))
        return

    if args.workload == "resnet18_full_forward":
        # the full-network configuration: fp32 stem and head in torch (timed, reported, excluded from the
        # ternary figure), the 8 ternary blocks through the library with every hand-over fused
        from paper_1912_02057_amd.resnet18 import TernaryResNet18
        prm = wl.resnet18_network_params(seed=4)
        rng = np.random.Generator(np.random.PCG64(44))
        images = to_dev(rng.standard_normal((args.batch, 3, 224, 224), dtype=np.float32))
        net = TernaryResNet18(prm, args.batch, dev, FMT)
        x0 = net.stem(images)
        out = net.trunk(x0)
        ms_stem = timed(lambda: net.stem(images), 5)
        ms_head = timed(lambda: net.head(out), 5)
        import gc
        gc.collect()
        gc.disable()
        for _ in range(args.warmup):
            net.trunk(x0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            net.trunk(x0)
        torch.cuda.synchronize()
        ms_trunk = (time.perf_counter() - t0) * 1e3 / args.steps
        gc.enable()
        macs, nbytes = net.trunk_macs(), net.trunk_bytes()
        cpu = None
        if not args.no_cpu_baseline:
            from oracle import rtn_oracle as orc
            n_img = max(1, args.cpu_images // 16)
            xs = x0[:n_img].cpu().numpy()
            lo, hi = -prm["delta_a"], prm["delta_a"]
            P = prm["layers"]

            def olayer(ta, p, relu):
                s_ = p["sh"]
                tw = orc.ternarize(p["w"], -np.asarray(p["dw"]), p["dw"])
                D = orc.conv_acc(ta, tw, s_.stride, s_.pad)
                Sa, Sw, Kv = orc.conv_sums(ta, tw, s_.stride, s_.pad, True)
                return orc.conv_epilogue(D, Sa, Sw, Kv, p["aa"], p["ba"], p["aw"], p["bw"], relu=relu,
                                         bn_scale=p["bs"], bn_shift=p["bh"])
            c0 = time.perf_counter()
            xo, ta = xs, orc.ternarize(xs, lo, hi)
            for i1, i2, ids in wl.resnet18_block_topology():
                y1 = olayer(ta, P[i1], True)
                y2 = olayer(orc.ternarize_nchw(y1, lo, hi), P[i2], False)
                sc = xo if ids is None else olayer(ta, P[ids], False)
                xo = orc.add_relu(y2, sc, True)
                ta = orc.ternarize_nchw(xo, lo, hi)
            t_cpu = time.perf_counter() - c0
            cpu = dict(value=round(macs / args.batch * n_img / t_cpu / 1e12, 6), unit="TMAC/s", cores=orc.num_threads(),
                       kind="oracle", sample="the chained trunk on %d images (of %d)" % (n_img, args.batch),
                       seconds=round(t_cpu, 2))
        gbs = nbytes / (ms_trunk * 1e-3) / 1e9
        print(json.dumps({
            "metric": "effective ternary MAC/s, ResNet-18 forward: the 19 ternary convs as 8 fused residual blocks "
                      "(fp32 stem and head timed separately and not counted)",
            "value": round(macs / (ms_trunk * 1e-3) / 1e12, 3), "unit": "TMAC/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(ms_trunk, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": args.format, "data": "synthetic",
            "config": {"workload": "full ResNet-18 forward, batch %d, 224x224x3, ternary trunk: 1 pack + 19 convs" % args.batch,
                       "batch": args.batch, "format": args.format},
            "fp32_parts_ms": {"stem_conv7x7_bn_relu_maxpool": round(ms_stem, 4), "avgpool_fc": round(ms_head, 4),
                              "note": "torch fp32 ops, outside the ternary library"},
            "images_per_s_trunk": round(args.batch / (ms_trunk * 1e-3), 0),
            "roofline": {"bound": "hbm", "kernel": "the trunk's 20 launches as a whole (k_pack + 19 k_tmm)",
                         "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                         "traffic": None, "bytes_per_step": nbytes,
                         "mfma_tops": round(2 * macs / (ms_trunk * 1e-3) / 1e12, 1),
                         "mfma_frac_of_int8_peak": round(2 * macs / (ms_trunk * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4)},
            "cpu_baseline": cpu}))
        return


    if args.workload == "quaternary_gemm":
        # the paper's hardware comparison (ternary circuit against the 2-bit quaternary one) on this machine:
        # the same M = N = K = 4096 product on the bit-plane / vector-ALU paths the two circuits map to
        # (ternary: 3 logic + 2 count operations per 64 products; quaternary: 4 AND + 4 count), and on the
        # matrix cores, where both are the same instruction stream
        rng = np.random.Generator(np.random.PCG64(21))
        x1 = to_dev(rng.random((4096, 4096), dtype=np.float32))
        x2 = to_dev(rng.random((4096, 4096), dtype=np.float32))
        acc = torch.empty((4096, 4096), dtype=torch.int32, device=dev)
        rowsq = {}
        macs = 4096.0 ** 3
        for fmt, name in ((B.RTN_CODE_BITPLANE, "bit-serial AND/popcount (vector ALU)"), (B.RTN_CODE_I8, "int8 matrix cores"),
                          (B.RTN_CODE_FP4, "FP4 matrix cores")):
            qa, qw = B.quaternary_pack(x1, 1 / 6, 0.5, 5 / 6, fmt), B.quaternary_pack(x2, 1 / 6, 0.5, 5 / 6, fmt)
            ms = timed(lambda: B.quaternary_gemm(qa, qw, 4096, 4096, 4096, fmt, acc_out=acc), 3 if fmt == B.RTN_CODE_BITPLANE else 10)
            ta, _ = B.ternarize_pack(x1, 0.33, 0.66, fmt)
            tw, _ = B.ternarize_pack(x2, 0.33, 0.66, fmt)
            mt = timed(lambda: B.ternary_gemm(ta, tw, 4096, 4096, 4096, fmt=fmt, acc_out=acc, want_acc=True),
                       3 if fmt == B.RTN_CODE_BITPLANE else 10)
            rowsq[name] = dict(quaternary_us=round(ms * 1e3, 1), quaternary_tmacs=round(macs / ms / 1e9, 1),
                               ternary_us=round(mt * 1e3, 1), ternary_tmacs=round(macs / mt / 1e9, 1),
                               ternary_speedup=round(ms / mt, 2))
        best = rowsq["FP4 matrix cores"]
        print(json.dumps({
            "metric": "effective MAC/s, 2-bit quaternary GEMM M=N=K=4096 (the paper's comparison system), accumulators only",
            "value": best["quaternary_tmacs"], "unit": "TMAC/s", "n_gpus": 1, "steps": 10, "warmup": 2,
            "ms_per_step": round(best["quaternary_us"] / 1e3, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "fp4", "data": "synthetic",
            "config": {"workload": "quaternary and ternary GEMM 4096^3 on the bit-plane, int8 and FP4 paths"},
            "roofline": {"bound": "mfma", "kernel": "k_tmm (FP4 MFMA) on quaternary codes", "achieved": round(2 * best["quaternary_tmacs"], 1),
                         "peak": FP4_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(2 * best["quaternary_tmacs"] / FP4_PEAK_TFLOPS, 4),
                         "traffic": None},
            "cpu_baseline": None, "paths": rowsq,
            "context": "the paper's circuits: ternary 22.17 uW / 199.43 um^2 against quaternary 76.09 uW / 831.62 um^2 "
                       "(3.43x power, 4.17x area; FPGA / 45 nm flow, Table 3)"}))
        return


    if args.workload == "mobilenet_layers":
        # MobileNet's ternary layers (the paper's third ImageNet network): 13 depthwise 3x3 convs (K = 9,
        # streaming kernel) and 13 pointwise 1x1 convs (matrix cores), each with its pack, batch 256
        cfgs = [(32, 112, 1, 64), (64, 112, 2, 128), (128, 56, 1, 128), (128, 56, 2, 256), (256, 28, 1, 256),
                (256, 28, 2, 512)] + [(512, 14, 1, 512)] * 5 + [(512, 14, 2, 1024), (1024, 7, 1, 1024)]
        rows_, tot_s, tot_macs = [], 0.0, 0.0
        rng = np.random.Generator(np.random.PCG64(9))
        for (Cc, H, st_, Op) in cfgs:
            OH = (H + 2 - 3) // st_ + 1
            x = torch.randn((args.batch, Cc, H, H), device=dev)
            wd = to_dev((rng.standard_normal((Cc, 9)) * 0.3).astype(np.float32))
            cwd, _ = B.ternarize_pack(wd, -0.2, 0.2, want_sum=False)
            aw = to_dev(rng.uniform(0.5, 1.5, Cc).astype(np.float32))
            epd = B.Epilogue(1.1, 0.1, aw, None, None, None, relu=True)
            ca = torch.empty((args.batch, H, H, B.padded_k(Cc)), dtype=torch.int8, device=dev)
            yd = torch.empty((args.batch, Cc, OH, OH), dtype=torch.float32, device=dev)
            ms_pack = timed(lambda: B.ternarize_pack(x, -0.5, 0.5, codes=ca, want_sum=False), 5)
            ms_dw = timed(lambda: B.ternary_depthwise_conv2d(ca, cwd, args.batch, Cc, H, H, 3, 3, st_, 1, ep=epd, y_out=yd), 5)
            dw_bytes = ca.numel() + yd.numel() * 4
            # pointwise conv on the depthwise output
            shp = wl.ConvShape("pw", Cc, OH, Op, 1, 1, 0)
            case = wl.conv_case(shp, batch=1, seed=Cc, per_channel=True, bn=True)
            dwp = np.asarray(case["delta_w"])
            cwp, pwp = B.ternarize_pack(to_dev(case["w"]), garg(-dwp), garg(dwp), FMT)
            epp = B.Epilogue(garg(case["alpha_a"]), garg(case["beta_a"]), garg(case["alpha_w"]), garg(case["beta_w"]),
                             None, pwp, relu=True, bn_scale=to_dev(case["bn_scale"]), bn_shift=to_dev(case["bn_shift"]))
            wsp = B.conv2d_prepare_constants(Cc, Op, 1, 1, 0, epp)
            cap = code_tensor(args.batch, OH, Cc)
            yp = torch.empty((args.batch, Op, OH, OH), dtype=torch.float32, device=dev)
            ms_pack2 = timed(lambda: B.ternarize_pack(yd, -0.5, 0.5, FMT, codes=cap, want_sum=False), 5)
            ms_pw = timed(lambda: B.ternary_conv2d(cap, cwp, args.batch, Cc, OH, OH, Op, 1, 1, 1, 0, ep=epp, y_out=yp,
                                                   workspace=wsp, fmt=FMT), 5)
            macs_dw = args.batch * Cc * OH * OH * 9.0
            macs_pw = args.batch * Op * OH * OH * float(Cc)
            rows_.append(dict(layer="dw %d@%d s%d -> pw %d" % (Cc, H, st_, Op), dw_us=round(ms_dw * 1e3, 1),
                              dw_gbs=round(dw_bytes / ms_dw / 1e6, 0), dw_pct_hbm=round(100 * dw_bytes / ms_dw / 1e6 / HBM_PEAK_GBS, 1),
                              pack_dw_us=round(ms_pack * 1e3, 1), pw_us=round(ms_pw * 1e3, 1), pack_pw_us=round(ms_pack2 * 1e3, 1),
                              pw_tmacs=round(macs_pw / ms_pw / 1e9, 1)))
            tot_s += (ms_pack + ms_dw + ms_pack2 + ms_pw) * 1e-3
            tot_macs += macs_dw + macs_pw
            del x, ca, yd, cap, yp
        dwb = sum(r["dw_gbs"] * r["dw_us"] for r in rows_) / sum(r["dw_us"] for r in rows_)
        print(json.dumps({
            "metric": "effective ternary MAC/s, MobileNet's 13 depthwise + 13 pointwise ternary layers, each with its pack",
            "value": round(tot_macs / tot_s / 1e12, 3), "unit": "TMAC/s", "n_gpus": 1, "steps": 5, "warmup": 2,
            "ms_per_step": round(tot_s * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": args.format, "data": "synthetic",
            "config": {"workload": "MobileNet ternary layers (depthwise 3x3 + pointwise 1x1), batch %d" % args.batch,
                       "batch": args.batch, "format": args.format},
            "roofline": {"bound": "hbm", "kernel": "k_dwconv (depthwise 3x3, int8 codes in, fp32 out)",
                         "achieved": round(dwb, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(dwb / HBM_PEAK_GBS, 4),
                         "traffic": None},
            "cpu_baseline": None, "layers": rows_}))
        return

    if args.workload == "gemm_sweep":
        # M x N x K sweep of the ternary GEMM over sparsity, on both contraction paths: codes resident,
        # one timed call = contraction + fused epilogue (the pack of the activations is timed beside it)
        rows = []
        tot_macs, tot_s = 0.0, 0.0
        for M in (8192, 16384):
            for NK in (4096, 8192):
                for p0 in (0.2, 0.5, 0.8):
                    case = wl.gemm_case(M, NK, NK, p_zero=p0, seed=int(1000 * p0) + 3)
                    xa, xw = to_dev(case["xa"]), to_dev(case["xw"])
                    for fmt, name in ((B.RTN_CODE_FP4, "mfma_fp4"), (B.RTN_CODE_I8, "mfma_i8"),
                                      (B.RTN_CODE_BITPLANE, "popcount")):
                        ca, sa = B.ternarize_pack(xa, -0.5, 0.5, fmt)
                        cw, sw = B.ternarize_pack(xw, -0.5, 0.5, fmt)
                        ep = B.Epilogue(garg(case["alpha_a"]), garg(case["beta_a"]), garg(case["alpha_w"]),
                                        garg(case["beta_w"]), sa, sw)
                        y = torch.empty((M, NK), dtype=torch.float32, device=dev)
                        reps = 2 if name == "popcount" else 5
                        for _ in range(2):
                            B.ternary_gemm(ca, cw, M, NK, NK, fmt=fmt, ep=ep, y_out=y)
                        # the better of two timing passes: a pass now and then catches a stall of tens
                        # of milliseconds that has nothing to do with the kernels (same launches, no
                        # allocation inside)
                        us = pus = float("inf")
                        for _ in range(2):
                            e0, e1, e2 = ev(enable_timing=True), ev(enable_timing=True), ev(enable_timing=True)
                            e0.record()
                            for _ in range(reps):
                                B.ternary_gemm(ca, cw, M, NK, NK, fmt=fmt, ep=ep, y_out=y)
                            e1.record()
                            for _ in range(reps):
                                B.ternarize_pack(xa, -0.5, 0.5, fmt, codes=ca, sum_t=sa)   # into the resident buffers
                            e2.record()
                            torch.cuda.synchronize()
                            us = min(us, e0.elapsed_time(e1) * 1e3 / reps)
                            pus = min(pus, e1.elapsed_time(e2) * 1e3 / reps)
                        macs = float(M) * NK * NK
                        row = dict(M=M, N=NK, K=NK, p_zero=p0, path=name, gemm_us=round(us, 1),
                                   pack_us=round(pus, 1), tmacs=round(macs / us / 1e6, 1),
                                   pct_int8_mfma_peak=round(100 * 2 * macs / us / 1e6 / INT8_PEAK_TOPS, 1))
                        if name == "mfma_fp4":
                            row["pct_fp4_mfma_peak"] = round(100 * 2 * macs / us / 1e6 / FP4_PEAK_TFLOPS, 1)
                        if name == "popcount":
                            # its own roof is the vector ALU: 5 64-bit operations (3 logic, 2 popcount-accumulate)
                            # per 64 MACs per lane, 64 lanes per clock per CU, 256 CUs at 2.4 GHz,
                            # a 64-bit operation being two 32-bit issue slots
                            valu_bound = 256 * 64 * 2.4e9 * 64 / (5 * 2) / 1e12
                            row["valu_bound_tmacs"] = round(valu_bound, 1)
                            row["frac_of_valu_bound"] = round(macs / us / 1e6 / valu_bound, 3)
                        rows.append(row)
                        if name == "mfma_fp4":
                            tot_macs += macs
                            tot_s += (us + pus) * 1e-6
                        del ca, cw, sa, sw, y, ep
                    del xa, xw, case
        mf = [r for r in rows if r["path"] == "mfma_fp4"]
        best = max(mf, key=lambda r: r["tmacs"])
        cpu = None
        if not args.no_cpu_baseline:
            from oracle import rtn_oracle as orc
            case = wl.gemm_case(8192, 4096, 4096, p_zero=0.5, seed=503)
            rws = np.arange(0, 8192, 8192 // 256, dtype=np.int64)
            c0 = time.perf_counter()
            ta = orc.ternarize(case["xa"][rws], -0.5, 0.5)
            tw = orc.ternarize(case["xw"], -0.5, 0.5)
            D = orc.gemm_acc_rows(ta, tw, np.arange(rws.size, dtype=np.int64))
            orc.gemm_epilogue(D, 4096, orc.row_sums(ta), orc.row_sums(tw), case["alpha_a"][rws], case["beta_a"][rws],
                              case["alpha_w"], case["beta_w"])
            t_cpu = time.perf_counter() - c0
            cpu = dict(value=round(rws.size * 4096 * 4096 / t_cpu / 1e12, 6), unit="TMAC/s", cores=orc.num_threads(),
                       kind="oracle", sample="256 of 8192 rows of the 8192 x 4096 x 4096 point, all columns",
                       seconds=round(t_cpu, 2))
        print(json.dumps({
            "metric": "effective ternary MAC/s, ternary GEMM sweep (pack + contraction + epilogue, FP4 matrix-core path)",
            "value": round(tot_macs / tot_s / 1e12, 3), "unit": "TMAC/s", "n_gpus": 1, "steps": 5, "warmup": 2,
            "ms_per_step": round(tot_s * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "fp4", "data": "synthetic",
            "config": {"workload": "ternary GEMM sweep: M in {8192,16384} x N=K in {4096,8192} x P(0) in {0.2,0.5,0.8}, "
                                   "FP4 and int8 matrix-core paths and the bit-plane popcount path"},
            "roofline": {"bound": "mfma", "kernel": "k_tmm (FP4 MFMA GEMM + fused epilogue), best point",
                         "achieved": round(2 * best["tmacs"], 1), "peak": FP4_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(2 * best["tmacs"] / FP4_PEAK_TFLOPS, 4),
                         "frac_of_int8_peak": round(2 * best["tmacs"] / INT8_PEAK_TOPS, 4), "traffic": None},
            "cpu_baseline": cpu, "sweep": rows}))
        return
    if args.workload == "resnet18_ternary_convs":
        shapes = wl.resnet18_ternary_layers()
        layers = []
        for i, sh in enumerate(shapes):
            case = wl.conv_case(sh, batch=args.batch, seed=100 + i, per_channel=True, bn=True)
            x = to_dev(case["x"])
            w = to_dev(case["w"])
            dw = np.asarray(case["delta_w"])
            cw, pw = B.ternarize_pack(w, garg(-dw), garg(dw), FMT)       # S0, offline
            ca = code_tensor(args.batch, sh.H, sh.C)
            pa = torch.empty((args.batch, sh.H, sh.H), dtype=torch.int32, device=dev)
            y = torch.empty((args.batch, sh.O, sh.OH, sh.OH), dtype=torch.float32, device=dev)
            ws = torch.empty(B.conv2d_workspace_bytes(sh.O, sh.k, sh.k, sh.pad), dtype=torch.uint8, device=dev)
            ep = B.Epilogue(garg(case["alpha_a"]), garg(case["beta_a"]), garg(case["alpha_w"]),
                            garg(case["beta_w"]), pa, pw, relu=True,
                            bn_scale=to_dev(case["bn_scale"]), bn_shift=to_dev(case["bn_shift"]))
            B.conv2d_prepare_constants(sh.C, sh.O, sh.k, sh.k, sh.pad, ep, ws)   # S0, offline
            # block tails: conv -> BN -> (+ shortcut) -> ReLU, i.e. no ReLU before the BN affine
            ep_tail = B.Epilogue(garg(case["alpha_a"]), garg(case["beta_a"]), garg(case["alpha_w"]),
                                 garg(case["beta_w"]), pa, pw, relu=False,
                                 bn_scale=to_dev(case["bn_scale"]), bn_shift=to_dev(case["bn_shift"]))
            ws_tail = torch.empty_like(ws)
            B.conv2d_prepare_constants(sh.C, sh.O, sh.k, sh.k, sh.pad, ep_tail, ws_tail)
            layers.append(dict(sh=sh, x=x, cw=cw, pw=pw, ca=ca, pa=pa, y=y, ws=ws, ep=ep,
                               ep_tail=ep_tail, ws_tail=ws_tail,
                               da=float(case["delta_a"]), case=case if i < 0 else None))
            del case
        L = B.lib()
        import ctypes as C

        def pack(l):
            sh = l["sh"]
            lo, hi = C.c_float(-l["da"]), C.c_float(l["da"])
            rc = L.rtn_ternarize_pack(l["x"].data_ptr(), B.RTN_NCHW, args.batch, sh.C, sh.H, sh.H,
                                      C.addressof(lo), C.addressof(hi), B.RTN_SCALAR, FMT,
                                      l["ca"].data_ptr(), l["pa"].data_ptr(), stream)
            assert rc == 0, rc

        def conv(l, ca=None):
            sh = l["sh"]
            B.ternary_conv2d(l["ca"] if ca is None else ca, l["cw"], args.batch, sh.C, sh.H, sh.H, sh.O,
                             sh.k, sh.k, sh.stride, sh.pad, B.RTN_PAD_TRUE_ZERO, ep=l["ep"], y_out=l["y"],
                             workspace=l["ws"], fmt=FMT)

        # The same 19 convs arranged as ResNet-18's 8 residual blocks, with the first conv
        # of each block handing its output to the second as codes (ternarizing epilogue):
        # one pack per block input (shared by conv1 and the downsample conv), no fp32
        # round trip between conv1 and conv2.
        blocks = [(0, 1, None), (2, 3, None)]
        for s_ in range(3):
            b_ = 4 + 5 * s_
            blocks += [(b_, b_ + 1, b_ + 2), (b_ + 3, b_ + 4, None)]

        def step_blocks():
            for i1, i2, ids in blocks:
                l1, l2 = layers[i1], layers[i2]
                sh = l1["sh"]
                pack(l1)
                B.ternary_conv2d_ternarize(l1["ca"], l1["cw"], args.batch, sh.C, sh.H, sh.H, sh.O, sh.k, sh.k,
                                           sh.stride, sh.pad, l1["ep"], -l2["da"], l2["da"],
                                           codes_out=l2["ca"], workspace=l1["ws"], fmt=FMT)
                conv(l2)
                if ids is not None:
                    conv(layers[ids], ca=l1["ca"])

        # The trunk as one chained forward: the input is packed once; conv1 of a block emits
        # conv2's codes; conv2's block-tail epilogue adds the shortcut (the block input, or
        # the downsample conv's output), applies the ReLU and writes both the fp32 block
        # output (the next shortcut) and the next block's codes.  1 pack + 19 convs.
        last_codes = code_tensor(args.batch, 7, 512)

        def trunk_forward():
            pack(layers[0])
            cur_x, cur_codes = layers[0]["x"], layers[0]["ca"]
            for bi, (i1, i2, ids) in enumerate(blocks):
                l1, l2 = layers[i1], layers[i2]
                sh, sh2 = l1["sh"], l2["sh"]
                B.ternary_conv2d_ternarize(cur_codes, l1["cw"], args.batch, sh.C, sh.H, sh.H, sh.O, sh.k, sh.k,
                                           sh.stride, sh.pad, l1["ep"], -l2["da"], l2["da"],
                                           codes_out=l2["ca"], workspace=l1["ws"], fmt=FMT)
                if ids is not None:
                    conv(layers[ids], ca=cur_codes)
                    res = layers[ids]["y"]
                else:
                    res = cur_x
                nxt = layers[blocks[bi + 1][0]] if bi + 1 < len(blocks) else None
                nxt_codes = nxt["ca"] if nxt is not None else last_codes
                nda = nxt["da"] if nxt is not None else 0.5
                B.ternary_conv2d_ternarize(l2["ca"], l2["cw"], args.batch, sh2.C, sh2.H, sh2.H, sh2.O, sh2.k,
                                           sh2.k, sh2.stride, sh2.pad, l2["ep_tail"], -nda, nda,
                                           codes_out=nxt_codes, workspace=l2["ws_tail"], residual=res,
                                           relu_out=True, y_out=l2["y"], fmt=FMT)
                cur_x, cur_codes = l2["y"], nxt_codes

        stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)

        def step(timers=None):
            for i, l in enumerate(layers):
                if timers is not None:
                    timers[i][0].record()
                pack(l)
                if timers is not None:
                    timers[i][1].record()
                conv(l)
                if timers is not None:
                    timers[i][2].record()

        macs_step = sum(l["sh"].macs(args.batch) for l in layers)
        workload = "ResNet-18 ternary conv stack (19 layers), batch %d, fp32 NCHW in/out, %s codes" % (args.batch,
                                                                                                     args.format)
        nlaunch = len(layers)
    elif args.workload == "act_backward":
        # backward of the reparameterized ternary activation over the largest activation tensor of
        # the stack (batch x 64 x 56 x 56): reads a and g, writes dL/da, reduces dgamma and dbeta
        nel = args.batch * 64 * 56 * 56
        rng = np.random.Generator(np.random.PCG64(11))
        ba_, bg_ = rng.standard_normal(nel, dtype=np.float32), rng.standard_normal(nel, dtype=np.float32)
        ad, gd = to_dev(ba_), to_dev(bg_)
        dad = torch.empty_like(ad)
        sums = torch.empty(2, dtype=torch.float64, device=dev)
        wsp = torch.empty(B.lib().rtn_activation_backward_workspace_bytes(nel), dtype=torch.uint8, device=dev)

        def step(timers=None):
            if timers is not None:
                timers[0][0].record()
                timers[0][1].record()
            B.activation_backward(ad, gd, -0.5, 0.5, 0.9, grad_in=dad, sums=sums, workspace=wsp)
            if timers is not None:
                timers[0][2].record()

        macs_step = nel          # "MACs" here: elements (one multiply-add into each of the two sums)
        workload = "backward of the reparameterized ternary activation, %d x 64 x 56 x 56 fp32" % args.batch
        nlaunch = 1
        layers = [dict(sh=None)]
    elif args.workload == "weight_backward":
        # backward of the ternary weight transform over the filters of the 19 ternary conv layers (one call
        # per layer): reads W and g, writes dL/dW, reduces dalpha, dk_W, db_W per filter
        wb = []
        rng = np.random.Generator(np.random.PCG64(12))
        for sh in wl.resnet18_ternary_layers():
            O_, K_ = sh.O, sh.C * sh.k * sh.k
            hw = (rng.standard_normal((O_, K_), dtype=np.float32) * np.float32(0.6))
            hg = rng.standard_normal((O_, K_), dtype=np.float32)
            hk = (0.7 + rng.random(O_)).astype(np.float32)
            hb = (rng.standard_normal(O_) * 0.1).astype(np.float32)
            ha = (0.2 + rng.random(O_)).astype(np.float32)
            wb.append(dict(host=(hw, hg, hk, hb, ha), dev=[to_dev(v) for v in (hw, hg, hk, hb, ha)],
                           dw=torch.empty((O_, K_), dtype=torch.float32, device=dev),
                           sums=torch.empty((O_, 3), dtype=torch.float64, device=dev)))

        def step(timers=None):
            for i, l in enumerate(wb):
                if timers is not None:
                    timers[i][0].record()
                    timers[i][1].record()
                w_, g_, k_, b_, a_ = l["dev"]
                B.weight_backward(w_, g_, -0.5, 0.5, k_, b_, a_, grad_w=l["dw"], sums=l["sums"])
                if timers is not None:
                    timers[i][2].record()

        macs_step = sum(l["host"][0].size for l in wb)   # "MACs" here: weight elements
        workload = "backward of the ternary weight transform, the filters of the 19 ternary convs of ResNet-18"
        nlaunch = len(wb)
        layers = [dict(sh=None)] * nlaunch
    elif args.workload == "resnet18_weight_only_convs":
        # the same 19 layer shapes with ternary weights and fp32 activations (per layer: weight side
        # prepared once, offline; the timed call splits the activations and runs the bf16 matrix-core conv)
        wlayers = []
        for i, sh in enumerate(wl.resnet18_ternary_layers()):
            case = wl.conv_case(sh, batch=args.batch, seed=100 + i, per_channel=True, bn=True)
            dw = np.asarray(case["delta_w"])
            cw, _ = B.ternarize_pack(to_dev(case["w"]), garg(-dw), garg(dw), want_sum=False)    # S0, offline
            prep = B.weight_conv2d_prepare(cw, sh.C, sh.O, sh.k, sh.k, sh.pad, to_dev(case["alpha_w"]),
                                           bn_scale=to_dev(case["bn_scale"]), bn_shift=to_dev(case["bn_shift"]))
            wlayers.append(dict(sh=sh, x=to_dev(case["x"]), prep=prep,
                                y=torch.empty((args.batch, sh.O, sh.OH, sh.OH), dtype=torch.float32, device=dev),
                                ws=torch.empty(B.lib().rtn_weight_conv2d_workspace_bytes(
                                    args.batch, sh.C, sh.H, sh.H, sh.O, sh.k, sh.k, sh.pad), dtype=torch.uint8,
                                    device=dev)))
            del case

        def step(timers=None):
            for i, l in enumerate(wlayers):
                sh = l["sh"]
                if timers is not None:
                    timers[i][0].record()
                    timers[i][1].record()
                B.ternary_weight_conv2d(l["x"], None, sh.O, sh.k, sh.k, sh.stride, sh.pad, relu=True,
                                        y_out=l["y"], workspace=l["ws"], prepared=l["prep"])
                if timers is not None:
                    timers[i][2].record()

        macs_step = sum(l["sh"].macs(args.batch) for l in wlayers)
        workload = "ResNet-18 conv stack (19 layers), ternary weights x fp32 activations, batch %d" % args.batch
        nlaunch = len(wlayers)
        layers = [dict(sh=None)] * nlaunch
    elif args.workload == "wgemm4096":
        # weight-only ternary GEMM: fp32 activations N(0,1), ternary weights, per-column alpha
        rng = np.random.Generator(np.random.PCG64(3))
        wx = rng.standard_normal((4096, 4096), dtype=np.float32)
        ww = rng.standard_normal((4096, 4096), dtype=np.float32) * np.float32(0.02)
        wdw = wl.twn_threshold(ww, axis=0)
        waw = rng.uniform(0.5, 1.5, 4096).astype(np.float32)
        xd, awd = to_dev(wx), to_dev(waw)
        cw, _ = B.ternarize_pack(to_dev(ww), garg(-wdw), garg(wdw), want_sum=False)        # S0, offline
        y = torch.empty((4096, 4096), dtype=torch.float32, device=dev)
        wsp = torch.empty(B.lib().rtn_weight_gemm_workspace_bytes(4096, 4096, 4096), dtype=torch.uint8, device=dev)
        wprep = B.weight_gemm_prepare(cw, 4096, 4096)                                       # S0, offline

        def step(timers=None):
            if timers is not None:
                timers[0][0].record()
                timers[0][1].record()
            B.ternary_weight_gemm(xd, None, 4096, 4096, 4096, awd, y_out=y, workspace=wsp, prepared=wprep)
            if timers is not None:
                timers[0][2].record()

        macs_step = 4096 ** 3
        workload = "weight-only ternary GEMM M=N=K=4096 (fp32 activations, ternary weights), fp32 out"
        nlaunch = 1
        layers = [dict(sh=None)]
    else:
        case = wl.gemm_case(4096, 4096, 4096, 0.4, seed=1)
        xa, xw = to_dev(case["xa"]), to_dev(case["xw"])
        cw, sw = B.ternarize_pack(xw, -0.5, 0.5, FMT)                        # S0, offline
        ca = torch.empty((4096, code_row_bytes(4096)), dtype=torch.uint8 if FMT == B.RTN_CODE_FP4 else torch.int8,
                         device=dev)
        sa = torch.empty(4096, dtype=torch.int32, device=dev)
        y = torch.empty((4096, 4096), dtype=torch.float32, device=dev)
        ep = B.Epilogue(garg(case["alpha_a"]), garg(case["beta_a"]), garg(case["alpha_w"]),
                        garg(case["beta_w"]), sa, sw)
        import ctypes as C
        L = B.lib()
        stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        lo, hi = C.c_float(-0.5), C.c_float(0.5)

        def step(timers=None):
            if timers is not None:
                timers[0][0].record()
            rc = L.rtn_ternarize_pack(xa.data_ptr(), B.RTN_ROWS_K_CONTIG, 4096, 4096, 1, 1, C.addressof(lo),
                                      C.addressof(hi), B.RTN_SCALAR, FMT, ca.data_ptr(),
                                      sa.data_ptr(), stream)
            assert rc == 0
            if timers is not None:
                timers[0][1].record()
            B.ternary_gemm(ca, cw, 4096, 4096, 4096, fmt=FMT, ep=ep, y_out=y)
            if timers is not None:
                timers[0][2].record()

        macs_step = 4096 ** 3
        workload = "ternary GEMM M=N=K=4096, P(0)=0.4, fp32 in/out, %s codes" % args.format
        nlaunch = 1
        layers = [dict(sh=None)]

    # ---- timed region: exactly K steps, bracketed by synchronize ------------
    # (the interpreter's cyclic garbage collector is held off while the clock runs, as
    # timeit does: a full collection takes tens of ms with torch's object graph loaded)
    import gc
    gc.collect()
    gc.disable()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # ---- the block-structured variant with the ternarizing epilogue ----------
    blocks_info = None
    if args.workload == "resnet18_ternary_convs":
        for _ in range(args.warmup):
            step_blocks()
        torch.cuda.synchronize()
        tb0 = time.perf_counter()
        for _ in range(args.steps):
            step_blocks()
        torch.cuda.synchronize()
        ms_blocks = (time.perf_counter() - tb0) * 1e3 / args.steps
        for _ in range(args.warmup):
            trunk_forward()
        torch.cuda.synchronize()
        tb0 = time.perf_counter()
        for _ in range(args.steps):
            trunk_forward()
        torch.cuda.synchronize()
        ms_trunk = (time.perf_counter() - tb0) * 1e3 / args.steps
        # algorithmic bytes of the chained pass: the fp32 trunk input once, every code tensor written and read
        # once (twice where the shortcut conv reads it too), filters, fp32 shortcut and block tensors
        nb_ = args.batch
        tr_bytes = nb_ * 56 * 56 * (64 * 4 + code_row_bytes(64))
        for i1, i2, ids in blocks:
            for i_, kind in ((i1, "c1"), (ids, "ds"), (i2, "c2")):
                if i_ is None:
                    continue
                s_ = layers[i_]["sh"]
                cin = nb_ * s_.H * s_.H * code_row_bytes(s_.C) + s_.O * s_.k * s_.k * code_row_bytes(s_.C)
                outs, cout = nb_ * s_.O * s_.OH * s_.OH, nb_ * s_.OH * s_.OH * code_row_bytes(s_.O)
                tr_bytes += cin + (cout if kind == "c1" else outs * 4 if kind == "ds" else outs * 8 + cout)
        blocks_info = {
            "what": "the same 19 convs as 8 residual blocks: conv1 of a block emits the next conv's codes "
                    "(rtn_ternary_conv2d_ternarize), one pack per block input; 8 packs + 19 convs per step",
            "ms_per_step": round(ms_blocks, 4),
            "tmacs": round(macs_step / (ms_blocks * 1e-3) / 1e12, 3),
            "trunk_forward": {
                "what": "the 8 blocks chained as one forward pass: 1 pack, conv1 emits codes, conv2's block-tail "
                        "epilogue adds the shortcut, applies ReLU and writes the fp32 block output and the next "
                        "block's codes; 1 pack + 19 convs per step, residual adds included",
                "ms_per_step": round(ms_trunk, 4),
                "tmacs": round(macs_step / (ms_trunk * 1e-3) / 1e12, 3),
                "roofline": {"bound": "hbm", "achieved": round(tr_bytes / (ms_trunk * 1e-3) / 1e9, 1),
                             "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": round(tr_bytes / (ms_trunk * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                             "bytes_per_step": tr_bytes,
                             "mfma_frac_of_int8_peak": round(2 * macs_step / (ms_trunk * 1e-3) / 1e12 / INT8_PEAK_TOPS,
                                                             4)}}}

    # ---- per-kernel durations with HIP events on the launch stream ---------
    reps = max(3, min(args.steps, 10))
    pack_ms = np.zeros(nlaunch)
    conv_ms = np.zeros(nlaunch)
    for _ in range(reps):
        timers = [[ev(enable_timing=True) for _ in range(3)] for _ in range(nlaunch)]
        step(timers)
        torch.cuda.synchronize()
        for i in range(nlaunch):
            pack_ms[i] += timers[i][0].elapsed_time(timers[i][1])
            conv_ms[i] += timers[i][1].elapsed_time(timers[i][2])
    pack_ms /= reps
    conv_ms /= reps
    gc.enable()

    per_layer = []
    if args.workload == "resnet18_ternary_convs":
        tot_bytes_conv = 0
        for i, l in enumerate(layers):
            sh = l["sh"]
            macs = sh.macs(args.batch)
            Cb = code_row_bytes(sh.C)                               # bytes of a pixel's code row
            in_b = args.batch * sh.H * sh.H * Cb                    # (the conv forms the pixel sums itself)
            w_b = sh.O * sh.k * sh.k * Cb
            out_b = args.batch * sh.O * sh.OH * sh.OH * 4
            conv_bytes = in_b + w_b + out_b
            pack_bytes = args.batch * sh.C * sh.H * sh.H * 4 + args.batch * sh.H * sh.H * (Cb + 4)
            tot_bytes_conv += conv_bytes
            # in-bounds MACs: taps that fall into the zero padding are counted by the dense figure only
            taps = sum(1 for o in range(sh.OH) for k in range(sh.k) if 0 <= o * sh.stride - sh.pad + k < sh.H)
            macs_inb = args.batch * sh.O * sh.C * taps * taps
            # which roof bounds the layer (MACs per algorithmic byte against the ridge of the int8 peak,
            # 2.5e15 MAC/s / 8e12 B/s = 312 MAC/B) and the target that goes with it
            pct_mfma = 100 * 2 * macs / (conv_ms[i] * 1e-3) / 1e12 / INT8_PEAK_TOPS
            pct_hbm = 100 * conv_bytes / (conv_ms[i] * 1e-3) / 1e9 / HBM_PEAK_GBS
            bound = "mfma" if macs / conv_bytes >= 312.0 else "hbm"
            frac, target = (pct_mfma, 50.0) if bound == "mfma" else (pct_hbm, 70.0)
            per_layer.append(dict(
                layer=sh.name, M=args.batch * sh.OH * sh.OH, N=sh.O, K=sh.K,
                conv_us=round(conv_ms[i] * 1e3, 1), pack_us=round(pack_ms[i] * 1e3, 1),
                conv_tops=round(2 * macs / (conv_ms[i] * 1e-3) / 1e12, 1),
                conv_pct_int8_peak=round(pct_mfma, 1),
                conv_gbs=round(conv_bytes / (conv_ms[i] * 1e-3) / 1e9, 0),
                conv_pct_hbm=round(pct_hbm, 1),
                mac_per_byte=round(macs / conv_bytes, 0), bound=bound, frac=round(frac / 100, 3),
                target=target / 100, target_met=bool(frac >= target),
                macs_dense=macs, macs_in_bounds=macs_inb,
                pack_gbs=round(pack_bytes / (pack_ms[i] * 1e-3) / 1e9, 0),
                pack_pct_hbm=round(100 * pack_bytes / (pack_ms[i] * 1e-3) / 1e9 / HBM_PEAK_GBS, 1)))
    conv_total_s = float(conv_ms.sum()) * 1e-3
    achieved_tops = 2 * macs_step / conv_total_s / 1e12
    if args.workload == "resnet18_ternary_convs":
        # The conv stack as a whole sits under the HBM roof: its algorithmic bytes
        # (codes + pixel sums + filters in, fp32 out) take longer at 8 TB/s than its
        # MACs at the int8 matrix-core peak, so that is the roof the dominant kernel
        # is priced against; the matrix-core fraction is reported beside it.
        alg_bytes_launch = tot_bytes_conv / nlaunch
        achieved_gbs = tot_bytes_conv / conv_total_s / 1e9
        traffic = None
        if args.batch == 256 and args.tile < 0 and args.format == "fp4":
            # HBM bytes per k_tmm launch from the FETCH_SIZE / WRITE_SIZE counter passes
            # summarised in profiles/k_tmm_conv_resnet18_b256.md (2 * FETCH_SIZE + WRITE_SIZE,
            # in KiB per dispatch, averaged over the 19 launches of a step)
            traffic = MEASURED_TRAFFIC_BYTES_PER_LAUNCH
        roofline = dict(bound="hbm", kernel="k_tmm (%s MFMA implicit-GEMM conv + fused epilogue)" % args.format,
                        achieved=round(achieved_gbs, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=round(achieved_gbs / HBM_PEAK_GBS, 4), traffic=traffic,
                        traffic_source=MEASURED_TRAFFIC_STAMP if traffic else None,
                        launches_per_step=nlaunch, avg_launch_us=round(conv_total_s / nlaunch * 1e6, 1),
                        bytes_per_launch=round(alg_bytes_launch, 0),
                        mfma_tops=round(achieved_tops, 1), mfma_frac=round(achieved_tops / INT8_PEAK_TOPS, 4))
    elif args.workload == "act_backward":
        gbs = 12.0 * macs_step / conv_total_s / 1e9      # 4 B a + 4 B g read, 4 B dL/da written per element
        roofline = dict(bound="hbm", kernel="k_act_backward (+ k_sum_partials)", achieved=round(gbs, 1),
                        peak=HBM_PEAK_GBS, unit="GB/s", frac=round(gbs / HBM_PEAK_GBS, 4), traffic=None,
                        launches_per_step=nlaunch, avg_launch_us=round(conv_total_s / nlaunch * 1e6, 1),
                        bytes_per_launch=12.0 * macs_step)
    elif args.workload == "weight_backward":
        gbs = 12.0 * macs_step / conv_total_s / 1e9      # 4 B W + 4 B g read, 4 B dL/dW written per element
        roofline = dict(bound="hbm", kernel="k_weight_backward", achieved=round(gbs, 1),
                        peak=HBM_PEAK_GBS, unit="GB/s", frac=round(gbs / HBM_PEAK_GBS, 4), traffic=None,
                        launches_per_step=nlaunch, avg_launch_us=round(conv_total_s / nlaunch * 1e6, 1),
                        bytes_per_launch=round(12.0 * macs_step / nlaunch, 0))
    elif args.workload == "resnet18_weight_only_convs":
        bf16_tflops = 3 * achieved_tops
        roofline = dict(bound="mfma", kernel="activation split + k_tmm (bf16 MFMA implicit-GEMM conv, fp32 accumulate)",
                        achieved=round(bf16_tflops, 1), peak=BF16_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=round(bf16_tflops / BF16_PEAK_TFLOPS, 4), traffic=None,
                        launches_per_step=nlaunch, avg_launch_us=round(conv_total_s / nlaunch * 1e6, 1),
                        flops_per_launch=6 * macs_step / nlaunch,
                        effective_fp32_tflops=round(achieved_tops, 1), fp32_vector_peak_tflops=157.3)
    elif args.workload == "wgemm4096":
        # the call = split kernel + weight conversion + matrix-core GEMM; the GEMM executes three
        # bf16 products per ternary MAC (the three terms of the exact fp32 split)
        bf16_tflops = 3 * achieved_tops
        roofline = dict(bound="mfma", kernel="activation split + k_tmm (bf16 MFMA, fp32 accumulate)",
                        achieved=round(bf16_tflops, 1), peak=BF16_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=round(bf16_tflops / BF16_PEAK_TFLOPS, 4), traffic=None,
                        launches_per_step=nlaunch, avg_launch_us=round(conv_total_s / nlaunch * 1e6, 1),
                        flops_per_launch=6 * macs_step / nlaunch,
                        effective_fp32_tflops=round(achieved_tops, 1), fp32_vector_peak_tflops=157.3)
    else:
        # a contraction is priced against the peak of its own operand type: the FP4 matrix path
        # against 10.1 PFLOP/s, the int8 path against 5.0 POP/s; the fraction of the int8 peak (the
        # stated target's yardstick) is given beside it either way
        peak = FP4_PEAK_TFLOPS if FMT == B.RTN_CODE_FP4 else INT8_PEAK_TOPS
        roofline = dict(bound="mfma", kernel="k_tmm (%s MFMA GEMM + fused epilogue)" % args.format,
                        achieved=round(achieved_tops, 1), peak=peak, unit="TFLOP/s" if FMT == B.RTN_CODE_FP4 else "TOP/s",
                        frac=round(achieved_tops / peak, 4), traffic=None,
                        frac_of_int8_peak=round(achieved_tops / INT8_PEAK_TOPS, 4),
                        launches_per_step=nlaunch, avg_launch_us=round(conv_total_s / nlaunch * 1e6, 1),
                        ops_per_launch=2 * macs_step / nlaunch)

    # ---- CPU baseline: the oracle, as it stands, on a bounded sample --------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import rtn_oracle as orc
        n_img = args.cpu_images
        t_cpu, macs_cpu = 0.0, 0
        if args.workload == "resnet18_ternary_convs":
            for i, sh in enumerate(wl.resnet18_ternary_layers()):
                case = wl.conv_case(sh, batch=n_img, seed=100 + i, per_channel=True, bn=True)
                c0 = time.perf_counter()
                ta = orc.ternarize(case["x"], -case["delta_a"], case["delta_a"])
                tw = orc.ternarize(case["w"], -case["delta_w"], case["delta_w"])
                D = orc.conv_acc(ta, tw, sh.stride, sh.pad)
                Sa, Sw, Kv = orc.conv_sums(ta, tw, sh.stride, sh.pad, True)
                orc.conv_epilogue(D, Sa, Sw, Kv, case["alpha_a"], case["beta_a"], case["alpha_w"],
                                  case["beta_w"], relu=True, bn_scale=case["bn_scale"], bn_shift=case["bn_shift"])
                t_cpu += time.perf_counter() - c0
                macs_cpu += sh.macs(n_img)
            sample = "all 19 layers, %d images each (of %d)" % (n_img, args.batch)
        elif args.workload == "act_backward":
            c0 = time.perf_counter()
            orc.act_backward(ba_, bg_, -0.5, 0.5, 0.9)
            t_cpu = time.perf_counter() - c0
            macs_cpu = nel
            sample = "the whole tensor (%d elements), single thread as the oracle is written" % nel
        elif args.workload == "weight_backward":
            c0 = time.perf_counter()
            for l in wb:
                hw, hg, hk, hb, ha = l["host"]
                orc.weight_backward(hw, hg, -0.5, 0.5, hk, hb, ha)
            t_cpu = time.perf_counter() - c0
            macs_cpu = macs_step
            sample = "all 19 weight tensors (%d elements), single thread as the oracle is written" % macs_step
        elif args.workload == "resnet18_weight_only_convs":
            n_img = max(1, args.cpu_images // 8)
            for i, sh in enumerate(wl.resnet18_ternary_layers()):
                case = wl.conv_case(sh, batch=n_img, seed=100 + i, per_channel=True, bn=True)
                c0 = time.perf_counter()
                tw = orc.ternarize(case["w"], -case["delta_w"], case["delta_w"])
                orc.wconv(case["x"], tw, sh.stride, sh.pad, case["alpha_w"], relu=True,
                          bn_scale=case["bn_scale"], bn_shift=case["bn_shift"])
                t_cpu += time.perf_counter() - c0
                macs_cpu += sh.macs(n_img)
            sample = "all 19 layers, %d images each (of %d)" % (n_img, args.batch)
        elif args.workload == "wgemm4096":
            rows = np.arange(0, 4096, 4096 // 64, dtype=np.int64)
            c0 = time.perf_counter()
            tw = orc.ternarize(ww, -wdw, wdw)
            orc.wgemm(wx[rows], tw, waw)
            t_cpu = time.perf_counter() - c0
            macs_cpu = rows.size * 4096 * 4096
            sample = "64 of 4096 output rows, all columns"
        else:
            rows = np.arange(0, 4096, 4096 // 64, dtype=np.int64)
            c0 = time.perf_counter()
            ta = orc.ternarize(case["xa"], -0.5, 0.5)
            tw = orc.ternarize(case["xw"], -0.5, 0.5)
            D = orc.gemm_acc_rows(ta, tw, rows)
            orc.gemm_epilogue(D, 4096, orc.row_sums(ta)[rows], orc.row_sums(tw), case["alpha_a"][rows],
                              case["beta_a"][rows], case["alpha_w"], case["beta_w"])
            t_cpu = time.perf_counter() - c0
            macs_cpu = rows.size * 4096 * 4096
            sample = "64 of 4096 output rows, all columns"
        cpu = dict(value=round(macs_cpu / t_cpu / 1e12, 6), unit="TMAC/s",
                   cores=1 if args.workload in ("act_backward", "weight_backward") else orc.num_threads(),
                   kind="oracle", sample=sample, seconds=round(t_cpu, 2))

    value = macs_step / (ms_per_step * 1e-3) / 1e12
    out = {
        "metric": "effective ternary MAC/s (dense MAC count, S1+S2+S3+S4 per layer), ResNet-18 ternary layers"
        if args.workload == "resnet18_ternary_convs" else
        ("elements/s (in units of 1e12), backward of the reparameterized ternary activation"
         if args.workload == "act_backward" else
         "elements/s (in units of 1e12), backward of the ternary weight transform"
         if args.workload == "weight_backward" else
         "effective MAC/s, weight-only ternary GEMM" if args.workload == "wgemm4096"
         else ("effective MAC/s, weight-only ternary convs of ResNet-18"
               if args.workload == "resnet18_weight_only_convs" else "effective ternary MAC/s, ternary GEMM")),
        "value": round(value, 3), "unit": "TMAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16x3" if args.workload in ("wgemm4096", "resnet18_weight_only_convs") else
        ("f32" if args.workload in ("act_backward", "weight_backward") else args.format), "data": "synthetic",
        "config": {"workload": workload, "batch": args.batch, "tile": args.tile, "format": args.format},
        "tops": round(2 * value, 1), "pct_int8_mfma_peak": round(100 * 2 * value / INT8_PEAK_TOPS, 2),
        "contraction_only": {"tmacs": round(macs_step / conv_total_s / 1e12, 3),
                             "pct_int8_mfma_peak": round(100 * achieved_tops / INT8_PEAK_TOPS, 2),
                             "ms": round(conv_total_s * 1e3, 4)},
        "pack_only_ms": round(float(pack_ms.sum()), 4),
        "roofline": roofline, "cpu_baseline": cpu, "fused_blocks": blocks_info, "layers": per_layer,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
