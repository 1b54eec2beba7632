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
BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
HBM_PEAK_GBS = 8000.0
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this file's default run (see profiles/)
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = 129.6e6


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--workload", default="resnet18_ternary_convs",
                    choices=["resnet18_ternary_convs", "gemm4096", "wgemm4096", "resnet18_weight_only_convs",
                             "act_backward", "weight_backward", "gemm_sweep"])
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
                    for fmt, name in ((B.RTN_CODE_I8, "mfma_i8"), (B.RTN_CODE_BITPLANE, "popcount")):
                        ca, sa = B.ternarize_pack(xa, -0.5, 0.5, fmt)
                        cw, sw = B.ternarize_pack(xw, -0.5, 0.5, fmt)
                        ep = B.Epilogue(garg(case["alpha_a"]), garg(case["beta_a"]), garg(case["alpha_w"]),
                                        garg(case["beta_w"]), sa, sw)
                        y = torch.empty((M, NK), dtype=torch.float32, device=dev)
                        reps = 5 if name == "mfma_i8" else 2
                        for _ in range(2):
                            B.ternary_gemm(ca, cw, M, NK, NK, fmt=fmt, ep=ep, y_out=y)
                        e0, e1, e2 = ev(enable_timing=True), ev(enable_timing=True), ev(enable_timing=True)
                        e0.record()
                        for _ in range(reps):
                            B.ternary_gemm(ca, cw, M, NK, NK, fmt=fmt, ep=ep, y_out=y)
                        e1.record()
                        for _ in range(reps):
                            B.ternarize_pack(xa, -0.5, 0.5, fmt)
                        e2.record()
                        torch.cuda.synchronize()
                        us, pus = e0.elapsed_time(e1) * 1e3 / reps, e1.elapsed_time(e2) * 1e3 / reps
                        macs = float(M) * NK * NK
                        rows.append(dict(M=M, N=NK, K=NK, p_zero=p0, path=name, gemm_us=round(us, 1),
                                         pack_us=round(pus, 1), tmacs=round(macs / us / 1e6, 1),
                                         pct_int8_mfma_peak=round(100 * 2 * macs / us / 1e6 / INT8_PEAK_TOPS, 1)))
                        if name == "mfma_i8":
                            tot_macs += macs
                            tot_s += (us + pus) * 1e-6
                        del ca, cw, sa, sw, y, ep
                    del xa, xw, case
        mf = [r for r in rows if r["path"] == "mfma_i8"]
        best = max(mf, key=lambda r: r["tmacs"])
        print(json.dumps({
            "metric": "effective ternary MAC/s, ternary GEMM sweep (pack + contraction + epilogue, matrix-core path)",
            "value": round(tot_macs / tot_s / 1e12, 3), "unit": "TMAC/s", "n_gpus": 1, "steps": 5, "warmup": 2,
            "ms_per_step": round(tot_s * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "i8", "data": "synthetic",
            "config": {"workload": "ternary GEMM sweep: M in {8192,16384} x N=K in {4096,8192} x P(0) in {0.2,0.5,0.8}, "
                                   "int8 matrix-core and bit-plane popcount paths"},
            "roofline": {"bound": "mfma", "kernel": "k_tmm (int8 MFMA GEMM + fused epilogue), best point",
                         "achieved": round(2 * best["tmacs"], 1), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                         "frac": round(2 * best["tmacs"] / INT8_PEAK_TOPS, 4), "traffic": None},
            "cpu_baseline": None, "sweep": rows}))
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
        workload = "ResNet-18 ternary conv stack (19 layers), batch %d, fp32 NCHW in/out" % args.batch
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
        # the same 19 layer shapes with ternary weights and fp32 activations (one call per layer:
        # activation split, weight copy, epilogue table, bf16 matrix-core conv)
        wlayers = []
        for i, sh in enumerate(wl.resnet18_ternary_layers()):
            case = wl.conv_case(sh, batch=args.batch, seed=100 + i, per_channel=True, bn=True)
            dw = np.asarray(case["delta_w"])
            cw, _ = B.ternarize_pack(to_dev(case["w"]), garg(-dw), garg(dw), want_sum=False)    # S0, offline
            wlayers.append(dict(sh=sh, x=to_dev(case["x"]), cw=cw, aw=to_dev(case["alpha_w"]),
                                bs=to_dev(case["bn_scale"]), bh=to_dev(case["bn_shift"]),
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
                B.ternary_weight_conv2d(l["x"], l["cw"], sh.O, sh.k, sh.k, sh.stride, sh.pad, l["aw"], relu=True,
                                        bn_scale=l["bs"], bn_shift=l["bh"], y_out=l["y"], workspace=l["ws"])
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

        def step(timers=None):
            if timers is not None:
                timers[0][0].record()
                timers[0][1].record()
            B.ternary_weight_gemm(xd, cw, 4096, 4096, 4096, awd, y_out=y, workspace=wsp)
            if timers is not None:
                timers[0][2].record()

        macs_step = 4096 ** 3
        workload = "weight-only ternary GEMM M=N=K=4096 (fp32 activations, ternary weights), fp32 out"
        nlaunch = 1
        layers = [dict(sh=None)]
    else:
        case = wl.gemm_case(4096, 4096, 4096, 0.4, seed=1)
        xa, xw = to_dev(case["xa"]), to_dev(case["xw"])
        cw, sw = B.ternarize_pack(xw, -0.5, 0.5)                             # S0, offline
        ca = torch.empty((4096, 4096), dtype=torch.int8, device=dev)
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
                                      C.addressof(hi), B.RTN_SCALAR, B.RTN_CODE_I8, ca.data_ptr(),
                                      sa.data_ptr(), stream)
            assert rc == 0
            if timers is not None:
                timers[0][1].record()
            B.ternary_gemm(ca, cw, 4096, 4096, 4096, ep=ep, y_out=y)
            if timers is not None:
                timers[0][2].record()

        macs_step = 4096 ** 3
        workload = "ternary GEMM M=N=K=4096, P(0)=0.4, fp32 in/out"
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
                "tmacs": round(macs_step / (ms_trunk * 1e-3) / 1e12, 3)}}

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
        if args.batch == 256 and args.tile < 0:
            # HBM bytes per k_tmm launch from the FETCH_SIZE / WRITE_SIZE counter passes
            # summarised in profiles/k_tmm_conv_resnet18_b256.md (2 * FETCH_SIZE + WRITE_SIZE,
            # in KiB per dispatch, averaged over the 19 launches of a step)
            traffic = MEASURED_TRAFFIC_BYTES_PER_LAUNCH
        roofline = dict(bound="hbm", kernel="k_tmm (int8 MFMA implicit-GEMM conv + fused epilogue)",
                        achieved=round(achieved_gbs, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=round(achieved_gbs / HBM_PEAK_GBS, 4), traffic=traffic,
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
        roofline = dict(bound="mfma", kernel="k_tmm (int8 MFMA GEMM + fused epilogue)",
                        achieved=round(achieved_tops, 1), peak=INT8_PEAK_TOPS, unit="TOP/s",
                        frac=round(achieved_tops / INT8_PEAK_TOPS, 4), traffic=None,
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
        ("f32" if args.workload in ("act_backward", "weight_backward") else "i8"), "data": "synthetic",
        "config": {"workload": workload, "batch": args.batch, "tile": args.tile},
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
