#!/usr/bin/env python3
"""Benchmark of the NVFP4 quantized linear layer hot path on one MI355X.

A step is one pass of the whole path - forward product, input-gradient product, weight-gradient product, with all
six quantizations (maxima, quantizers, re-quantizers: the "full overhead" of the paper's single-linear figure) -
over every linear layer of the workload, on synthetic inputs that are resident in HBM before the clock starts.
The default workload is the largest single-GPU one: the square M = N = K = 8192 layer with outlier channels.

Prints ONE JSON line.  `value` = algorithmic flops of a step (3 * sum 2*N*D*C) / wall time.
`roofline` describes the dominant kernel (the packed-operand GEMM) measured with events on the launch stream;
`cpu_baseline` times the CPU oracle on a bounded sample of the same workload; `extras` carries the other
workloads' steps, the quantizer bandwidth lines on the 8192 x 8192 stress tensor and the product alone.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_F16_PEAK_TFLOPS = 2500.0     # MI355X dense FP16/BF16 MFMA, vendor figure
HBM_PEAK_GBS = 8000.0             # MI355X HBM3E, vendor figure
DEFAULT_WORKLOAD = "cfg5_square8192"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps; the default is long enough (tens of ms) for the GPU clocks to settle")
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--outer", default="tensor", choices=["tensor", "block128"],
                    help="outer scale of every operand: per tensor, or the paper's 1 x 128 blocks")
    ap.add_argument("--rht", action="store_true",
                    help="random Hadamard transform (block 16) on both operands of both backward products; needs --outer block128")
    ap.add_argument("--outctl", type=int, default=0, metavar="CHANNELS",
                    help="outlier-control split layer: this many input channels of every linear (those with the largest "
                         "activation norm; a multiple of 128) stay in bf16")
    ap.add_argument("--no-extras", action="store_true", help="skip the side measurements (other workloads, quantizer bandwidth)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device copy of 1 GiB five times (reference point for HBM byte counters)")
    ap.add_argument("--square-gemm", type=int, default=0, metavar="REPS",
                    help="only run the 8192^3 product on pre-quantized operands REPS times (for counter profiles)")
    ap.add_argument("--quantizers", type=int, default=0, metavar="REPS",
                    help="only run each quantizer of the 8192 x 8192 stress tensor REPS times (for counter profiles)")
    return ap.parse_args()


def dev_bf16(torch, np, bits, dev):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)


class Workload:
    """Resident inputs, contexts, outputs and workspaces of every linear of one workload, and its step."""

    def __init__(self, tj, wl, np, torch, dev, name, outer, rht=False, n_hp=0):
        B = tj.binding
        self.tj, self.B, self.name, self.outer, self.rht, self.n_hp = tj, B, name, outer, rht, n_hp
        self.layers = []
        for li, (lname, N, D, C, seed, kind) in enumerate(wl.config_linears(name)):
            Xb, Wb, dYb = wl.linear_inputs(N, D, C, seed, kind)
            L = dict(name=lname, N=N, D=D, C=C, li=li, X=dev_bf16(torch, np, Xb, dev), W=dev_bf16(torch, np, Wb, dev),
                     dY=dev_bf16(torch, np, dYb, dev))
            if n_hp:
                Xl, Wl, Xh, Wh, _ = wl.outlier_channel_split(Xb, Wb, n_hp)
                L.update(X=dev_bf16(torch, np, Xl, dev), W=dev_bf16(torch, np, Wl, dev), Xh=dev_bf16(torch, np, Xh, dev),
                         Wh=dev_bf16(torch, np, Wh, dev))
                D = D - n_hp
                L["outs"] = [torch.empty(sh, dtype=torch.bfloat16, device=dev) for sh in ((N, D), (N, n_hp), (C, D), (C, n_hp))]
                L["ws"] = tj.alloc_workspace(max(B.lib().nvfp4_outctl_workspace_bytes(b, N, D, n_hp, C, outer, B.OUT_BF16)
                                                 for b in (0, 1)))
            L["Xq"] = tj.alloc_nvfp4(N, D, outer)
            L["Wq"] = tj.alloc_nvfp4(C, D, outer)
            L["Y"] = torch.empty((N, C), dtype=torch.bfloat16, device=dev)
            L["dX"] = torch.empty((N, D), dtype=torch.bfloat16, device=dev)
            L["dW"] = torch.empty((C, D), dtype=torch.bfloat16, device=dev)
            if not n_hp:
                nbytes = max(tj.workspace_bytes(op, N, D, C, outer) for op in (B.OP_LINEAR_FWD, B.OP_LINEAR_BWD))
                L["ws"] = tj.alloc_workspace(nbytes)
            self.layers.append(L)
        self.flops = wl.config_flops(name)
        # lower bound of a step from the two rooflines, per linear: bf16 reads of X, W, dY, packed operands written
        # and read once each (Q1..Q6), bf16 writes of Y, dX, dW
        self.t_min = 0.0
        for L in self.layers:
            N, D, C = L["N"], L["D"], L["C"]
            nbytes = 2.0 * (N * D + C * D + N * C) + 2 * 0.5625 * (N * D + C * D) * 2 + 2 * 0.5625 * (2 * N * C) \
                + 2.0 * (N * C + N * D + C * D)
            self.t_min += max(3 * 2.0 * N * D * C / (MFMA_F16_PEAK_TFLOPS * 1e12), nbytes / (HBM_PEAK_GBS * 1e9))

    def step(self, sr_seed):
        tj, B = self.tj, self.B
        if self.n_hp:
            for L in self.layers:
                tj.outctl_fwd(L["X"], L["W"], L["Xh"], L["Wh"], B.OUT_BF16, outer=self.outer, Y=L["Y"], Xq=L["Xq"], Wq=L["Wq"],
                              ws=L["ws"])
            for L in reversed(self.layers):
                tj.outctl_bwd(L["dY"], L["Xq"], L["Wq"], L["Xh"], L["Wh"], sr_seed, L["li"], B.OUT_BF16, rht=self.rht, ws=L["ws"],
                              outs=L["outs"])
            return
        for L in self.layers:
            tj.linear_fwd(L["X"], L["W"], B.OUT_BF16, Y=L["Y"], Xq=L["Xq"], Wq=L["Wq"], ws=L["ws"], outer=self.outer)
        for L in reversed(self.layers):
            tj.linear_bwd(L["dY"], L["Xq"], L["Wq"], sr_seed, L["li"], B.OUT_BF16, dX=L["dX"], dW=L["dW"], ws=L["ws"], rht=self.rht)

    def settle(self, torch, seconds):
        """Untimed steps for about `seconds` before the warm-up proper: a cold chip needs a few hundred milliseconds of
        this load before its clocks stop moving, more than a handful of warm-up steps last."""
        t0 = time.perf_counter()
        n = 0
        while time.perf_counter() - t0 < seconds:
            self.step(5000 + n)
            n += 1
            if n % 8 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        return n

    def time_steps(self, torch, steps, warmup):
        import gc
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        gc.collect()
        gc.disable()                                      # no collector pause inside the timed region
        try:
            t0 = time.perf_counter()
            for i in range(steps):
                self.step(1000 + i)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
        finally:
            gc.enable()
        return dt * 1e3 / steps


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not provided."
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calibration:
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": src.numel() * 4, "copy_calibration_bytes_written": src.numel() * 4,
                          "launches": 5}))
        return

    import paper_2510_27527_amd as tj
    import workloads as wl
    B = tj.binding
    B.lib()
    outer = B.OUTER_TENSOR if args.outer == "tensor" else B.OUTER_BLOCK128

    if args.square_gemm:
        n = 8192
        gen = torch.Generator(device=dev).manual_seed(0)
        ops = []
        for _ in range(2):
            t = tj.alloc_nvfp4(n, n, outer)
            t.codes.copy_(torch.randint(0, 256, t.codes.shape, dtype=torch.uint8, device=dev, generator=gen))
            t.scales.copy_(torch.randint(0x30, 0x40, t.scales.shape, dtype=torch.uint8, device=dev, generator=gen))
            t.gscale.fill_(1.0)
            ops.append(t)
        out = torch.empty((n, n), dtype=torch.bfloat16, device=dev)
        ws = tj.alloc_workspace(16)
        for _ in range(args.square_gemm):
            tj.gemm_nt(ops[0], ops[1], B.OUT_BF16, out=out, ws=ws)
        torch.cuda.synchronize()
        print(json.dumps({"square_gemm_launches": args.square_gemm, "flops_per_launch": 2.0 * n ** 3}))
        return

    if args.quantizers:
        res = quantizer_lines(tj, wl, np, torch, dev, warm=3, reps=args.quantizers)
        print(json.dumps({"quantizer_launches_each": args.quantizers + 3, "lines": res}))
        return

    if args.rht and outer != B.OUTER_BLOCK128:
        print("bench.py: --rht needs --outer block128", file=sys.stderr)
        sys.exit(2)
    w = Workload(tj, wl, np, torch, dev, args.workload, outer, args.rht, args.outctl)
    settle_steps = w.settle(torch, 0.3)
    ms_per_step = w.time_steps(torch, args.steps, args.warmup)
    value = w.flops / (ms_per_step * 1e-3) / 1e12
    layers = w.layers

    # ---- dominant kernel: the packed GEMM (gemm_nt_kernel), on the operands the step just produced ----------
    # The three products of every linear are launched back to back between two events recorded on the launch
    # stream; duration per launch = elapsed / launches (a product whose reduction is split over workgroups is still
    # one launch of this kernel).
    gemm_jobs = []
    for L in layers:
        dYq = tj.quantize(L["dY"], 0, B.ROUND_SR, seed=1, tensor_id=L["li"] * 16 + 3, outer=outer)
        Wq2 = tj.quantize(L["Wq"], 1, B.ROUND_SR, seed=1, tensor_id=L["li"] * 16 + 4, outer=outer)
        dYq2 = tj.quantize(L["dY"], 1, B.ROUND_SR, seed=1, tensor_id=L["li"] * 16 + 5, outer=outer)
        Xq2 = tj.quantize(L["Xq"], 1, B.ROUND_SR, seed=1, tensor_id=L["li"] * 16 + 6, outer=outer)
        for A, Bt, out in ((L["Xq"], L["Wq"], L["Y"]), (dYq, Wq2, L["dX"]), (dYq2, Xq2, L["dW"])):
            nws = tj.workspace_bytes(B.OP_GEMM, A.rows, A.K, Bt.rows, outer)
            gemm_jobs.append((A, Bt, out, tj.alloc_workspace(max(nws, 16)), 2.0 * A.rows * Bt.rows * A.K))
    for _ in range(10):
        for A, Bt, out, ws, _f in gemm_jobs:
            tj.gemm_nt(A, Bt, B.OUT_BF16, out=out, ws=ws)
    torch.cuda.synchronize()
    reps = max(3, min(args.steps, 50))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        for A, Bt, out, ws, _f in gemm_jobs:
            tj.gemm_nt(A, Bt, B.OUT_BF16, out=out, ws=ws)
    e1.record()
    torch.cuda.synchronize()
    gemm_ms = e0.elapsed_time(e1) / (reps * len(gemm_jobs))
    gemm_flops = sum(j[4] for j in gemm_jobs) / len(gemm_jobs)
    achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12
    traffic = None    # HBM bytes per launch from the committed rocprofv3 counter summary of this same command
    tpath = os.path.join(ROOT, "profiles", "gemm_nt_%s_hbm_traffic.txt" % args.workload)
    if outer == B.OUTER_TENSOR and os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch="):
                traffic = int(line.split("=")[1])
    roofline = {"kernel": "gemm_nt_kernel", "bound": "mfma", "achieved": round(achieved, 2),
                "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / MFMA_F16_PEAK_TFLOPS, 4),
                "traffic": traffic, "avg_launch_ms": round(gemm_ms, 5), "flops_per_launch": gemm_flops,
                "launches_timed": reps * len(gemm_jobs),
                "note": "mean over the %d products of a step (2*M*N*K flops each)" % len(gemm_jobs)}
    del gemm_jobs

    out = {"metric": "nvfp4_linear_fwd_bwd_tflops", "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "settle_steps_before_warmup": settle_steps, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp4xfp4->f32 (fp16 MFMA)",
           "data": "synthetic",
           "config": {"workload": args.workload, "tokens": layers[0]["N"],
                      "linears": [[L["name"], L["D"], L["C"]] for L in layers],
                      "outer_scale": "per-tensor" if outer == B.OUTER_TENSOR else "1x128 blocks",
                      "rht": bool(args.rht), "bf16_outlier_channels": args.outctl,
                      "flops_per_step": w.flops},
           "frac_of_mfma_peak": round(value / MFMA_F16_PEAK_TFLOPS, 4),
           "frac_of_roofline_lower_bound": round(w.t_min * 1e3 / ms_per_step, 4),
           "roofline": roofline}
    del w, layers

    if not args.no_extras:
        out["extras"] = extras(tj, wl, np, torch, dev, args.workload, outer)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(wl, np, args.workload)
    print(json.dumps(out))


def time_events(torch, fn, reps):
    """Duration of one call of fn: reps back-to-back calls in batches of at most 20, each batch bracketed by two events
    on the launch stream; the median batch (a host-side hiccup - the collector, an allocator call - in one batch does
    not reach the figure).  Used for the side lines only; the headline step is timed whole, by the wall clock."""
    import gc
    batches = []
    done = 0
    gc.collect()
    gc.disable()
    try:
        while done < reps:
            nb = min(20, reps - done)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(nb):
                fn(done + i)
            e1.record()
            torch.cuda.synchronize()
            batches.append(e0.elapsed_time(e1) / nb)
            done += nb
    finally:
        gc.enable()
    batches.sort()
    return batches[len(batches) // 2]


def quantizer_lines(tj, wl, np, torch, dev, warm=300, reps=200):
    """Quantizer GB/s on the 8192 x 8192 stress tensor.  Sources rotate through buffers that together exceed the
    256 MB last-level cache (four bf16 copies = 536 MB; eight packed copies = 302 MB), so the bytes come from HBM."""
    B = tj.binding
    res = {}
    R = Cc = 8192
    cfg = wl.CONFIGS["cfg4_quant_stress"]
    bits = wl.student_t_bf16((R, Cc), cfg["nu"], cfg["scale"], cfg["seed"])
    bufs = [dev_bf16(torch, np, bits, dev)]
    for _ in range(3):
        bufs.append(bufs[0].clone())
    outs = [tj.alloc_nvfp4(R, Cc) for _ in range(2)]
    outs128 = [tj.alloc_nvfp4(R, Cc, B.OUTER_BLOCK128, with_amax=False) for _ in range(2)]
    ws = tj.alloc_workspace(tj.workspace_bytes(B.OP_QUANTIZE, R, Cc, 0))
    amax = tj.amax_bf16(bufs[0], ws)
    alg_bytes = R * Cc * 2 + R * Cc // 2 + R * Cc // 16 + 4
    dual_bytes = R * Cc * 2 + 2 * (R * Cc // 2 + R * Cc // 16) + 8
    cases = {
        "row_rtn_amax_given": (alg_bytes, lambda i: tj.quantize(bufs[i % 4], 0, B.ROUND_RTN, outs[i % 2], amax_in=amax, ws=ws)),
        "row_rtn_with_amax_pass": (alg_bytes, lambda i: tj.quantize(bufs[i % 4], 0, B.ROUND_RTN, outs[i % 2], ws=ws)),
        "row_sr_amax_given": (alg_bytes, lambda i: tj.quantize(bufs[i % 4], 0, B.ROUND_SR, outs[i % 2], seed=7, amax_in=amax, ws=ws)),
        "col_sr_amax_given": (alg_bytes, lambda i: tj.quantize(bufs[i % 4], 1, B.ROUND_SR, outs[i % 2], seed=7, amax_in=amax, ws=ws)),
        "col_sr_with_amax_pass": (alg_bytes, lambda i: tj.quantize(bufs[i % 4], 1, B.ROUND_SR, outs[i % 2], seed=7, ws=ws)),
        # the paper's own outer scale (1 x 128 blocks) needs no maximum pass at all
        "row_rtn_block128_single_pass": (alg_bytes, lambda i: tj.quantize(bufs[i % 4], 0, B.ROUND_RTN, outs128[i % 2],
                                                                          outer=B.OUTER_BLOCK128, ws=ws)),
        "row_sr_block128_single_pass": (alg_bytes, lambda i: tj.quantize(bufs[i % 4], 0, B.ROUND_SR, outs128[i % 2], seed=7,
                                                                         outer=B.OUTER_BLOCK128, ws=ws)),
        "col_sr_block128_single_pass": (alg_bytes, lambda i: tj.quantize(bufs[i % 4], 1, B.ROUND_SR, outs128[i % 2], seed=7,
                                                                         outer=B.OUTER_BLOCK128, ws=ws)),
        "row_sr_block128_rht": (alg_bytes, lambda i: tj.quantize(bufs[i % 4], 0, B.ROUND_SR, outs128[i % 2], seed=7,
                                                                 outer=B.OUTER_BLOCK128, ws=ws, rht_id=7)),
        "col_sr_block128_rht": (alg_bytes, lambda i: tj.quantize(bufs[i % 4], 1, B.ROUND_SR, outs128[i % 2], seed=7,
                                                                 outer=B.OUTER_BLOCK128, ws=ws, rht_id=0)),
        # both backward operands of one tensor from a single read: 2 B in + 2 x 0.5625 B out per element
        "dual_row_col_sr_amax_given": (dual_bytes, lambda i: tj.quantize_dual(
            bufs[i % 4], B.ROUND_SR, outs[0], outs[1], seed=7, tensor_id_row=3, tensor_id_col=5, amax_in=amax, ws=ws)),
    }
    for name, (nbytes, fn) in cases.items():
        try:
            for i in range(warm):                           # long enough for the clocks to settle
                fn(i)
        except B.NVFP4Error as e:                           # a combination this build does not provide
            res["quant_8192x8192_" + name] = {"error": str(e)}
            continue
        torch.cuda.synchronize()
        ms = time_events(torch, fn, reps)
        gbs = nbytes / (ms * 1e-3) / 1e9
        res["quant_8192x8192_" + name] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    del bufs
    # re-quantization of a packed tensor (Q4 / Q6): 0.5625 B in + 0.5625 B out per element
    srcs = [outs[0]]
    tj.quantize(dev_bf16(torch, np, bits, dev), 0, B.ROUND_RTN, srcs[0], ws=ws)
    for _ in range(7):
        t = tj.alloc_nvfp4(R, Cc)
        for a, b in ((t.codes, srcs[0].codes), (t.scales, srcs[0].scales), (t.gscale, srcs[0].gscale), (t.amax_deq, srcs[0].amax_deq)):
            a.copy_(b)
        srcs.append(t)
    dsts = [tj.alloc_nvfp4(Cc, R) for _ in range(2)]
    fn = lambda i: tj.quantize(srcs[i % 8], 1, B.ROUND_SR, dsts[i % 2], seed=7, tensor_id=i, ws=ws)
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    ms = time_events(torch, fn, reps)
    gbs = (R * Cc * 9 // 8 + 8) / (ms * 1e-3) / 1e9
    res["requant_col_sr_8192x8192"] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    return res


def osci_lines(tj, torch, dev):
    """OsciReset kernels on an 8192 x 8192 binary32 weight (1 GiB of state: larger than the last-level cache):
    statistics step 28 B per weight (W, W', dist_M, dist_Q read; W', dist_M, dist_Q written), reset up to 16 B per weight."""
    n = 8192
    gen = torch.Generator(device=dev).manual_seed(1)
    W = torch.randn((n, n), device=dev, generator=gen) * 0.02
    Wp, dm, dq = torch.empty_like(W), torch.empty_like(W), torch.empty_like(W)
    tj.osci_update(W, Wp, dm, dq, 0)
    W2 = W + torch.randn((n, n), device=dev, generator=gen) * 1e-4
    res = {}
    fn = lambda i: tj.osci_update(W2 if i % 2 == 0 else W, Wp, dm, dq, 1 + i)
    for i in range(20):
        fn(i)
    torch.cuda.synchronize()
    ms = time_events(torch, fn, 40)
    gbs = 28.0 * n * n / (ms * 1e-3) / 1e9
    res["osci_update_8192x8192"] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    cnt = torch.zeros(1, dtype=torch.int64, device=dev)
    fn = lambda i: tj.osci_suppress(W, dm, dq, 8.0, cnt)
    for i in range(10):
        fn(i)
    torch.cuda.synchronize()
    ms = time_events(torch, fn, 40)
    gbs = 16.0 * n * n / (ms * 1e-3) / 1e9         # reads of W, dist_M, dist_Q, and (worst case, as here: nearly every
                                                    # weight is over the threshold) W written back
    res["osci_suppress_8192x8192"] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    # memory-efficient statistics (Appendix Alg. 3) on the 5 % of the weights closest to a rounding threshold: the
    # selection reads W five times (three radix digits, count, emit); a later step reads W once (4 B per weight) and
    # moves 36 B per tracked weight
    del Wp, dm, dq
    k = n * n // 20
    st = tj.osci_select(W, k)
    torch.cuda.synchronize()
    ms = time_events(torch, lambda i: tj.osci_select(W, k), 5)
    res["osci_select_top5pct_8192x8192"] = {"ms": round(ms, 4), "GB/s": round(5 * 4.0 * n * n / (ms * 1e-3) / 1e9, 1)}
    fn = lambda i: tj.osci_update_sparse(W2 if i % 2 == 0 else W, *st)
    for i in range(5):
        fn(i)
    torch.cuda.synchronize()
    ms = time_events(torch, fn, 20)
    gbs = (4.0 * n * n + 36.0 * k) / (ms * 1e-3) / 1e9
    res["osci_update_top5pct_8192x8192"] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    return res


def extras(tj, wl, np, torch, dev, headline, outer):
    """Side measurements named by the metric: the steps of the other workloads, the quantizer GB/s on the 8192 x 8192
    stress tensor and the square 8192^3 product alone."""
    B = tj.binding
    res = {}
    for name, steps, warmup in (("cfg1_single", 200, 50), ("cfg2_block768", 100, 30), ("cfg3_block1024", 50, 15),
                                ("cfg5_square8192", 30, 10)):
        if name == headline:
            continue
        w = Workload(tj, wl, np, torch, dev, name, outer)
        ms = w.time_steps(torch, steps, warmup)
        tf = w.flops / (ms * 1e-3) / 1e12
        res["step_" + name] = {"ms": round(ms, 4), "TFLOP/s": round(tf, 1), "frac_mfma_peak": round(tf / MFMA_F16_PEAK_TFLOPS, 4),
                               "frac_of_roofline_lower_bound": round(w.t_min * 1e3 / ms, 4)}
        del w
    res.update(quantizer_lines(tj, wl, np, torch, dev))

    res.update(osci_lines(tj, torch, dev))

    # the square product alone, on pre-quantized operands: M = N = K = 8192
    n = 8192
    Xb, Wb, _dYb = wl.linear_inputs(n, n, n, wl.CONFIGS["cfg5_square8192"]["seed"], "square")
    Y, Xq, Wq = tj.linear_fwd(dev_bf16(torch, np, Xb, dev), dev_bf16(torch, np, Wb, dev), outer=outer)
    gws = tj.alloc_workspace(max(tj.workspace_bytes(B.OP_GEMM, n, n, n, outer), 16))
    fn = lambda i: tj.gemm_nt(Xq, Wq, B.OUT_BF16, out=Y, ws=gws)
    for i in range(150):                               # ~0.1 s: the clocks settle under matrix load
        fn(i)
    torch.cuda.synchronize()
    ms = time_events(torch, fn, 50)
    tf = 2.0 * n ** 3 / (ms * 1e-3) / 1e12
    res["gemm_8192_cubed"] = {"ms": round(ms, 4), "TFLOP/s": round(tf, 1), "frac_mfma_peak": round(tf / MFMA_F16_PEAK_TFLOPS, 4)}
    return res


def cpu_baseline(wl, np, workload):
    """The CPU oracle, as it stands, on a bounded sample of the workload: every linear on a slab of its tokens (all of
    them for the small workloads) - all six quantizations and the three float64 products - on all host threads.
    Weights are quantized whole (they do not shrink with the token slab)."""
    import oracle
    oracle.lib()
    flops = 0.0
    names = []
    dt = 0.0
    budget = 5e11                                      # flops of the whole sample: roughly 10-20 s of CPU work
    lin = wl.config_linears(workload)
    for name, N, D, C, seed, kind in lin:
        n = N
        while n > 256 and 3 * 2.0 * n * D * C > budget / len(lin):
            n //= 2
        Xb, Wb, dYb = wl.linear_inputs(N, D, C, seed, kind)
        Xb, dYb = np.ascontiguousarray(Xb[:n]), np.ascontiguousarray(dYb[:n])
        t0 = time.perf_counter()
        Xq, Wq = oracle.linear_fwd(Xb, Wb)
        oracle.gemm_nt(Xq, Wq)
        a, b = oracle.linear_bwd_dx_operands(dYb, Wq, 0, 0)
        oracle.gemm_nt(a, b)
        a, b = oracle.linear_bwd_dw_operands(dYb, Xq, 0, 0)
        oracle.gemm_nt(a, b)
        dt += time.perf_counter() - t0
        flops += 3 * 2.0 * n * D * C
        names.append("%s %d->%d on %d of %d tokens" % (name, D, C, n, N))
    try:
        cores = len(os.sched_getaffinity(0))
    except Exception:
        cores = os.cpu_count()
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp:
        cores = min(cores, int(omp))
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "seconds": round(dt, 2),
            "sample": "oracle fwd+bwd (6 quantizations + 3 float64 products per linear; flops of the slab / its time) of: "
                      + "; ".join(names)}


if __name__ == "__main__":
    main()
