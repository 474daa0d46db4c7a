#!/usr/bin/env python3
"""Benchmark of the NVFP4 quantized linear layer hot path on one MI355X.

A step is one pass of the whole path (forward product, input-gradient product, weight-gradient
product, with all six quantizations) over every linear layer of one transformer block of the
768-hidden model shape (tokens 8192; QKV 768->2304, O 768->768, up 768->3072, down 3072->768),
on synthetic inputs that are resident in HBM before the clock starts.

Prints ONE JSON line.  `value` = algorithmic flops of a step (3 * sum 2*N*D*C) / wall time.
`roofline` describes the dominant kernel (the packed-operand GEMM) measured with events on the
launch stream; `cpu_baseline` times the CPU oracle on a bounded sample of the same workload.
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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed steps; the default is long enough (tens of ms) for the GPU clocks to settle")
    ap.add_argument("--workload", default="cfg2_block768")
    ap.add_argument("--no-extras", action="store_true", help="skip the quantizer-bandwidth and square-GEMM side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device copy of 1 GiB five times (reference point for HBM byte counters)")
    ap.add_argument("--square-gemm", type=int, default=0, metavar="REPS",
                    help="only run the 8192^3 product on pre-quantized operands REPS times (for counter profiles)")
    return ap.parse_args()


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

    if args.square_gemm:
        n = 8192
        gen = torch.Generator(device=dev).manual_seed(0)
        ops = []
        for _ in range(2):
            t = tj.alloc_nvfp4(n, n)
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

    def dev_bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    # ---- resident inputs, contexts, outputs and workspaces for every linear of the block -----------------
    layers = []
    for li, (name, N, D, C, seed, kind) in enumerate(wl.config_linears(args.workload)):
        Xb, Wb, dYb = wl.linear_inputs(N, D, C, seed, kind)
        L = dict(name=name, N=N, D=D, C=C, li=li, X=dev_bf16(Xb), W=dev_bf16(Wb), dY=dev_bf16(dYb))
        L["Xq"] = tj.alloc_nvfp4(N, D)
        L["Wq"] = tj.alloc_nvfp4(C, D)
        L["Y"] = torch.empty((N, C), dtype=torch.bfloat16, device=dev)
        L["dX"] = torch.empty((N, D), dtype=torch.bfloat16, device=dev)
        L["dW"] = torch.empty((C, D), dtype=torch.bfloat16, device=dev)
        nbytes = max(tj.workspace_bytes(op, N, D, C) for op in (B.OP_LINEAR_FWD, B.OP_LINEAR_BWD))
        L["ws"] = tj.alloc_workspace(nbytes)
        layers.append(L)
    flops_step = wl.config_flops(args.workload)
    # lower bound of a step from the two rooflines, per linear: bf16 reads of X, W, dY, packed operands written and
    # read once each (Q1..Q6), bf16 writes of Y, dX, dW
    t_min = 0.0
    for L in layers:
        N, D, C = L["N"], L["D"], L["C"]
        nbytes = 2.0 * (N * D + C * D + N * C) + 2 * 0.5625 * (N * D + C * D) * 2 + 2 * 0.5625 * (2 * N * C) \
            + 2.0 * (N * C + N * D + C * D)
        t_min += max(3 * 2.0 * N * D * C / (MFMA_F16_PEAK_TFLOPS * 1e12), nbytes / (HBM_PEAK_GBS * 1e9))

    def step(sr_seed):
        for L in layers:
            tj.linear_fwd(L["X"], L["W"], B.OUT_BF16, Y=L["Y"], Xq=L["Xq"], Wq=L["Wq"], ws=L["ws"])
        for L in reversed(layers):
            tj.linear_bwd(L["dY"], L["Xq"], L["Wq"], sr_seed, L["li"], B.OUT_BF16, dX=L["dX"], dW=L["dW"], ws=L["ws"])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(1000 + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = flops_step / (ms_per_step * 1e-3) / 1e12

    # ---- dominant kernel: the packed GEMM (gemm_nt_kernel), on the operands the step just produced ----------
    # The products of a step that run as ONE gemm_nt_kernel launch (forward and input-gradient products; the
    # weight-gradient products are split along K and add a reduction kernel) are launched back to back between
    # two events recorded on the launch stream; duration per launch = elapsed / launches.
    gemm_jobs = []
    for L in layers:
        dYq = tj.quantize(L["dY"], 0, B.ROUND_SR, seed=1, tensor_id=L["li"] * 8 + 3)
        Wq2 = tj.quantize(L["Wq"], 1, B.ROUND_SR, seed=1, tensor_id=L["li"] * 8 + 4)
        dYq2 = tj.quantize(L["dY"], 1, B.ROUND_SR, seed=1, tensor_id=L["li"] * 8 + 5)
        Xq2 = tj.quantize(L["Xq"], 1, B.ROUND_SR, seed=1, tensor_id=L["li"] * 8 + 6)
        for A, Bt, out in ((L["Xq"], L["Wq"], L["Y"]), (dYq, Wq2, L["dX"]), (dYq2, Xq2, L["dW"])):
            nws = tj.workspace_bytes(B.OP_GEMM, A.rows, A.K, Bt.rows)
            if nws == 0:
                gemm_jobs.append((A, Bt, out, tj.alloc_workspace(16), 2.0 * A.rows * Bt.rows * A.K))
    for _ in range(20):
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
    tpath = os.path.join(ROOT, "profiles", "gemm_quant_cfg2_block768_hbm_traffic.txt")
    if args.workload == "cfg2_block768" and os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch="):
                traffic = int(line.split("=")[1])
    roofline = {"kernel": "gemm_nt_kernel", "bound": "mfma", "achieved": round(achieved, 2),
                "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / MFMA_F16_PEAK_TFLOPS, 4),
                "traffic": traffic, "avg_launch_ms": round(gemm_ms, 5), "flops_per_launch": gemm_flops,
                "launches_timed": reps * len(gemm_jobs),
                "note": "mean over the %d single-launch products of a step (2*M*N*K flops each)" % len(gemm_jobs)}

    out = {"metric": "nvfp4_linear_fwd_bwd_tflops", "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp4xfp4->f32 (fp16 MFMA)",
           "data": "synthetic",
           "config": {"workload": args.workload, "tokens": layers[0]["N"],
                      "linears": [[L["name"], L["D"], L["C"]] for L in layers], "outer_scale": "per-tensor",
                      "flops_per_step": flops_step},
           "frac_of_mfma_peak": round(value / MFMA_F16_PEAK_TFLOPS, 4),
           "frac_of_roofline_lower_bound": round(t_min * 1e3 / ms_per_step, 4),
           "roofline": roofline}

    if not args.no_extras:
        out["extras"] = extras(tj, wl, np, torch, dev_bf16)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(wl, np, args.workload)
    print(json.dumps(out))


def time_events(torch, fn, reps):
    """Mean duration of fn over reps back-to-back calls, bracketed by two events on the launch stream."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def extras(tj, wl, np, torch, dev_bf16):
    """Side measurements named by the metric: quantizer GB/s on the 8192 x 8192 stress tensor and the square
    8192^3 products.  Inputs rotate through four buffers (4 x 134 MB > the 256 MB last-level cache)."""
    B = tj.binding
    res = {}
    R = Cc = 8192
    cfg = wl.CONFIGS["cfg4_quant_stress"]
    bits = wl.student_t_bf16((R, Cc), cfg["nu"], cfg["scale"], cfg["seed"])
    bufs = [dev_bf16(bits)]
    for _ in range(3):
        bufs.append(bufs[0].clone())
    outs = [tj.alloc_nvfp4(R, Cc) for _ in range(2)]
    ws = tj.alloc_workspace(tj.workspace_bytes(B.OP_QUANTIZE, R, Cc, 0))
    amax = tj.amax_bf16(bufs[0], ws)
    alg_bytes = R * Cc * 2 + R * Cc // 2 + R * Cc // 16 + 4
    cases = {
        "row_rtn_amax_given": lambda i: tj.quantize(bufs[i % 4], 0, B.ROUND_RTN, outs[i % 2], amax_in=amax, ws=ws),
        "row_rtn_with_amax_pass": lambda i: tj.quantize(bufs[i % 4], 0, B.ROUND_RTN, outs[i % 2], ws=ws),
        "row_sr_amax_given": lambda i: tj.quantize(bufs[i % 4], 0, B.ROUND_SR, outs[i % 2], seed=7, amax_in=amax, ws=ws),
        "col_sr_amax_given": lambda i: tj.quantize(bufs[i % 4], 1, B.ROUND_SR, outs[i % 2], seed=7, amax_in=amax, ws=ws),
        "col_sr_with_amax_pass": lambda i: tj.quantize(bufs[i % 4], 1, B.ROUND_SR, outs[i % 2], seed=7, ws=ws),
        # the paper's own outer scale (1 x 128 blocks) needs no maximum pass at all (the optional dequantized maximum,
        # which only a later tensor-mode re-quantization would use, is not requested)
        "row_rtn_block128_single_pass": lambda i: tj.quantize(bufs[i % 4], 0, B.ROUND_RTN, outs128[i % 2],
                                                              outer=B.OUTER_BLOCK128, ws=ws),
        "row_sr_block128_single_pass": lambda i: tj.quantize(bufs[i % 4], 0, B.ROUND_SR, outs128[i % 2], seed=7,
                                                             outer=B.OUTER_BLOCK128, ws=ws),
    }
    outs128 = [tj.alloc_nvfp4(R, Cc, B.OUTER_BLOCK128, with_amax=False) for _ in range(2)]
    for name, fn in cases.items():
        for i in range(300):                           # long enough for the clocks to settle
            fn(i)
        torch.cuda.synchronize()
        ms = time_events(torch, fn, 200)
        gbs = alg_bytes / (ms * 1e-3) / 1e9
        res["quant_8192x8192_" + name] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    # both backward operands of one tensor from a single read: 2 B in + 2 x 0.5625 B out per element
    fn = lambda i: tj.quantize_dual(bufs[i % 4], B.ROUND_SR, outs[0], outs[1], seed=7, tensor_id_row=3, tensor_id_col=5,
                                    amax_in=amax, ws=ws)
    for i in range(300):
        fn(i)
    torch.cuda.synchronize()
    ms = time_events(torch, fn, 200)
    gbs = (R * Cc * 2 + 2 * (R * Cc // 2 + R * Cc // 16) + 8) / (ms * 1e-3) / 1e9
    res["quant_8192x8192_dual_row_col_sr_amax_given"] = {"ms": round(ms, 4), "GB/s": round(gbs, 1),
                                                          "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    # re-quantization of a packed tensor (Q4 / Q6): 0.5625 B in + 0.5625 B out per element
    src = outs[0]
    tj.quantize(bufs[0], 0, B.ROUND_RTN, src, ws=ws)
    dst = tj.alloc_nvfp4(Cc, R)
    fn = lambda i: tj.quantize(src, 1, B.ROUND_SR, dst, seed=7, tensor_id=i)
    for i in range(300):
        fn(i)
    torch.cuda.synchronize()
    ms = time_events(torch, fn, 200)
    gbs = (R * Cc * 9 // 8 + 8) / (ms * 1e-3) / 1e9
    res["requant_col_sr_8192x8192"] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    del bufs

    # square products on pre-quantized operands: M = N = K = 8192
    n = 8192
    Xb, Wb, dYb = wl.linear_inputs(n, n, n, wl.CONFIGS["cfg5_square8192"]["seed"], "square")
    X, W, dY = dev_bf16(Xb), dev_bf16(Wb), dev_bf16(dYb)
    Y, Xq, Wq = tj.linear_fwd(X, W)
    wsd = tj.alloc_workspace(max(tj.workspace_bytes(op, n, n, n) for op in (B.OP_LINEAR_FWD, B.OP_LINEAR_BWD)))
    dX = torch.empty_like(Y)
    dW = torch.empty_like(Y)
    gws = tj.alloc_workspace(tj.workspace_bytes(B.OP_GEMM, n, n, n))
    fn = lambda i: tj.gemm_nt(Xq, Wq, B.OUT_BF16, out=Y, ws=gws)
    for i in range(150):                               # ~0.1 s: the clocks settle under matrix load
        fn(i)
    torch.cuda.synchronize()
    ms = time_events(torch, fn, 50)
    tf = 2.0 * n ** 3 / (ms * 1e-3) / 1e12
    res["gemm_8192_cubed"] = {"ms": round(ms, 4), "TFLOP/s": round(tf, 1), "frac_mfma_peak": round(tf / MFMA_F16_PEAK_TFLOPS, 4)}

    def full(i):
        tj.linear_fwd(X, W, B.OUT_BF16, Y=Y, Xq=Xq, Wq=Wq, ws=wsd)
        tj.linear_bwd(dY, Xq, Wq, i, 0, B.OUT_BF16, dX=dX, dW=dW, ws=wsd)
    for i in range(20):
        full(i)
    torch.cuda.synchronize()
    ms = time_events(torch, full, 20)
    tf = 3 * 2.0 * n ** 3 / (ms * 1e-3) / 1e12
    res["linear_fwd_bwd_8192_cubed_full_overhead"] = {"ms": round(ms, 4), "TFLOP/s": round(tf, 1),
                                                      "frac_mfma_peak": round(tf / MFMA_F16_PEAK_TFLOPS, 4)}
    return res


def cpu_baseline(wl, np, workload):
    """The CPU oracle, as it stands, on a bounded sample of the workload: every linear of the block on (at most)
    8192 tokens - all six quantizations and the three float64 products each - on all host threads."""
    import oracle
    oracle.lib()
    flops = 0.0
    names = []
    dt = 0.0
    for name, N, D, C, seed, kind in wl.config_linears(workload):
        n = min(N, 8192)
        if 3 * 2.0 * n * D * C > 1.5e11:
            continue                                   # keep the sample to roughly 10 s of CPU work
        Xb, Wb, dYb = wl.linear_inputs(n, D, C, seed, kind)
        t0 = time.perf_counter()
        Xq, Wq = oracle.linear_fwd(Xb, Wb)
        oracle.gemm_nt(Xq, Wq)
        a, b = oracle.linear_bwd_dx_operands(dYb, Wq, 0, 0)
        oracle.gemm_nt(a, b)
        a, b = oracle.linear_bwd_dw_operands(dYb, Xq, 0, 0)
        oracle.gemm_nt(a, b)
        dt += time.perf_counter() - t0
        flops += 3 * 2.0 * n * D * C
        names.append("%s %d->%d x %d tokens" % (name, D, C, n))
    try:
        cores = len(os.sched_getaffinity(0))
    except Exception:
        cores = os.cpu_count()
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp:
        cores = min(cores, int(omp))
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "seconds": round(dt, 2),
            "sample": "oracle fwd+bwd (6 quantizations + 3 float64 products per linear) of: " + "; ".join(names)}


if __name__ == "__main__":
    main()
