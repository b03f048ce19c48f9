"""Benchmark of the binary-layer hot path on one MI355X.

Workload: BASELINE configuration 2, the ResNet-18 stage convolution (x [16,64,56,56] fp32,
3x3, stride 1, pad 1, 64 filters, alpha epilogue, fp32 NCHW output).  One step is one call of
bmx_binary_conv2d: channel pack of the activations + implicit-GEMM xor/popcount convolution
with the alpha epilogue.  Weights are packed and alpha is computed once, outside the step
(the paper packs weights offline with its model converter).  Inputs are seeded synthetic
tensors that are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is 2*M*N*K binary operations per second of the whole step;
`roofline` prices the dominant kernel (the convolution) against the VALU xor+popcount peak,
its duration measured with HIP events on the launch stream; `cpu_baseline` times the CPU
oracle on the same layer on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# VALU integer peak: 256 CUs x 64 lanes x 2.4 GHz lane-ops/s; one xor + one popcount-accumulate
# handle 32 bit pairs = 64 binary ops per 2 lane-ops.
VALU_PEAK_BINOPS = 256 * 64 * 2.4e9 * 32
HBM_PEAK = 8.0e12


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--all-configs", action="store_true", help="also time configs 1, 3, 4, 5 (stderr)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1705_09864_amd import binding as B
    from paper_1705_09864_amd import synth

    torch.cuda.set_device(0)
    c = synth.config2()
    x_h, w_h = c["x"], c["w"]
    N, C, H, W = x_h.shape
    O, _, KH, KW = w_h.shape
    stride, pad = c["stride"], c["pad"]
    Ho, Wo = B.conv_out_hw(H, W, KH, KW, stride, pad)
    M_, N_, K_ = O, N * Ho * Wo, C * KH * KW
    binops = 2.0 * M_ * N_ * K_

    x = torch.from_numpy(x_h).cuda()
    w = torch.from_numpy(w_h).cuda()
    Wp = B.pack_conv_weights(w)
    alpha = B.alpha_mean_abs(w)
    ws = torch.empty(B.workspace_bytes(B.OP_BINARY_CONV2D, (N, C, H, W, O, KH, KW, stride, pad)),
                     dtype=torch.uint8, device="cuda")
    out = torch.empty((N, O, Ho, Wo), dtype=torch.float32, device="cuda")
    xp = ws.view(torch.int64)[: N * (H + 2 * pad) * (W + 2 * pad) * ((C + 63) // 64)].view(
        N, H + 2 * pad, W + 2 * pad, (C + 63) // 64)

    def step():
        B.binary_conv2d(x, Wp, O, KH, KW, stride, pad, alpha=alpha, out=out, workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = binops / (dt / args.steps) / 1e9

    # per-kernel durations with events on the launch stream (torch's current stream)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for i in range(args.steps):
        ev[i][0].record()
        B.pack_nchw(x, pad, out=xp)
        ev[i][1].record()
        B.binary_conv2d_packed(xp, C, Wp, O, KH, KW, stride, pad, alpha=alpha, out=out)
        ev[i][2].record()
    torch.cuda.synchronize()
    pack_us = float(np.mean([e[0].elapsed_time(e[1]) for e in ev])) * 1e3
    conv_us = float(np.mean([e[1].elapsed_time(e[2]) for e in ev])) * 1e3
    achieved = binops / (conv_us * 1e-6)
    pack_bytes = x_h.nbytes + xp.numel() * 8
    roofline = {"bound": "alu", "kernel": "binary_conv2d implicit GEMM (xor+popcount)",
                "achieved": achieved / 1e12, "peak": VALU_PEAK_BINOPS / 1e12, "unit": "Tbinop/s",
                "frac": achieved / VALU_PEAK_BINOPS, "traffic": None, "avg_us": conv_us,
                "pack_kernel": {"bound": "hbm", "achieved": pack_bytes / (pack_us * 1e-6) / 1e9,
                                "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                                "frac": pack_bytes / (pack_us * 1e-6) / HBM_PEAK, "avg_us": pack_us}}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        alpha_h = oracle.alpha_mean_abs(w_h)
        oracle.binary_conv2d(x_h[:1], w_h, stride, pad, alpha_h)  # page in
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 20:
            t1 = time.perf_counter()
            oracle.binary_conv2d(x_h, w_h, stride, pad, alpha_h)
            t_cpu += time.perf_counter() - t1
            reps += 1
        cpu = {"value": binops * reps / t_cpu / 1e9, "unit": "GOPS", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": "%d full passes of the config-2 layer (%.2f s each)"
               % (reps, t_cpu / reps)}

    line = {"metric": "binary GOPS (2*M*N*K xnor-popcount)", "value": value, "unit": "GOPS",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64 bits -> i32",
            "data": "synthetic",
            "config": {"workload": "config2: binary conv2d 3x3 s1 p1, x[16,64,56,56], 64 filters, "
                                   "alpha epilogue, fp32 out (GEMM view M=64 N=50176 K=576)",
                       "step": "bmx_binary_conv2d = channel pack + implicit-GEMM conv + alpha"},
            "roofline": roofline, "cpu_baseline": cpu}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
