"""Benchmark of the binary-layer hot path on one MI355X.

Workload: BASELINE configuration 2, the ResNet-18 stage convolution (x [16,64,56,56] fp32,
3x3, stride 1, pad 1, 64 filters, alpha epilogue, fp32 NCHW output).  One step is one call of
bmx_binary_conv2d: channel pack of the activations + implicit-GEMM xor/popcount convolution
with the alpha epilogue.  Weights are packed and alpha is computed once, outside the step
(the paper packs weights offline with its model converter).  Inputs are seeded synthetic
tensors that are resident in HBM before the timed region starts.

The kernels run for a few microseconds each, less than the host needs to enqueue them, so
the K timed steps are captured once into a HIP graph (the library launches on the capturing
stream) and the timed region is one replay of that graph: exactly K steps, device-bound.
The eager (host-enqueued) rate is reported next to it.

Prints ONE JSON line.  `value` is 2*M*N*K binary operations per second over the whole step;
`roofline` prices the dominant kernel (the convolution) against the VALU xor+popcount peak,
its duration measured with HIP events on the launch stream around K back-to-back launches;
`cpu_baseline` times the CPU oracle on the same layer on the host cores; `other_configs`
gives the same event-timed kernel figures for BASELINE configurations 1, 3, 4 and 5.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# VALU integer peak: 256 CUs x 64 lanes x 2.4 GHz lane-ops/s; one v_xor_b32 plus one
# v_bcnt_u32_b32 (popcount-accumulate) handle 32 bit pairs = 64 binary ops per 2 lane-ops.
VALU_PEAK_BINOPS = 256 * 64 * 2.4e9 * 32
HBM_PEAK = 8.0e12


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
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
    K_STEPS = args.steps

    def graph_of(fn, reps):
        """Capture `reps` calls of fn (library launches on the capturing stream)."""
        g = torch.cuda.CUDAGraph()
        st = torch.cuda.Stream()
        with torch.cuda.graph(g, stream=st):
            for _ in range(reps):
                fn()
        torch.cuda.synchronize()
        return g

    def event_us(g, reps, rounds=3):
        """Average microseconds per captured call over one replay (best of `rounds`)."""
        g.replay()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(rounds):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e3 / reps)
        return best

    def kernel_us(fn, reps=100):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        return event_us(graph_of(fn, reps), reps)

    # ------------------------------------------------------------------ config 2 (headline)
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
    Cw = (C + 63) // 64
    xp = ws.view(torch.int64)[: N * (H + 2 * pad) * (W + 2 * pad) * Cw].view(
        N, H + 2 * pad, W + 2 * pad, Cw)

    def step():
        B.binary_conv2d(x, Wp, O, KH, KW, stride, pad, alpha=alpha, out=out, workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    g_steps = graph_of(step, K_STEPS)
    g_steps.replay()  # untimed replay: graph upload
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g_steps.replay()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / K_STEPS * 1e3
    value = binops / (dt / K_STEPS) / 1e9

    # eager rate (host enqueues every launch): context only
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K_STEPS):
        step()
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) / K_STEPS * 1e3

    conv_us = kernel_us(lambda: B.binary_conv2d_packed(xp, C, Wp, O, KH, KW, stride, pad,
                                                       alpha=alpha, out=out), K_STEPS)
    pack_us = kernel_us(lambda: B.pack_nchw(x, pad, out=xp), K_STEPS)
    achieved = binops / (conv_us * 1e-6)
    pack_bytes = x_h.nbytes + xp.numel() * 8
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic_conv2d_config2.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
    roofline = {"bound": "alu", "kernel": "conv_stationary_kernel<9> (implicit-GEMM xor+popcount)",
                "achieved": achieved / 1e12, "peak": VALU_PEAK_BINOPS / 1e12, "unit": "Tbinop/s",
                "frac": achieved / VALU_PEAK_BINOPS, "traffic": traffic, "avg_us": conv_us,
                "algorithmic_binops_per_launch": binops,
                "pack_kernel": {"bound": "hbm", "achieved": pack_bytes / (pack_us * 1e-6) / 1e9,
                                "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                                "frac": pack_bytes / (pack_us * 1e-6) / HBM_PEAK, "avg_us": pack_us,
                                "algorithmic_bytes_per_launch": pack_bytes}}

    # ------------------------------------------------------------------ other configurations
    other = None
    if not args.no_other_configs:
        other = {}

        def alu(ops, us):
            return {"us": us, "Tbinop_s": ops / us / 1e6, "frac_valu": ops / (us * 1e-6) / VALU_PEAK_BINOPS}

        def hbm(nbytes, us):
            return {"us": us, "GB_s": nbytes / us / 1e3, "frac_hbm": nbytes / (us * 1e-6) / HBM_PEAK}

        # config 1: FC GEMM 64 x 256 x 512 (launch-latency bound)
        c1 = synth.config1()
        a1 = torch.from_numpy(c1["a"]).cuda()
        W1p = B.binarize_pack(torch.from_numpy(c1["w_kn"]).cuda(), 0)
        o1 = torch.empty((64, 256), dtype=torch.int32, device="cuda")
        ws1 = torch.empty(B.workspace_bytes(B.OP_BINARY_FC, (64, 512, 256)), dtype=torch.uint8, device="cuda")
        other["config1_fc_64x256x512"] = alu(2.0 * 64 * 256 * 512, kernel_us(
            lambda: B.binary_fc(a1, W1p, integer_out=True, out=o1, workspace=ws1)))
        # config 3: AlexNet classifier layers (pack + GEMM + alpha), and the big weight pack
        c3 = synth.config3()
        x3 = torch.from_numpy(c3["x"]).cuda()
        w31 = torch.from_numpy(c3["w1"]).cuda()
        w32 = torch.from_numpy(c3["w2"]).cuda()
        W31p, W32p = B.binarize_pack(w31, 1), B.binarize_pack(w32, 1)
        al1, al2 = B.alpha_mean_abs(w31), B.alpha_mean_abs(w32)
        h1 = torch.empty((256, 4096), dtype=torch.float32, device="cuda")
        h2 = torch.empty((256, 4096), dtype=torch.float32, device="cuda")
        ws3 = torch.empty(B.workspace_bytes(B.OP_BINARY_FC, (256, 9216, 4096)), dtype=torch.uint8, device="cuda")
        other["config3_fc1_256x4096x9216"] = alu(2.0 * 256 * 4096 * 9216, kernel_us(
            lambda: B.binary_fc(x3, W31p, alpha=al1, out=h1, workspace=ws3), 50))
        other["config3_fc2_256x4096x4096"] = alu(2.0 * 256 * 4096 * 4096, kernel_us(
            lambda: B.binary_fc(h1, W32p, alpha=al2, out=h2, workspace=ws3), 50))
        other["config3_weight_pack_4096x9216"] = hbm(w31.numel() * 4 + W31p.numel() * 8, kernel_us(
            lambda: B.binarize_pack(w31, 1, out=W31p), 20))
        del w31, w32
        # config 4: deep conv stage, stride 1 and 2 (conv kernel alone, and pack alone)
        for s4 in (1, 2):
            c4 = synth.config4(stride=s4)
            x4 = torch.from_numpy(c4["x"]).cuda()
            w4 = torch.from_numpy(c4["w"]).cuda()
            W4p, al4 = B.pack_conv_weights(w4), B.alpha_mean_abs(w4)
            xp4 = B.pack_nchw(x4, 1)
            ho4, wo4 = B.conv_out_hw(14, 14, 3, 3, s4, 1)
            o4 = torch.empty((64, 256, ho4, wo4), dtype=torch.float32, device="cuda")
            ops4 = 2.0 * 256 * 64 * ho4 * wo4 * 2304
            other["config4_conv_s%d" % s4] = alu(ops4, kernel_us(
                lambda: B.binary_conv2d_packed(xp4, 256, W4p, 256, 3, 3, s4, 1, alpha=al4, out=o4)))
            if s4 == 1:
                other["config4_pack_nchw"] = hbm(x4.numel() * 4 + xp4.numel() * 8, kernel_us(
                    lambda: B.pack_nchw(x4, 1, out=xp4)))
        # config 5: 2-bit x 1-bit GEMM, whole call (quantise + plane pack + weight pack + GEMM)
        c5 = synth.config5()
        a5 = torch.from_numpy(c5["a"]).cuda()
        w5 = torch.from_numpy(c5["w"]).cuda()
        ws5 = torch.empty(B.workspace_bytes(B.OP_QUANT_GEMM, (1024, 1024, 4096, 2, 1)), dtype=torch.uint8,
                          device="cuda")
        o5 = torch.empty((1024, 1024), dtype=torch.float32, device="cuda")
        other["config5_quant_gemm_call_2planes"] = alu(2.0 * 2 * 1024 * 1024 * 4096, kernel_us(
            lambda: B.quant_gemm(a5, w5, 2, want_int=False, out_float=o5, workspace=ws5), 20))

    # ------------------------------------------------------------------ CPU oracle beside it
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
            "n_gpus": 1, "steps": K_STEPS, "warmup": args.warmup, "ms_per_step": ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64 bits -> i32",
            "data": "synthetic",
            "config": {"workload": "config2: binary conv2d 3x3 s1 p1, x[16,64,56,56], 64 filters, "
                                   "alpha epilogue, fp32 out (GEMM view M=64 N=50176 K=576)",
                       "step": "bmx_binary_conv2d = channel pack + implicit-GEMM conv + alpha",
                       "timed_region": "one replay of a HIP graph holding the K steps",
                       "ms_per_step_eager": eager_ms},
            "roofline": roofline, "cpu_baseline": cpu, "other_configs": other}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
