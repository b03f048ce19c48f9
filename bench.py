"""Benchmark of the binary-layer hot path on one MI355X.

Workload: configuration 2 of the benchmark set, the ResNet-18 stage convolution (x [16,64,56,56] fp32,
3x3, stride 1, pad 1, 64 filters, alpha epilogue, fp32 NCHW output).  One step is one call of
bmx_binary_conv2d: channel pack of the activations + implicit-GEMM xor/popcount convolution
with the alpha epilogue.  Weights are packed and alpha is computed once, outside the step
(the paper packs weights offline with its model converter).  Inputs are seeded synthetic
tensors that are resident in HBM before the timed region starts.

HBM residency.  One step touches 26 MB, far less than the 256 MB memory-side cache of the
part, so a loop over one buffer set would measure the cache.  The steps therefore rotate
over enough copies of (input, workspace, output) to exceed that cache; the cache-hot rate
(one buffer set) is reported beside it in `config`.

The kernels run for a few microseconds each, less than the host needs to enqueue them, so
the K timed steps are captured once into a HIP graph (the library launches on the capturing
stream) and the timed region is one replay of that graph: exactly K steps, device-bound.
The eager (host-enqueued) rate is reported next to it.

Prints ONE JSON line.  `value` is 2*M*N*K binary operations per second over the whole step;
`roofline` prices the dominant kernel (the convolution).  It runs on the FP4 matrix cores,
where its 3.7 G multiply-adds x 2 are 0.37 us of work against 1.66 us for the 13.3 MB it must
move, so HBM is the roof that bounds it; the fractions of the VALU xor+popcount peak and of
the FP4 peak are given beside it, and `--tune 5=1` puts the xor/popcount kernel in its place.
Its duration is measured with HIP events on the launch stream around K back-to-back launches
on the same rotating buffers; `cpu_baseline` times the CPU oracle on the same layer on the
host cores; `other_configs` gives event-timed figures for configurations 1, 3, 4, 5 of the set.
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
MALL_BYTES = 256 << 20  # memory-side cache the rotation has to exceed


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="run the steps eagerly next to a plain 256 MiB device copy and exit: the "
                         "workload for the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="pin a kernel choice through bmx_tune_set for the whole run (A/B measurements)")
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
    for kv in args.tune:
        k, v = kv.split("=")
        assert B.lib().bmx_tune_set(int(k), int(v)) == 0

    def graph_of(fns):
        """Capture the calls in `fns`, in order (library launches on the capturing stream)."""
        g = torch.cuda.CUDAGraph()
        st = torch.cuda.Stream()
        with torch.cuda.graph(g, stream=st):
            for fn in fns:
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
        return event_us(graph_of([fn] * reps), reps)

    def rotating_us(make_fn, nsets, reps):
        fns = [make_fn(i % nsets) for i in range(reps)]
        for f in fns[:nsets]:
            f()
        torch.cuda.synchronize()
        return event_us(graph_of(fns), reps)

    # ------------------------------------------------------------------ config 2 (headline)
    c = synth.config2()
    x_h, w_h = c["x"], c["w"]
    N, C, H, W = x_h.shape
    O, _, KH, KW = w_h.shape
    stride, pad = c["stride"], c["pad"]
    Ho, Wo = B.conv_out_hw(H, W, KH, KW, stride, pad)
    M_, N_, K_ = O, N * Ho * Wo, C * KH * KW
    binops = 2.0 * M_ * N_ * K_

    w = torch.from_numpy(w_h).cuda()
    Wp = B.pack_conv_weights(w)
    alpha = B.alpha_mean_abs(w)
    ws_bytes = B.workspace_bytes(B.OP_BINARY_CONV2D, (N, C, H, W, O, KH, KW, stride, pad))
    Cw = (C + 63) // 64
    out_bytes = N * O * Ho * Wo * 4
    step_bytes = x_h.nbytes + ws_bytes + out_bytes
    nsets = MALL_BYTES // step_bytes + 2
    x0 = torch.from_numpy(x_h).cuda()
    xs = [x0] + [x0.clone() for _ in range(nsets - 1)]
    wss = [torch.empty(ws_bytes, dtype=torch.uint8, device="cuda") for _ in range(nsets)]
    outs = [torch.empty((N, O, Ho, Wo), dtype=torch.float32, device="cuda") for _ in range(nsets)]
    xps = [t.view(torch.int64)[: N * (H + 2 * pad) * (W + 2 * pad) * Cw].view(
        N, H + 2 * pad, W + 2 * pad, Cw) for t in wss]

    def make_step(i):
        return lambda: B.binary_conv2d(xs[i], Wp, O, KH, KW, stride, pad, alpha=alpha, out=outs[i],
                                       workspace=wss[i])

    steps = [make_step(i % nsets) for i in range(K_STEPS)]
    if args.traffic_probe:
        # the copy of known size that calibrates the counters: reads 256 MiB, writes 256 MiB
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        for f in steps:
            f()
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": True, "steps": K_STEPS, "copy_bytes_each_way": 256 << 20,
                          "buffer_sets_rotated": int(nsets)}))
        return
    for i in range(args.warmup):
        steps[i % K_STEPS]()
    torch.cuda.synchronize()
    g_steps = graph_of(steps)
    g_steps.replay()  # untimed replay: graph upload
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g_steps.replay()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / K_STEPS * 1e3
    value = binops / (dt / K_STEPS) / 1e9

    # cache-hot rate (one buffer set) and eager rate (host enqueues every launch): context
    hot_us = kernel_us(steps[0], K_STEPS)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for f in steps:
        f()
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) / K_STEPS * 1e3

    # The same K steps with independent batches dealt over four streams (branches of one graph):
    # what a server that overlaps batches would see.  Context only; `value` is the in-order rate.
    n_str = 4
    g4 = torch.cuda.CUDAGraph()
    st4 = [torch.cuda.Stream() for _ in range(n_str)]
    with torch.cuda.graph(g4, stream=st4[0]):
        for s_ in st4[1:]:
            s_.wait_stream(st4[0])
        for i, f in enumerate(steps):  # steps on one buffer set stay on one stream, in order
            with torch.cuda.stream(st4[(i % nsets) % n_str]):
                f()
        for s_ in st4[1:]:
            st4[0].wait_stream(s_)
    torch.cuda.synchronize()
    g4.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g4.replay()
    torch.cuda.synchronize()
    overlapped_ms = (time.perf_counter() - t0) / K_STEPS * 1e3
    del g4

    conv_us = rotating_us(lambda i: (lambda: B.binary_conv2d_packed(
        xps[i], C, Wp, O, KH, KW, stride, pad, alpha=alpha, out=outs[i])), nsets, K_STEPS)
    pack_us = rotating_us(lambda i: (lambda: B.pack_nchw(xs[i], pad, out=xps[i])), nsets, K_STEPS)
    achieved = binops / (conv_us * 1e-6)
    pack_bytes = x_h.nbytes + xps[0].numel() * 8
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic_conv2d_config2.txt")
    if os.path.exists(tpath):  # scaled FETCH_SIZE + WRITE_SIZE of the convolution kernel
        for ln in open(tpath):
            if ln.startswith("hbm_bytes_per_launch:"):
                traffic = int(ln.split(":")[1])
    popcount_conv = any(kv.split("=") == ["5", "1"] for kv in args.tune)
    # bytes the convolution kernel must move: packed image in, packed filters in, fp32 out
    conv_bytes = xps[0].numel() * 8 + Wp.numel() * 8 + out_bytes
    if popcount_conv:
        roofline = {"bound": "alu", "kernel": "conv_stationary_kernel<9,2> (implicit-GEMM xor+popcount)",
                    "achieved": achieved / 1e12, "peak": VALU_PEAK_BINOPS / 1e12, "unit": "Tbinop/s",
                    "frac": achieved / VALU_PEAK_BINOPS}
    else:
        roofline = {"bound": "hbm", "kernel": "conv_mfma_ws_kernel<9,1,4,false> (implicit GEMM on the FP4 matrix cores)",
                    "achieved": conv_bytes / (conv_us * 1e-6) / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                    "frac": conv_bytes / (conv_us * 1e-6) / HBM_PEAK,
                    "algorithmic_bytes_per_launch": conv_bytes,
                    "binops_frac_of_valu_xor_popcount_peak": achieved / VALU_PEAK_BINOPS,
                    "flops_frac_of_fp4_matrix_core_peak": achieved / 10.1e15}
    roofline.update({"traffic": traffic, "avg_us": conv_us,
                "algorithmic_binops_per_launch": binops,
                "output_bytes_per_launch": out_bytes,
                "pack_kernel": {"kernel": "pack_nchw_kernel", "bound": "hbm",
                                "achieved": pack_bytes / (pack_us * 1e-6) / 1e9,
                                "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                                "frac": pack_bytes / (pack_us * 1e-6) / HBM_PEAK, "avg_us": pack_us,
                                "algorithmic_bytes_per_launch": pack_bytes}})
    del xs, wss, outs, xps, steps, g_steps

    # ------------------------------------------------------------------ other configurations
    other = None
    if not args.no_other_configs:
        other = {}

        def alu(ops, us):
            return {"us": us, "Tbinop_s": ops / us / 1e6, "frac_valu": ops / (us * 1e-6) / VALU_PEAK_BINOPS}

        MFMA_FP4_PEAK = 10.1e15  # dense FP4 matrix-core peak, flop/s

        def mfma(ops, us, mfma_flops=None):
            # kernels that run on the matrix cores (bits expanded to FP4 nibbles in registers):
            # binary ops as for the popcount path, plus the multiply-adds actually issued (all
            # bit planes of a k-bit operand in one pass) against the FP4 matrix-core peak
            d = alu(ops, us)
            d["engine"] = "FP4 matrix cores"
            d["frac_mfma_fp4"] = (mfma_flops if mfma_flops is not None else ops) / (us * 1e-6) / MFMA_FP4_PEAK
            return d

        def popcount_engine(fn):
            B.lib().bmx_tune_set(7, 1)
            try:
                return kernel_us(fn, 50)
            finally:
                B.lib().bmx_tune_set(7, 0)

        def hbm(nbytes, us):
            return {"us": us, "GB_s": nbytes / us / 1e3, "frac_hbm": nbytes / (us * 1e-6) / HBM_PEAK}

        # config 1: FC GEMM 64 x 256 x 512 (launch-latency bound)
        c1 = synth.config1()
        a1 = torch.from_numpy(c1["a"]).cuda()
        W1p = B.binarize_pack(torch.from_numpy(c1["w_kn"]).cuda(), 0)
        o1 = torch.empty((64, 256), dtype=torch.int32, device="cuda")
        ws1 = torch.empty(B.workspace_bytes(B.OP_BINARY_FC, (64, 512, 256)), dtype=torch.uint8, device="cuda")
        other["config1_fc_call_64x256x512"] = alu(2.0 * 64 * 256 * 512, kernel_us(
            lambda: B.binary_fc(a1, W1p, integer_out=True, out=o1, workspace=ws1)))
        # config 3: AlexNet classifier layers: GEMM kernel alone (pre-packed activations),
        # the layer call (pack + GEMM + alpha), and the big weight pack
        c3 = synth.config3()
        x3 = torch.from_numpy(c3["x"]).cuda()
        w31 = torch.from_numpy(c3["w1"]).cuda()
        w32 = torch.from_numpy(c3["w2"]).cuda()
        W31p, W32p = B.binarize_pack(w31, 1), B.binarize_pack(w32, 1)
        al1, al2 = B.alpha_mean_abs(w31), B.alpha_mean_abs(w32)
        h1 = torch.empty((256, 4096), dtype=torch.float32, device="cuda")
        h2 = torch.empty((256, 4096), dtype=torch.float32, device="cuda")
        i3 = torch.empty((256, 4096), dtype=torch.int32, device="cuda")
        ws3 = torch.empty(B.workspace_bytes(B.OP_BINARY_FC, (256, 9216, 4096)), dtype=torch.uint8, device="cuda")
        other["config3_fc1_call_256x4096x9216"] = mfma(2.0 * 256 * 4096 * 9216, kernel_us(
            lambda: B.binary_fc(x3, W31p, alpha=al1, out=h1, workspace=ws3), 50))
        other["config3_fc2_call_256x4096x4096"] = mfma(2.0 * 256 * 4096 * 4096, kernel_us(
            lambda: B.binary_fc(h1, W32p, alpha=al2, out=h2, workspace=ws3), 50))
        X3p, H1p = B.binarize_pack(x3, 1), B.binarize_pack(h1, 1)
        other["config3_fc1_gemm_kernel"] = mfma(2.0 * 256 * 4096 * 9216, kernel_us(
            lambda: B.xnor_gemm(X3p, W31p, 9216, out=i3), 50))
        other["config3_fc2_gemm_kernel"] = mfma(2.0 * 256 * 4096 * 4096, kernel_us(
            lambda: B.xnor_gemm(H1p, W32p, 4096, out=i3), 50))
        # the same products on the xor/popcount kernel (the engine is kept where it wins)
        other["config3_fc1_gemm_kernel_popcount_engine"] = alu(2.0 * 256 * 4096 * 9216, popcount_engine(
            lambda: B.xnor_gemm(X3p, W31p, 9216, out=i3)))
        other["config3_fc2_gemm_kernel_popcount_engine"] = alu(2.0 * 256 * 4096 * 4096, popcount_engine(
            lambda: B.xnor_gemm(H1p, W32p, 4096, out=i3)))
        # the two layers chained: through fp32 activations (pack + GEMM, twice) and through
        # packed sign bits handed from layer to layer (one pack, two GEMMs)
        chain_ops = 2.0 * 256 * 4096 * (9216 + 4096)

        def chain_fp32():
            B.binary_fc(x3, W31p, alpha=al1, out=h1, workspace=ws3)
            B.binary_fc(h1, W32p, alpha=al2, out=h2, workspace=ws3)

        bits1 = B.binary_fc_packed(X3p, 9216, W31p, alpha=al1, mode="bits")

        def chain_bits():
            B.binarize_pack(x3, 1, out=X3p)
            B.binary_fc_packed(X3p, 9216, W31p, alpha=al1, mode="bits", out=bits1)
            B.binary_fc_packed(bits1, 4096, W32p, alpha=al2, mode="f32", out=h2)

        other["config3_chain_via_fp32_activations"] = mfma(chain_ops, kernel_us(chain_fp32, 50))
        other["config3_chain_via_packed_bits"] = mfma(chain_ops, kernel_us(chain_bits, 50))
        other["config3_activation_pack_256x9216"] = hbm(x3.numel() * 4 + X3p.numel() * 8, kernel_us(
            lambda: B.binarize_pack(x3, 1, out=X3p)))
        other["config3_weight_pack_4096x9216_cache_assisted"] = hbm(w31.numel() * 4 + W31p.numel() * 8, kernel_us(
            lambda: B.binarize_pack(w31, 1, out=W31p), 20))
        del w31, w32
        # a 1 GiB row pack: larger than the memory-side cache, the sustained HBM figure
        big = torch.empty((8192, 32768), dtype=torch.float32, device="cuda").normal_()
        bigp = B.binarize_pack(big, 1)
        other["row_pack_1GiB_hbm_resident"] = hbm(big.numel() * 4 + bigp.numel() * 8, kernel_us(
            lambda: B.binarize_pack(big, 1, out=bigp), 5))
        del big, bigp
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
            other["config4_conv_s%d_kernel" % s4] = mfma(ops4, kernel_us(
                lambda: B.binary_conv2d_packed(xp4, 256, W4p, 256, 3, 3, s4, 1, alpha=al4, out=o4)))
            ws4 = torch.empty(B.workspace_bytes(B.OP_BINARY_CONV2D, (64, 256, 14, 14, 256, 3, 3, s4, 1)),
                              dtype=torch.uint8, device="cuda")
            other["config4_conv_s%d_call" % s4] = mfma(ops4, kernel_us(
                lambda: B.binary_conv2d(x4, W4p, 256, 3, 3, s4, 1, alpha=al4, out=o4, workspace=ws4)))
            B.lib().bmx_tune_set(5, 1)  # the register-stationary xor/popcount kernel beside it
            try:
                other["config4_conv_s%d_kernel_popcount_engine" % s4] = alu(ops4, kernel_us(
                    lambda: B.binary_conv2d_packed(xp4, 256, W4p, 256, 3, 3, s4, 1, alpha=al4, out=o4)))
            finally:
                B.lib().bmx_tune_set(5, 0)
            if s4 == 1:
                other["config4_pack_nchw"] = hbm(x4.numel() * 4 + xp4.numel() * 8, kernel_us(
                    lambda: B.pack_nchw(x4, 1, out=xp4)))
        # configuration-2 blocks chained (Sec. 2: QActivation -> QConvolution -> BatchNorm, three in
        # a row, 64 -> 64 channels on 16 x 56 x 56): every layer through an fp32 feature map
        # (pack + convolution each), or handing the next layer its packed image (one pack, the
        # BatchNorm folded into a per-channel threshold)
        xc = torch.from_numpy(x_h).cuda()
        wc = [torch.empty((64, 64, 3, 3), dtype=torch.float32, device="cuda").normal_() for _ in range(3)]
        Wc = [B.pack_conv_weights(t) for t in wc]
        alc = [B.alpha_mean_abs(t) for t in wc]
        thc = torch.empty((64,), dtype=torch.float32, device="cuda").normal_()
        wsc = torch.empty(B.workspace_bytes(B.OP_BINARY_CONV2D, (16, 64, 56, 56, 64, 3, 3, 1, 1)),
                          dtype=torch.uint8, device="cuda")
        fa = torch.empty((16, 64, 56, 56), dtype=torch.float32, device="cuda")
        fb = torch.empty_like(fa)
        xpc = B.pack_nchw(xc, 1)
        ia = torch.empty_like(xpc)
        ib = torch.empty_like(xpc)
        ops_c = 3 * 2.0 * 64 * 16 * 56 * 56 * 576

        def blocks_fp32():
            B.binary_conv2d(xc, Wc[0], 64, 3, 3, 1, 1, alpha=alc[0], out=fa, workspace=wsc)
            B.binary_conv2d(fa, Wc[1], 64, 3, 3, 1, 1, alpha=alc[1], out=fb, workspace=wsc)
            B.binary_conv2d(fb, Wc[2], 64, 3, 3, 1, 1, alpha=alc[2], out=fa, workspace=wsc)

        def blocks_packed():
            B.pack_nchw(xc, 1, out=xpc)
            B.binary_conv2d_bits(xpc, 64, Wc[0], 64, 3, 3, 1, 1, alpha=alc[0], thr=thc, out_pad=1, out=ia)
            B.binary_conv2d_bits(ia, 64, Wc[1], 64, 3, 3, 1, 1, alpha=alc[1], thr=thc, out_pad=1, out=ib)
            B.binary_conv2d_packed(ib, 64, Wc[2], 64, 3, 3, 1, 1, alpha=alc[2], out=fa)

        other["config2_three_blocks_via_fp32_maps"] = mfma(ops_c, kernel_us(blocks_fp32, 50))
        other["config2_three_blocks_via_packed_images"] = mfma(ops_c, kernel_us(blocks_packed, 50))
        other["config2_conv_to_packed_image_kernel"] = mfma(ops_c / 3, kernel_us(
            lambda: B.binary_conv2d_bits(xpc, 64, Wc[0], 64, 3, 3, 1, 1, alpha=alc[0], thr=thc, out_pad=1, out=ia)))
        del xc, fa, fb
        # config 5: 2-bit x 1-bit GEMM, whole call (quantise + plane pack + weight pack + GEMM)
        c5 = synth.config5()
        a5 = torch.from_numpy(c5["a"]).cuda()
        w5 = torch.from_numpy(c5["w"]).cuda()
        ws5 = torch.empty(B.workspace_bytes(B.OP_QUANT_GEMM, (1024, 1024, 4096, 2, 1)), dtype=torch.uint8,
                          device="cuda")
        o5 = torch.empty((1024, 1024), dtype=torch.float32, device="cuda")
        other["config5_quant_gemm_call_2planes"] = mfma(2.0 * 2 * 1024 * 1024 * 4096, kernel_us(
            lambda: B.quant_gemm(a5, w5, 2, want_int=False, out_float=o5, workspace=ws5), 20),
            mfma_flops=2.0 * 1024 * 1024 * 4096)
        other["config5_quant_gemm_call_2planes_popcount_engine"] = alu(2.0 * 2 * 1024 * 1024 * 4096, popcount_engine(
            lambda: B.quant_gemm(a5, w5, 2, want_int=False, out_float=o5, workspace=ws5)))

        # the paper's own efficiency workload (Sec. 3.1): 5x5 kernels, 64 filters, batch 200,
        # 8x8 outputs -> GEMM view M = 64, N = 12800, K = 25 * C_in, C_in swept
        for cin in (64, 128, 256, 512):
            xq = torch.empty((200, cin, 12, 12), dtype=torch.float32, device="cuda").normal_()
            wq = torch.empty((64, cin, 5, 5), dtype=torch.float32, device="cuda").normal_()
            Wq, alq = B.pack_conv_weights(wq), B.alpha_mean_abs(wq)
            oq = torch.empty((200, 64, 8, 8), dtype=torch.float32, device="cuda")
            wsq = torch.empty(B.workspace_bytes(B.OP_BINARY_CONV2D, (200, cin, 12, 12, 64, 5, 5, 1, 0)),
                              dtype=torch.uint8, device="cuda")
            other["paper_sec3_1_conv5x5_cin%d_call" % cin] = mfma(
                2.0 * 64 * 12800 * 25 * cin, kernel_us(
                    lambda: B.binary_conv2d(xq, Wq, 64, 5, 5, 1, 0, alpha=alq, out=oq, workspace=wsq)))

        # Sec. 3.1's other two sweeps at 256 input channels, batch 200: filter count (5x5) and
        # kernel size (64 filters), whole calls
        def conv_call(cin, cout, k):
            hw = 8 + k - 1
            xq = torch.empty((200, cin, hw, hw), dtype=torch.float32, device="cuda").normal_()
            wq = torch.empty((cout, cin, k, k), dtype=torch.float32, device="cuda").normal_()
            Wq, alq = B.pack_conv_weights(wq), B.alpha_mean_abs(wq)
            oq = torch.empty((200, cout, 8, 8), dtype=torch.float32, device="cuda")
            wsq = torch.empty(B.workspace_bytes(B.OP_BINARY_CONV2D, (200, cin, hw, hw, cout, k, k, 1, 0)),
                              dtype=torch.uint8, device="cuda")
            us = kernel_us(lambda: B.binary_conv2d(xq, Wq, cout, k, k, 1, 0, alpha=alq, out=oq, workspace=wsq))
            return alu(2.0 * cout * 12800 * k * k * cin, us)

        for cout in (16, 128, 512):
            other["paper_sec3_1_conv5x5_cin256_filters%d_call" % cout] = conv_call(256, cout, 5)
        for k in (1, 3, 7):
            other["paper_sec3_1_conv%dx%d_cin256_call" % (k, k)] = conv_call(256, 64, k)

    # ------------------------------------------------------------------ CPU oracle beside it
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        alpha_h = oracle.alpha_mean_abs(w_h)
        oracle.binary_conv2d(x_h[:1], w_h, stride, pad, alpha_h)  # page in
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 400:
            t1 = time.perf_counter()
            oracle.binary_conv2d(x_h, w_h, stride, pad, alpha_h)
            t_cpu += time.perf_counter() - t1
            reps += 1
        cpu = {"value": binops * reps / t_cpu / 1e9, "unit": "GOPS", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": "%d full passes of the config-2 layer (%.3f s each)"
               % (reps, t_cpu / reps)}
        # the paper's own method on the same host cores (Sec. 2.2.1: xnor + popcount over 64-bit
        # words), GEMM only on the layer's im2col view, as the paper times it (Sec. 3.1)
        col = oracle.im2col(x_h, KH, KW, stride, pad)
        Ap = oracle.binarize_pack(w_h.reshape(O, -1), 1)
        Bp = oracle.binarize_pack(col, 1)
        del col
        oracle.xnor_gemm(Ap, Bp, C * KH * KW)
        t1 = time.perf_counter()
        for _ in range(5):
            oracle.xnor_gemm(Ap, Bp, C * KH * KW)
        t_x = (time.perf_counter() - t1) / 5
        cpu["xnor_popcount_gemm_only"] = {"value": binops / t_x / 1e9, "unit": "GOPS",
                                          "sample": "5 passes of the 64 x 50176 x 576 GEMM on packed words (%.4f s each), "
                                                    "packing not timed" % t_x}

    line = {"metric": "binary GOPS (2*M*N*K xnor-popcount)", "value": value, "unit": "GOPS",
            "n_gpus": 1, "steps": K_STEPS, "warmup": args.warmup, "ms_per_step": ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64 bits -> i32",
            "data": "synthetic",
            "config": {"workload": "config2: binary conv2d 3x3 s1 p1, x[16,64,56,56], 64 filters, "
                                   "alpha epilogue, fp32 out (GEMM view M=64 N=50176 K=576)",
                       "step": "bmx_binary_conv2d = channel pack + implicit-GEMM conv + alpha",
                       "kernels": "pack_nchw_kernel + " + ("conv_stationary_kernel<9,2>" if popcount_conv
                                                           else "conv_mfma_ws_kernel<9,1,4,false>"),
                       "timed_region": "one replay of a HIP graph holding the K steps",
                       "buffer_sets_rotated": int(nsets),
                       "ms_per_step_cache_hot": hot_us * 1e-3,
                       "ms_per_step_eager": eager_ms,
                       "ms_per_step_batches_overlapped_on_streams": overlapped_ms,
                       "streams_for_overlap": n_str},
            "roofline": roofline, "cpu_baseline": cpu, "other_configs": other}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
