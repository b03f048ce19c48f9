"""Benchmark of the binary-layer hot path on one MI355X.

Workload (headline): configuration 3 of the benchmark set, the largest one, the AlexNet classifier
pair: batch 256, 9216 -> 4096 then 4096 -> 4096, fp32 activations in, fp32 out, alpha per output
row.  One step is the whole configuration: bmx_binary_fc on the input (binarise + pack, xnor GEMM,
alpha epilogue), then bmx_binary_fc on the first layer's fp32 output.  Weights are packed and
alpha is computed once, outside the step (the paper packs weights offline with its model
converter, Sec. 2.2.3).  Inputs are seeded synthetic tensors resident in HBM before the timed
region starts.

HBM residency.  One step touches about 25 MB (activations, packed weights, outputs), far less
than the 256 MB memory-side cache of the part, so a loop over one buffer set would measure the
cache.  Every timed figure here therefore rotates over enough independent copies of all its
buffers, weights included, to exceed that cache; the cache-hot rate of the headline is reported
beside it in `config` and labelled as such.

The kernels run for a few microseconds each, less than the host needs to enqueue them, so the K
timed steps are captured once into a HIP graph (the library launches on the capturing stream) and
the timed region is one replay of that graph: exactly K steps, device-bound.  Kernel durations are
measured the same way (events on the launch stream around one replay of back-to-back launches on
the rotating buffers).

Prints ONE JSON line.  `value` is 2*M*N*K binary operations per second over the whole step.
`roofline` prices the dominant kernel, the first layer's GEMM; every other kernel and every other
configuration carries the same kind of block (`bound` = the roof with the larger ideal time for
that launch: HBM bytes, matrix-core flops of the operand type that ran, or VALU xor+popcount
operations).  `cpu_baseline` times the CPU oracle on the host cores, per configuration, and the
paper's own method (xnor + popcount on 64-bit words, OpenMP) beside it.

`--phase NAME` runs one section only (headline, config1, config2, config4, config5, sec31, biggemm,
packs, probe): the workload of the per-configuration rocprofv3 summaries under profiles/.
"""
import argparse
import ctypes
import json
import os
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# VALU integer peak: 256 CUs x 64 lanes x 2.4 GHz lane-ops/s; one v_xor_b32 plus one
# v_bcnt_u32_b32 (popcount-accumulate) handle 32 bit pairs = 64 binary ops per 2 lane-ops.
VALU_PEAK_BINOPS = 256 * 64 * 2.4e9 * 32
HBM_PEAK = 8.0e12
FP4_PEAK = 10.1e15   # dense FP4 matrix-core peak, flop/s
INT8_PEAK = 5.0e15   # dense int8 matrix-core peak, op/s
MALL_BYTES = 256 << 20  # memory-side cache
# what a rotation over buffer sets has to cover: with 1.1 times the cache a cyclic walk still finds
# much of its data there (the fc1 GEMM: 8.5 us at 285 MB, 9.3 at 590 MB, 9.5 at 1.2 GB)
ROTATE_BYTES = 4 * MALL_BYTES
PHASES = ("headline", "fc1", "fc2", "config1", "config2", "config4", "config5", "sec31", "packs", "biggemm", "probe")


def roofline_block(kernel, us, binops=0.0, nbytes=0.0, mfma_flops=None):
    """Roofline of one launch.  The engine is read off the kernel's name: FP4 / int8 matrix cores
    (flops against that operand type's dense peak) or the VALU xor+popcount form (binary ops
    against 256 CUs x 64 lanes x 2.4 GHz x 32); every kernel also has its algorithmic HBM bytes.
    `bound` is the roof whose ideal time for this launch is larger, `frac` = ideal / measured."""
    t = us * 1e-6
    if "fp4" in kernel or "conv_mfma_ws" in kernel:
        bound, peak, unit, work = "mfma", FP4_PEAK, "TFLOP/s", (binops if mfma_flops is None else mfma_flops)
        dtype = "fp4 e2m1 x fp4 e2m1 -> fp32"
    elif "int8" in kernel:
        bound, peak, unit, work, dtype = "mfma", INT8_PEAK, "TOP/s", (binops if mfma_flops is None else mfma_flops), "i8 x i8 -> i32"
    elif binops > 0:
        bound, peak, unit, work, dtype = "alu", VALU_PEAK_BINOPS, "Tbinop/s", binops, "u32 xor/and + popcount -> i32"
    else:
        bound, peak, unit, work, dtype = "hbm", HBM_PEAK, "GB/s", 0.0, "f32 compare -> bits"
    t_compute = work / peak if work else 0.0
    t_hbm = nbytes / HBM_PEAK
    d = {"kernel": kernel, "avg_us": us, "dtype": dtype}
    if t_hbm >= t_compute:
        d.update({"bound": "hbm", "achieved": nbytes / t / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                  "frac": t_hbm / t})
    else:
        d.update({"bound": bound, "achieved": work / t / 1e12, "peak": peak / 1e12, "unit": unit,
                  "frac": t_compute / t})
    d["algorithmic_bytes_per_launch"] = int(nbytes)
    if work:
        d["algorithmic_ops_per_launch"] = work
        d["frac_of_%s_peak" % ("valu_xor_popcount" if bound == "alu" else "matrix_core")] = t_compute / t
        d["frac_of_hbm_peak"] = t_hbm / t
    if binops and bound != "alu":
        # a comparison, not a roofline: the same binary ops against the VALU xor+popcount peak
        d["binops_vs_valu_xor_popcount_peak"] = binops / t / VALU_PEAK_BINOPS
    return d


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--phase", choices=("all",) + PHASES, default="all",
                    help="run one section only (the workload of a per-configuration profile)")
    ap.add_argument("--lean", action="store_true",
                    help="HBM-resident rotating launches only: skip the cache-hot, eager and other-engine context "
                         "figures (the workload of the rocprofv3 kernel-trace summaries, whose per-kernel averages "
                         "then mix nothing else in)")
    ap.add_argument("--eager", action="store_true",
                    help="with --phase: issue the timed launches eagerly instead of replaying a graph")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="run the headline steps eagerly next to a plain 256 MiB device copy and exit: the "
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
    want = (lambda name: args.phase in ("all", name))

    # ------------------------------------------------------------------ timing helpers
    def graph_of(fns):
        """Capture the calls in `fns`, in order (library launches on the capturing stream)."""
        g = torch.cuda.CUDAGraph()
        st = torch.cuda.Stream()
        with torch.cuda.graph(g, stream=st):
            for fn in fns:
                fn()
        torch.cuda.synchronize()
        return g

    def graph_of_lanes(fns, lanes):
        """Capture the calls in `fns` with call i on side stream i % lanes: the calls of one lane
        run in order, the lanes beside each other (independent batches in flight at once)."""
        g = torch.cuda.CUDAGraph()
        st = torch.cuda.Stream()
        side = [torch.cuda.Stream() for _ in range(lanes)]
        with torch.cuda.graph(g, stream=st):
            fork = torch.cuda.Event()
            fork.record(st)
            for sd in side:
                sd.wait_event(fork)
            for i, fn in enumerate(fns):
                with torch.cuda.stream(side[i % lanes]):
                    fn()
            for sd in side:
                join = torch.cuda.Event()
                join.record(sd)
                st.wait_event(join)
        torch.cuda.synchronize()
        return g

    def event_us(run, reps, rounds=3):
        """Average microseconds per call over `run()` (reps calls), best of `rounds`."""
        run()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(rounds):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            run()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e3 / reps)
        return best

    def nsets_for(bytes_per_set, cap=512):
        return int(min(cap, ROTATE_BYTES // max(int(bytes_per_set), 1) + 2))

    def rotating_us(calls, reps=None):
        """calls[i] runs the measured call on buffer set i.  The sets together exceed the
        memory-side cache, so every launch finds its inputs in HBM.  Returns (us per call, name
        of the last kernel the call launched)."""
        # (at least 200 launches per figure whatever K is: the replay's fixed cost, some tens of
        # microseconds of graph launch, must not weigh on a per-launch average of a few microseconds)
        reps = reps or max(K_STEPS, 200)
        reps = max(reps, len(calls))
        fns = [calls[i % len(calls)] for i in range(reps)]
        for f in calls:
            f()
        name = B.last_kernel()
        torch.cuda.synchronize()
        if args.eager:
            us = event_us(lambda: [f() for f in fns], reps, rounds=2)
        else:
            g = graph_of(fns)
            us = event_us(g.replay, reps)
            del g
        return us, name

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    def with_tune(kv, fn):
        for k, v in kv.items():
            assert B.lib().bmx_tune_set(k, v) == 0
        try:
            return fn()
        finally:
            B.lib().bmx_tune_set(0, 0)
            for kv2 in args.tune:  # the run-wide pins stay
                k, v = kv2.split("=")
                B.lib().bmx_tune_set(int(k), int(v))

    f32 = lambda *shape: torch.empty(shape, dtype=torch.float32, device="cuda")
    i32 = lambda *shape: torch.empty(shape, dtype=torch.int32, device="cuda")
    u8 = lambda n: torch.empty(int(n), dtype=torch.uint8, device="cuda")

    # ------------------------------------------------------------------ clock and VALU peak, measured
    probe = None
    if want("probe") or args.phase == "all":
        out3 = torch.zeros(3, dtype=torch.int64, device="cuda")
        iters, wgs = 4000, 256 * 8  # eight waves per SIMD
        khz = B.probe_valu(wgs, iters, out3)
        us = event_us(lambda: B.probe_valu(wgs, iters, out3), 1, rounds=5)
        cyc, ticks = int(out3[0].item()), int(out3[1].item())
        ops = wgs * 256.0 * iters * 128 * 64
        probe = {"kernel": B.last_kernel(), "us": us, "measured_valu_xor_popcount_peak_Tbinop_s": ops / us / 1e6,
                 "vs_nominal_peak_at_2.4GHz": ops / (us * 1e-6) / VALU_PEAK_BINOPS,
                 "shader_clock_GHz_observed_under_load": (cyc / max(ticks, 1)) * khz * 1e3 / 1e9,
                 "wall_clock_kHz": khz, "waves_per_simd": 8}
        probe_peak = ops / (us * 1e-6)
    else:
        probe_peak = None

    def add_measured_peak(block):
        """Second denominator for a VALU-bound kernel: the peak the probe reached in this run."""
        if probe_peak and block.get("bound") == "alu":
            block["frac_of_measured_valu_peak"] = block["achieved"] * 1e12 / probe_peak
        return block

    line = {"metric": "binary GOPS (2*M*N*K xnor-popcount)", "unit": "GOPS", "n_gpus": 1,
            "steps": K_STEPS, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "data": "synthetic"}
    other = {}
    cpu = None

    # ------------------------------------------------------------------ configuration 3 (headline)
    c3 = synth.config3()
    Bt, F0, F1, F2 = 256, 9216, 4096, 4096
    ops1, ops2 = 2.0 * Bt * F1 * F0, 2.0 * Bt * F2 * F1
    sub = args.phase if args.phase in ("fc1", "fc2") else None  # one layer of the headline alone (profiles)
    if want("headline") or args.traffic_probe or sub:
        w1, w2 = dev(c3["w1"]), dev(c3["w2"])
        W1p0, W2p0 = B.binarize_pack(w1, 1), B.binarize_pack(w2, 1)
        al1, al2 = B.alpha_mean_abs(w1), B.alpha_mean_abs(w2)
        del w2
        ws_bytes = B.workspace_bytes(B.OP_BINARY_FC, (Bt, F0, F1))
        x0 = dev(c3["x"])
        step_bytes = (x0.numel() * 4 + ws_bytes + Bt * F1 * 4 + Bt * F2 * 4 + W1p0.numel() * 8 + W2p0.numel() * 8)
        # enough sets that the smallest single-kernel timing below (the second layer's pack: its
        # fp32 input and its packed output) also walks through more than the memory-side cache
        nsets = nsets_for(Bt * F1 * 4 + Bt * F1 // 8, cap=128)
        xs = [x0] + [x0.clone() for _ in range(nsets - 1)]
        W1s = [W1p0] + [W1p0.clone() for _ in range(nsets - 1)]
        W2s = [W2p0] + [W2p0.clone() for _ in range(nsets - 1)]
        wss = [u8(ws_bytes) for _ in range(nsets)]
        h1s = [f32(Bt, F1) for _ in range(nsets)]
        h2s = [f32(Bt, F2) for _ in range(nsets)]

        def make_step(i):
            def step():
                B.binary_fc(xs[i], W1s[i], alpha=al1, out=h1s[i], workspace=wss[i])
                B.binary_fc(h1s[i], W2s[i], alpha=al2, out=h2s[i], workspace=wss[i])
            return step

        steps = [make_step(i % nsets) for i in range(K_STEPS)]
        if args.traffic_probe:
            # the copy of known size that calibrates the counters: reads 256 MiB, writes 256 MiB
            src = u8(256 << 20).fill_(1)
            dst = torch.empty_like(src)
            for _ in range(5):
                dst.copy_(src)
            for f in steps:
                f()
            torch.cuda.synchronize()
            print(json.dumps({"traffic_probe": True, "steps": K_STEPS, "copy_bytes_each_way": 256 << 20,
                              "buffer_sets_rotated": int(nsets)}))
            return
        ms_per_step = value = hot_us = eager_ms = None
        lanes_us = {}
        if not sub:
            for i in range(args.warmup):
                steps[i % K_STEPS]()
            torch.cuda.synchronize()
            if args.eager:
                t0 = time.perf_counter()
                for f in steps:
                    f()
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
            else:
                g_steps = graph_of(steps)
                g_steps.replay()  # untimed replay: graph upload
                # K steps may use fewer buffer sets than the rotation has: steps on the other sets
                # push what the untimed replay left in the memory-side cache out again
                for i in range(K_STEPS, nsets):
                    make_step(i)()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                g_steps.replay()
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
                del g_steps
            ms_per_step = dt / K_STEPS * 1e3
            value = (ops1 + ops2) / (dt / K_STEPS) / 1e9

            # cache-hot (one buffer set) and eager (host enqueues every launch) step rates: context
            hot_us, eager_ms = None, None
            if not args.lean:
                hot_us = event_us(graph_of([steps[0]] * K_STEPS).replay, K_STEPS)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for f in steps:
                    f()
                torch.cuda.synchronize()
                eager_ms = (time.perf_counter() - t0) / K_STEPS * 1e3
                # the same K steps with 2 and 4 independent batches in flight (every buffer set
                # has its own workspace; steps that share a set sit on the same lane): what a
                # serving loop that overlaps batches gets out of the same kernels.  Context, not
                # the headline: `value` is the chain of dependent launches above.
                # (at least 200 steps per replay: the fixed cost of a replay with side streams
                # would otherwise weigh on a per-step figure of some twenty microseconds)
                n_l = max(K_STEPS, 200)
                steps_l = [make_step(i % nsets) for i in range(n_l)]
                for lanes in (2, 4):
                    if nsets % lanes == 0:
                        gl = graph_of_lanes(steps_l, lanes)
                        gl.replay()
                        for i in range(n_l, nsets):
                            make_step(i)()
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                        gl.replay()
                        torch.cuda.synchronize()
                        lanes_us[lanes] = (time.perf_counter() - t0) / n_l * 1e6
                        del gl
                del steps_l
            del steps
        else:  # one layer alone: the first layer's outputs must exist for the second
            for i in range(nsets):
                B.binary_fc(xs[i], W1s[i], alpha=al1, out=h1s[i], workspace=wss[i])
            torch.cuda.synchronize()
            del steps

        # the step's kernels one by one, on the same rotating buffers
        Kw0p = ws_bytes // (Bt * 8)  # chunk-padded row length of the packed activations, in words
        xps = [t.view(torch.int64)[: Bt * Kw0p].view(Bt, Kw0p) for t in wss]
        Kw1 = F1 // 64
        h1ps = [t.view(torch.int64)[: Bt * Kw1].view(Bt, Kw1) for t in wss]
        gemm1_us = pack1_us = fc1_us = gemm2_us = pack2_us = fc2_us = float("nan")
        gemm1_name = pack1_name = gemm2_name = pack2_name = ""
        if sub != "fc2":
            gemm1_us, gemm1_name = rotating_us([(lambda i=i: B.binary_fc_packed(
                xps[i], F0, W1s[i], alpha=al1, mode="f32", out=h1s[i])) for i in range(nsets)])
            pack1_us, pack1_name = rotating_us([(lambda i=i: B.binarize_pack(xs[i], 1, out=xps[i])) for i in range(nsets)])
            fc1_us, _ = rotating_us([(lambda i=i: B.binary_fc(xs[i], W1s[i], alpha=al1, out=h1s[i], workspace=wss[i]))
                                     for i in range(nsets)])
        if sub != "fc1":
            gemm2_us, gemm2_name = rotating_us([(lambda i=i: B.binary_fc_packed(
                h1ps[i], F1, W2s[i], alpha=al2, mode="f32", out=h2s[i])) for i in range(nsets)])
            pack2_us, pack2_name = rotating_us([(lambda i=i: B.binarize_pack(h1s[i], 1, out=h1ps[i])) for i in range(nsets)])
            fc2_us, _ = rotating_us([(lambda i=i: B.binary_fc(h1s[i], W2s[i], alpha=al2, out=h2s[i], workspace=wss[i]))
                                     for i in range(nsets)])
        gemm1_bytes = Bt * (F0 // 8) + F1 * (F0 // 8) + Bt * F1 * 4   # packed x, packed W1 in; fp32 out
        gemm2_bytes = Bt * (F1 // 8) + F2 * (F1 // 8) + Bt * F2 * 4
        pack1_bytes = Bt * F0 * 4 + Bt * (F0 // 8)
        pack2_bytes = Bt * F1 * 4 + Bt * (F1 // 8)
        roofline = roofline_block(gemm1_name, gemm1_us, binops=ops1, nbytes=gemm1_bytes)
        traffic, tsrc = None, None
        tpath = os.path.join(ROOT, "profiles", "traffic_fc1_gemm_config3.txt")
        if os.path.exists(tpath):  # scaled FETCH_SIZE + WRITE_SIZE of this kernel, from its rocprofv3 --pmc runs
            for ln in open(tpath):
                if ln.startswith("hbm_bytes_per_launch:"):
                    traffic = int(ln.split(":")[1])
                    tsrc = "profiles/traffic_fc1_gemm_config3.txt (rocprofv3 --pmc, not measured in this run)"
        roofline["traffic"] = traffic
        roofline["traffic_source"] = tsrc
        kernels = {}
        if sub != "fc2":
            kernels["fc1_pack"] = roofline_block(pack1_name, pack1_us, nbytes=pack1_bytes)
            kernels["fc1_gemm"] = dict(roofline)
        if sub != "fc1":
            kernels["fc2_pack"] = roofline_block(pack2_name, pack2_us, nbytes=pack2_bytes)
            kernels["fc2_gemm"] = roofline_block(gemm2_name, gemm2_us, binops=ops2, nbytes=gemm2_bytes)
        # the same GEMMs on the xor/popcount engine (the benchmark spec's VALU target names it)
        for tag, Wl, xl, hl, fin, al_, ops_, nb in (() if (args.lean or sub) else (
                ("fc1", W1s, xps, h1s, F0, al1, ops1, gemm1_bytes), ("fc2", W2s, h1ps, h2s, F1, al2, ops2, gemm2_bytes))):
            us_, nm_ = with_tune({7: 1}, lambda: rotating_us([(lambda i=i: B.binary_fc_packed(
                xl[i], fin, Wl[i], alpha=al_, mode="f32", out=hl[i])) for i in range(nsets)], reps=60))
            kernels[tag + "_gemm_popcount_engine"] = add_measured_peak(roofline_block(nm_, us_, binops=ops_, nbytes=nb))
        # the two layers handing packed sign bits to each other instead of fp32 activations
        bits1 = None if (args.lean or sub) else [B.binary_fc_packed(xps[i], F0, W1s[i], alpha=al1, mode="bits")
                                                 for i in range(nsets)]

        def chain_bits(i):
            def run():
                B.binarize_pack(xs[i], 1, out=xps[i])
                B.binary_fc_packed(xps[i], F0, W1s[i], alpha=al1, mode="bits", out=bits1[i])
                B.binary_fc_packed(bits1[i], F1, W2s[i], alpha=al2, mode="f32", out=h2s[i])
            return run

        chain_bits_us = None if (args.lean or sub) else rotating_us([chain_bits(i) for i in range(nsets)])[0]
        if sub:  # a phase line, not the benchmark line
            roofline = roofline_block(gemm2_name, gemm2_us, binops=ops2, nbytes=gemm2_bytes) if sub == "fc2" else roofline
        line.update({"value": value, "ms_per_step": ms_per_step,
                     "dtype": "f32 in -> sign bits (u64 words) -> %s -> f32 out" % roofline["dtype"],
                     "config": {"workload": "config3: binary FC pair, batch 256, 9216 -> 4096 -> 4096, fp32 in, alpha per "
                                            "output row, fp32 out (GEMM views 256 x 4096 x 9216 and 256 x 4096 x 4096)",
                                "step": "bmx_binary_fc (pack + xnor GEMM + alpha) on x, then bmx_binary_fc on its fp32 output",
                                "kernels": [pack1_name, gemm1_name, pack2_name, gemm2_name],
                                "timed_region": "K eager steps" if args.eager else "one replay of a HIP graph holding the K steps",
                                "buffer_sets_rotated": int(nsets), "bytes_per_buffer_set": int(step_bytes),
                                "ms_per_step_cache_hot": None if hot_us is None else hot_us * 1e-3,
                                "ms_per_step_eager": eager_ms,
                                "fc1_call_us_hbm_resident": fc1_us, "fc2_call_us_hbm_resident": fc2_us,
                                "step_us_via_packed_sign_bits_between_layers": chain_bits_us,
                                "step_us_with_independent_batches_in_flight": {str(k): v for k, v in lanes_us.items()} or None,
                                "gops_fc1_call": ops1 / fc1_us / 1e3, "gops_fc2_call": ops2 / fc2_us / 1e3,
                                "phase": args.phase},
                     "roofline": roofline, "kernels": kernels})
        del xs, W1s, W2s, wss, h1s, h2s, xps, h1ps, bits1
        torch.cuda.empty_cache()

        del w1
        torch.cuda.empty_cache()

    run_others = not args.no_other_configs

    if want("packs") and run_others:
        # weight pack of the first layer (151 MB fp32 -> 4.7 MB), eight copies rotating, and a
        # 1 GiB row pack: the sustained HBM figures of the pack kernel
        w1 = dev(c3["w1"])
        W1p0 = B.binarize_pack(w1, 1)
        wcopies = [w1] + [w1.clone() for _ in range(7)]
        us_, nm_ = rotating_us([(lambda i=i: B.binarize_pack(wcopies[i], 1, out=W1p0)) for i in range(8)], reps=32)
        other["config3_weight_pack_4096x9216"] = roofline_block(nm_, us_, nbytes=w1.numel() * 4 + W1p0.numel() * 8)
        del wcopies, w1
        big = f32(8192, 32768).normal_()
        bigp = B.binarize_pack(big, 1)
        us_, nm_ = rotating_us([lambda: B.binarize_pack(big, 1, out=bigp)], reps=5)
        other["row_pack_1GiB"] = roofline_block(nm_, us_, nbytes=big.numel() * 4 + bigp.numel() * 8)
        del big, bigp
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ a chip-filling xnor GEMM
    if want("biggemm") and run_others:
        # 8192^3 on packed operands (no configuration of the set: the matrix-core kernel away from
        # launch costs).  16 MB of operands, 268 MB of int32 results per launch, four sets rotating.
        Mb = Nb = Kb = 8192
        gen = torch.Generator(device="cuda").manual_seed(8192)
        Ab = [torch.randint(-2 ** 62, 2 ** 62, (Mb, Kb // 64), dtype=torch.int64, device="cuda", generator=gen) for _ in range(4)]
        Bb = [torch.randint(-2 ** 62, 2 ** 62, (Nb, Kb // 64), dtype=torch.int64, device="cuda", generator=gen) for _ in range(4)]
        Cb = [i32(Mb, Nb) for _ in range(4)]
        us_, nm_ = rotating_us([(lambda i=i: B.xnor_gemm(Ab[i], Bb[i], Kb, out=Cb[i])) for i in range(4)], reps=12)
        blk = roofline_block(nm_, us_, binops=2.0 * Mb * Nb * Kb, nbytes=2 * Mb * Kb // 8 + Mb * Nb * 4)
        blk["note"] = ("268 MB of results per launch: 34 us of HBM time at the peak rate beside 109 us of matrix-core "
                       "time; the shader clock under this load was measured at 1.8 - 2.0 GHz, against the 2.4 GHz "
                       "the peak assumes")
        other["xnor_gemm_8192x8192x8192_i32_out"] = blk
        del Ab, Bb, Cb
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ configuration 1
    if want("config1") and run_others:
        c1 = synth.config1()
        n1 = nsets_for(64 * 512 * 4 + 256 * 8 * 8 + 64 * 256 * 4 + 4096, cap=400)
        a1 = [dev(c1["a"]) for _ in range(n1)]
        W1p = [B.binarize_pack(dev(c1["w_kn"]), 0) for _ in range(n1)]
        o1 = [i32(64, 256) for _ in range(n1)]
        ws1 = [u8(B.workspace_bytes(B.OP_BINARY_FC, (64, 512, 256))) for _ in range(n1)]
        us_, nm_ = rotating_us([(lambda i=i: B.binary_fc(a1[i], W1p[i], integer_out=True, out=o1[i], workspace=ws1[i]))
                                for i in range(n1)])
        # (fp32 activations in, packed weights in, int32 out: what the one-launch form moves)
        blk = roofline_block(nm_, us_, binops=2.0 * 64 * 256 * 512, nbytes=64 * 512 * 4 + 256 * 64 + 64 * 256 * 4)
        blk["note"] = ("whole call in one launch (sign bits of a batch row in LDS, xor + popcount per output feature); "
                       "13 ns of arithmetic behind a launch and two trips to memory")
        two_us, two_nm = with_tune({15: 1}, lambda: rotating_us(
            [(lambda i=i: B.binary_fc(a1[i], W1p[i], integer_out=True, out=o1[i], workspace=ws1[i])) for i in range(n1)]))
        blk["general_path_two_launches"] = {"kernel": two_nm, "call_us": two_us}
        other["config1_fc_call_64x256x512"] = blk
        del a1, W1p, o1, ws1

    # ------------------------------------------------------------------ convolutions (configs 2, 4)
    def conv_config(tag, c, popcount_path):
        x_h, w_h = c["x"], c["w"]
        N, C, H, W = x_h.shape
        O, _, KH, KW = w_h.shape
        stride, pad = c["stride"], c["pad"]
        Ho, Wo = B.conv_out_hw(H, W, KH, KW, stride, pad)
        binops = 2.0 * O * N * Ho * Wo * C * KH * KW
        w = dev(w_h)
        Wp0, alpha = B.pack_conv_weights(w), B.alpha_mean_abs(w)
        ws_bytes = B.workspace_bytes(B.OP_BINARY_CONV2D, (N, C, H, W, O, KH, KW, stride, pad))
        Cw = (C + 63) // 64
        out_bytes = N * O * Ho * Wo * 4
        # (enough sets that each kernel timed alone, the pack on x and the packed image, the
        # convolution on the packed image and the output, also walks through more than the cache)
        n = nsets_for(min(x_h.nbytes + ws_bytes, ws_bytes + out_bytes + Wp0.numel() * 8), cap=128)
        x0 = dev(x_h)
        xs = [x0] + [x0.clone() for _ in range(n - 1)]
        Wps = [Wp0] + [Wp0.clone() for _ in range(n - 1)]
        wss = [u8(ws_bytes) for _ in range(n)]
        outs = [f32(N, O, Ho, Wo) for _ in range(n)]
        xps = [t.view(torch.int64)[: N * (H + 2 * pad) * (W + 2 * pad) * Cw].view(N, H + 2 * pad, W + 2 * pad, Cw)
               for t in wss]
        call_us, _ = rotating_us([(lambda i=i: B.binary_conv2d(xs[i], Wps[i], O, KH, KW, stride, pad, alpha=alpha,
                                                               out=outs[i], workspace=wss[i])) for i in range(n)])
        conv_calls = [(lambda i=i: B.binary_conv2d_packed(xps[i], C, Wps[i], O, KH, KW, stride, pad, alpha=alpha,
                                                          out=outs[i])) for i in range(n)]
        conv_us, conv_name = rotating_us(conv_calls)
        pack_us, pack_name = rotating_us([(lambda i=i: B.pack_nchw(xs[i], pad, out=xps[i])) for i in range(n)])
        conv_bytes = xps[0].numel() * 8 + Wp0.numel() * 8 + out_bytes
        pack_bytes = x_h.nbytes + xps[0].numel() * 8
        d = {"call_us_hbm_resident": call_us, "gops_call": binops / call_us / 1e3, "buffer_sets_rotated": n,
             "conv_kernel": roofline_block(conv_name, conv_us, binops=binops, nbytes=conv_bytes),
             "pack_kernel": roofline_block(pack_name, pack_us, nbytes=pack_bytes)}
        if not args.lean:
            us_, nm_ = with_tune({5: popcount_path}, lambda: rotating_us(conv_calls, reps=60))
            d["conv_kernel_popcount_engine"] = add_measured_peak(roofline_block(nm_, us_, binops=binops, nbytes=conv_bytes))
        other[tag] = d

    if want("config2") and run_others:
        conv_config("config2_conv3x3_16x64x56x56_64filters", synth.config2(), 1)
    if want("config2") and run_others and not args.lean:
        # three configuration-2 blocks in a row (Sec. 2: QActivation -> QConvolution -> BatchNorm):
        # through fp32 feature maps (pack + convolution each) or handing the next layer its packed
        # image (one pack, the BatchNorm folded into a per-channel threshold)
        n = nsets_for(2 * 12845056 + 430592 * 3)
        x_h = synth.config2()["x"]
        xc = [dev(x_h) for _ in range(n)]
        wc = [f32(64, 64, 3, 3).normal_() for _ in range(3)]
        Wc = [B.pack_conv_weights(t) for t in wc]
        alc = [B.alpha_mean_abs(t) for t in wc]
        thc = f32(64).normal_()
        wsc = [u8(B.workspace_bytes(B.OP_BINARY_CONV2D, (16, 64, 56, 56, 64, 3, 3, 1, 1))) for _ in range(n)]
        fa = [f32(16, 64, 56, 56) for _ in range(n)]
        fb = [f32(16, 64, 56, 56) for _ in range(n)]
        xpc = [B.pack_nchw(xc[i], 1) for i in range(n)]
        ia = [torch.empty_like(xpc[0]) for _ in range(n)]
        ib = [torch.empty_like(xpc[0]) for _ in range(n)]
        ops_c = 3 * 2.0 * 64 * 16 * 56 * 56 * 576

        def blocks_fp32(i):
            def run():
                B.binary_conv2d(xc[i], Wc[0], 64, 3, 3, 1, 1, alpha=alc[0], out=fa[i], workspace=wsc[i])
                B.binary_conv2d(fa[i], Wc[1], 64, 3, 3, 1, 1, alpha=alc[1], out=fb[i], workspace=wsc[i])
                B.binary_conv2d(fb[i], Wc[2], 64, 3, 3, 1, 1, alpha=alc[2], out=fa[i], workspace=wsc[i])
            return run

        def blocks_packed(i):
            def run():
                B.pack_nchw(xc[i], 1, out=xpc[i])
                B.binary_conv2d_bits(xpc[i], 64, Wc[0], 64, 3, 3, 1, 1, alpha=alc[0], thr=thc, out_pad=1, out=ia[i])
                B.binary_conv2d_bits(ia[i], 64, Wc[1], 64, 3, 3, 1, 1, alpha=alc[1], thr=thc, out_pad=1, out=ib[i])
                B.binary_conv2d_packed(ib[i], 64, Wc[2], 64, 3, 3, 1, 1, alpha=alc[2], out=fa[i])
            return run

        us_a, _ = rotating_us([blocks_fp32(i) for i in range(n)], reps=60)
        us_b, _ = rotating_us([blocks_packed(i) for i in range(n)], reps=60)
        other["config2_three_blocks_in_a_row"] = {"via_fp32_feature_maps_us": us_a, "via_packed_images_us": us_b,
                                                  "gops_via_fp32": ops_c / us_a / 1e3, "gops_via_packed": ops_c / us_b / 1e3}
        del xc, fa, fb, xpc, ia, ib, wsc

    if want("config4") and run_others:
        conv_config("config4_conv3x3_64x256x14x14_256filters_stride1", synth.config4(stride=1), 1)
        conv_config("config4_conv3x3_64x256x14x14_256filters_stride2", synth.config4(stride=2), 1)

    # ------------------------------------------------------------------ configuration 5
    if want("config5") and run_others:
        c5 = synth.config5()
        M5, N5, K5 = 1024, 1024, 4096
        wsb = B.workspace_bytes(B.OP_QUANT_GEMM, (M5, N5, K5, 2, 1))
        n = nsets_for(2 * M5 * K5 * 4 + wsb + M5 * N5 * 4)
        a5 = [dev(c5["a"]) for _ in range(n)]
        w5 = [dev(c5["w"]) for _ in range(n)]
        ws5 = [u8(wsb) for _ in range(n)]
        o5 = [f32(M5, N5) for _ in range(n)]
        calls5 = [(lambda i=i: B.quant_gemm(a5[i], w5[i], 2, want_int=False, out_float=o5[i], workspace=ws5[i]))
                  for i in range(n)]
        us_, nm_ = rotating_us(calls5, reps=60)
        binops5 = 2.0 * 2 * M5 * N5 * K5            # two plane pairs
        d = {"call_us_hbm_resident": us_, "gops_call": binops5 / us_ / 1e3, "buffer_sets_rotated": n,
             "note": "whole call: quantise + plane pack of a and sign pack of w (one launch), then the plane GEMM",
             # priced as if the GEMM kernel had the whole call to itself (the split per kernel is in profiles/)
             "gemm_kernel_upper_bound": roofline_block(nm_, us_, binops=binops5, nbytes=3 * M5 * K5 // 8 + M5 * N5 * 4,
                                                       mfma_flops=2.0 * M5 * N5 * K5),
             "whole_call_vs_hbm": roofline_block("quant_pack_kernel + " + nm_, us_, nbytes=2 * M5 * K5 * 4 + M5 * N5 * 4)}
        if not args.lean:
            us_, nm_ = with_tune({7: 1}, lambda: rotating_us(calls5, reps=40))
            d["call_popcount_engine"] = add_measured_peak(roofline_block(nm_, us_, binops=binops5,
                                                                         nbytes=3 * M5 * K5 // 8 + M5 * N5 * 4))
        other["config5_quant_gemm_2bit_x_1bit_1024x1024x4096"] = d
        del a5, w5, ws5, o5

    # ------------------------------------------------------------------ the paper's Sec. 3.1 workloads
    if want("sec31") and run_others:
        def conv_call(cin, cout, k):
            hw = 8 + k - 1
            wq = f32(cout, cin, k, k).normal_()
            Wq, alq = B.pack_conv_weights(wq), B.alpha_mean_abs(wq)
            wsb = B.workspace_bytes(B.OP_BINARY_CONV2D, (200, cin, hw, hw, cout, k, k, 1, 0))
            n = nsets_for(200 * cin * hw * hw * 4 + wsb + 200 * cout * 64 * 4, cap=64)
            xq = [f32(200, cin, hw, hw).normal_() for _ in range(n)]
            oq = [f32(200, cout, 8, 8) for _ in range(n)]
            wsq = [u8(wsb) for _ in range(n)]
            us, nm = rotating_us([(lambda i=i: B.binary_conv2d(xq[i], Wq, cout, k, k, 1, 0, alpha=alq, out=oq[i],
                                                               workspace=wsq[i])) for i in range(n)], reps=60)
            ops = 2.0 * cout * 12800 * k * k * cin
            return {"call_us_hbm_resident": us, "gops_call": ops / us / 1e3, "conv_kernel": nm}

        # 5x5 kernels, 64 filters, batch 200, 8x8 outputs: GEMM view M = 64, N = 12800, K = 25 * C_in
        for cin in (64, 128, 256, 512):
            other["paper_sec3_1_conv5x5_cin%d_call" % cin] = conv_call(cin, 64, 5)
        for cout in (16, 128, 512):
            other["paper_sec3_1_conv5x5_cin256_filters%d_call" % cout] = conv_call(256, cout, 5)
        for k in (1, 3, 7):
            other["paper_sec3_1_conv%dx%d_cin256_call" % (k, k)] = conv_call(256, 64, k)

    # ------------------------------------------------------------------ CPU oracle beside it
    if not args.no_cpu_baseline and args.phase == "all":
        import oracle
        gomp = None
        try:
            gomp = ctypes.CDLL("libgomp.so.1")
        except OSError:
            pass
        cores = oracle.num_threads()

        def timed(fn, budget_s, max_reps=1000):
            fn()  # page in
            reps, t = 0, 0.0
            while t < budget_s and reps < max_reps:
                t1 = time.perf_counter()
                fn()
                t += time.perf_counter() - t1
                reps += 1
            return t / reps, reps

        def entry(ops, fn, budget_s, what):
            s, reps = timed(fn, budget_s)
            return {"value": ops / s / 1e9, "unit": "GOPS", "cores": cores, "seconds_per_pass": s,
                    "sample": "%d full passes of %s" % (reps, what)}

        a1h, a2h = oracle.alpha_mean_abs(c3["w1"]), oracle.alpha_mean_abs(c3["w2"])

        def chain():
            _, r1 = oracle.binary_fc(c3["x"], c3["w1"], a1h)
            oracle.binary_fc(r1, c3["w2"], a2h)

        cpu = entry(ops1 + ops2, chain, 6.0, "the config-3 layer pair")
        cpu["kind"] = "oracle"
        per = {}
        c1 = synth.config1()
        w1t = c1["w_kn"].T.copy()
        per["config1"] = entry(2.0 * 64 * 256 * 512, lambda: oracle.binary_fc(c1["a"], w1t), 0.5, "the config-1 layer")
        c2 = synth.config2()
        al2h = oracle.alpha_mean_abs(c2["w"])
        ops_c2 = 2.0 * 64 * 50176 * 576
        per["config2"] = entry(ops_c2, lambda: oracle.binary_conv2d(c2["x"], c2["w"], 1, 1, al2h), 2.0, "the config-2 layer")
        for s4 in (1, 2):
            c4 = synth.config4(stride=s4)
            al4h = oracle.alpha_mean_abs(c4["w"])
            ho = 14 // s4
            per["config4_stride%d" % s4] = entry(2.0 * 256 * 64 * ho * ho * 2304,
                                                 lambda: oracle.binary_conv2d(c4["x"], c4["w"], s4, 1, al4h), 2.0,
                                                 "the config-4 layer, stride %d" % s4)
        c5 = synth.config5()
        per["config5"] = entry(2.0 * 2 * 1024 * 1024 * 4096, lambda: oracle.quant_gemm(c5["a"], c5["w"], 2), 2.0,
                               "the config-5 GEMM (2 plane pairs counted)")
        if gomp is not None:  # one thread, for the two small configurations
            gomp.omp_set_num_threads(1)
            try:
                e = entry(2.0 * 64 * 256 * 512, lambda: oracle.binary_fc(c1["a"], w1t), 0.3, "the config-1 layer")
                e["cores"] = 1
                per["config1_one_thread"] = e
                e = entry(ops_c2, lambda: oracle.binary_conv2d(c2["x"], c2["w"], 1, 1, al2h), 1.0, "the config-2 layer")
                e["cores"] = 1
                per["config2_one_thread"] = e
            finally:
                gomp.omp_set_num_threads(cores)
        cpu["per_config"] = per

        # the paper's own method on the same host cores (Sec. 2.2.1: xnor + popcount over 64-bit
        # words, OpenMP), GEMM only, packing not timed, as the paper times it (Sec. 3.1)
        try:
            so = os.path.join(tempfile.mkdtemp(prefix="bmx_host_xnor_"), "host_xnor.so")
            subprocess.check_call(["gcc", "-O3", "-march=native", "-fopenmp", "-fPIC", "-shared",
                                   os.path.join(ROOT, "bench_host_xnor.c"), "-o", so])
            hx = ctypes.CDLL(so)
            hx.host_xnor_gemm.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_long] * 4 + [ctypes.c_int]
            hx.host_xnor_threads.restype = ctypes.c_int
            xn = {}
            host_threads = int(hx.host_xnor_threads())
            for tag, a_f, b_f in (("config3_fc1_gemm_256x4096x9216", c3["x"], c3["w1"]),
                                  ("config2_gemm_view_64x50176x576", c2["w"].reshape(64, -1),
                                   oracle.im2col(c2["x"], 3, 3, 1, 1))):
                Ap, Bp = oracle.binarize_pack(a_f, 1), oracle.binarize_pack(b_f, 1)
                M_, N_, Kw_, K_ = Ap.shape[0], Bp.shape[0], Ap.shape[1], a_f.shape[1]
                Cc = np.empty((M_, N_), dtype=np.int32)
                for thr_ in (host_threads, 1):
                    s, reps = timed(lambda: hx.host_xnor_gemm(Ap.ctypes.data, Bp.ctypes.data, Cc.ctypes.data,
                                                              M_, N_, Kw_, K_, thr_), 1.0)
                    xn[tag + ("_one_thread" if thr_ == 1 else "")] = {
                        "value": 2.0 * M_ * N_ * K_ / s / 1e9, "unit": "GOPS", "cores": thr_, "seconds_per_pass": s,
                        "sample": "%d passes of the GEMM on packed 64-bit words, packing not timed" % reps}
            cpu["host_xnor_popcount_gemm"] = dict(xn, kind="uint64 xor + popcount GEMM with OpenMP (bench_host_xnor.c): "
                                                            "the paper's method on this host, context only, not the oracle")
        except (OSError, subprocess.CalledProcessError) as e:  # no host compiler: the figure is context only
            cpu["host_xnor_popcount_gemm"] = {"error": str(e)}

    if "value" not in line:  # a phase without the headline: the line still parses
        line.update({"value": None, "ms_per_step": None, "dtype": None, "config": {"workload": "phase " + args.phase},
                     "roofline": None})
    line["valu_probe"] = probe
    line["cpu_baseline"] = cpu
    line["other_configs"] = other or None
    print(json.dumps(line).replace('NaN', 'null'))


if __name__ == "__main__":
    main()
