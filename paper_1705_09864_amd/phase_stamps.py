"""Where a wave's time goes inside the two kernels that carry the configurations: per-wave
shader-clock stamps at the phase boundaries of gemm_fp4_kernel and conv_mfma_ws_kernel.

The kernels hold the stamps behind BMX_FP4_STAMPS / BMX_WS_STAMPS (compiled out of libbmx.so).
This module builds a second library with both defined (libbmx_stamps.so, beside libbmx.so),
runs one launch of a workload on operands that no cache holds, and prints, per phase, the median
and the 10th and 90th percentile over the launch's waves, in shader clocks.

    python -m paper_1705_09864_amd.phase_stamps --build            (on the build host: hipcc only)
    python -m paper_1705_09864_amd.phase_stamps fc1 fc2 config4 config4s2 config2   (on the GPU)

A profiling aid: nothing in the library, the tests or bench.py depends on it.  The stamped
kernels spend registers and stores on the stamps (at 36 words the convolution kernel then runs
two waves per SIMD instead of three), so their totals are a little above the plain kernels'.
"""
import ctypes
import os
import subprocess
import sys

from . import build as _build

STAMPED = os.path.join(_build.HERE, "libbmx_stamps.so")


def build_stamped():
    out = os.path.join(_build.BUILD, "stamps")
    os.makedirs(out, exist_ok=True)
    objs = []
    for src in _build.SOURCES:
        o = os.path.join(out, src + ".o")
        cmd = [_build.HIPCC] + _build.FLAGS + ["-DBMX_FP4_STAMPS", "-DBMX_WS_STAMPS", "-c", os.path.join(_build.CSRC, src), "-o", o]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stdout))
        objs.append(o)
    subprocess.check_call([_build.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,-z,defs"] + objs + ["-o", STAMPED])
    return STAMPED


def _table(title, rows):
    print(title)
    for name, d in rows:
        if len(d) == 0:
            continue
        d = sorted(d)
        print("  %-52s median %8d  p10 %8d  p90 %8d  max %8d" % (name, d[len(d) // 2], d[len(d) // 10], d[len(d) * 9 // 10], d[-1]))


def main(argv):
    if "--build" in argv:
        print(build_stamped())
        return
    sources = [os.path.join(_build.CSRC, f) for f in os.listdir(_build.CSRC)]
    if _build._stale(STAMPED, sources):  # missing, or older than a source file
        build_stamped()
    import numpy as np
    import torch
    from . import binding as B
    from . import synth
    B.LIB_PATH = STAMPED
    L = B.lib()
    ws_ptr = ctypes.c_void_p.in_dll(L, "_ZN3bmx9ws_stampsE")
    fp4_ptr = ctypes.c_void_p.in_dll(L, "_ZN3bmx10fp4_stampsE")
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    sweep = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")  # four times the memory-side cache

    def cold():
        sweep.add_(1)
        torch.cuda.synchronize()

    def stamps_of(ptr, per_wave, run):
        """One stamped launch of run() on cold operands; the stamps as [waves, per_wave] of uint64
        (rows of waves that wrote nothing dropped)."""
        buf = torch.zeros((1 << 16) * per_wave, dtype=torch.int64, device="cuda")
        run()  # (first call: code upload, not stamped)
        cold()
        ptr.value = buf.data_ptr()
        run()
        torch.cuda.synchronize()
        ptr.value = None
        h = buf.cpu().numpy().view(np.uint64).reshape(-1, per_wave)
        return h[h[:, 0] != 0]

    def diffs(h, a, b):
        ok = (h[:, a] != 0) & (h[:, b] != 0)
        return (h[ok, b].astype(np.int64) - h[ok, a].astype(np.int64)).tolist()

    def fp4_report(tag, run):
        h = stamps_of(fp4_ptr, 8, run)
        _table("%s: %s, %d waves (shader clocks)" % (tag, B.last_kernel(), len(h)),
               [("start -> first segment's loads issued", diffs(h, 0, 1)),
                ("-> first segment in registers", diffs(h, 1, 2)),
                ("-> main loop done", diffs(h, 2, 3)),
                ("-> partial tile written, barrier passed", diffs(h, 3, 4)),
                ("   (barrier -> first group's partials summed)", diffs(h, 4, 7)),
                ("-> reduction done, stores issued", diffs(h, 4, 5)),
                ("-> last store acknowledged", diffs(h, 5, 6)),
                ("wave lifetime", diffs(h, 0, 6))])

    def ws_report(tag, run):
        h = stamps_of(ws_ptr, 16, run)
        rows = [("start -> first pixel loads issued", diffs(h, 0, 1)),
                ("-> filters loaded, expanded, written to LDS", diffs(h, 1, 2)),
                ("-> barrier passed", diffs(h, 2, 3)),
                ("-> first block transposed, next fetch issued", diffs(h, 3, 10)),
                ("-> first block's MFMAs issued", diffs(h, 10, 8)),
                ("-> accumulator chains added", diffs(h, 8, 9)),
                ("-> all blocks done (first: epilogue, stores issued)", diffs(h, 9, 6)),
                ("-> last store acknowledged", diffs(h, 6, 7)),
                ("wave lifetime", diffs(h, 0, 7))]
        _table("%s: %s, %d waves (shader clocks)" % (tag, B.last_kernel(), len(h)), rows)
        ok = (h[:, 4] != 0) & (h[:, 5] != 0)
        if ok.any():  # the 100 MHz counter all parts of the chip share
            t0 = int(h[ok, 4].min())
            start = sorted(((h[ok, 4].astype(np.int64) - t0) * 10).tolist())
            end = sorted(((h[ok, 5].astype(np.int64) - t0) * 10).tolist())
            life = (h[ok, 5].astype(np.int64) - h[ok, 4].astype(np.int64)) * 10
            clk = (h[ok, 7].astype(np.int64) - h[ok, 0].astype(np.int64)) * 1000.0 / np.maximum(life, 1)
            print("  wave start after the first wave's: median %d ns, p90 %d, max %d; wave end: median %d ns, max %d; shader clock %.0f MHz"
                  % (start[len(start) // 2], start[len(start) * 9 // 10], start[-1], end[len(end) // 2], end[-1], float(np.median(clk))))

    for what in [a for a in argv if not a.startswith("-")]:
        if what in ("fc1", "fc2"):
            c3 = synth.config3()
            Bt, F0, F1 = c3["x"].shape[0], c3["x"].shape[1], c3["w1"].shape[0]
            if what == "fc1":
                x, w = dev(c3["x"]), dev(c3["w1"])
            else:
                rng = np.random.default_rng(3)
                x, w = dev(rng.standard_normal((Bt, F1)).astype(np.float32)), dev(c3["w2"])
            xp, Wp, al = B.binarize_pack(x, 1), B.binarize_pack(w, 1), B.alpha_mean_abs(w)
            out = torch.empty((Bt, Wp.shape[0]), dtype=torch.float32, device="cuda")
            fp4_report(what, lambda: B.binary_fc_packed(xp, x.shape[1], Wp, alpha=al, mode="f32", out=out))
        elif what in ("config2", "config4", "config4s2"):
            c = synth.config2() if what == "config2" else synth.config4(stride=2 if what.endswith("s2") else 1)
            x, w = dev(c["x"]), dev(c["w"])
            N, C, H, W = c["x"].shape
            O, _, KH, KW = c["w"].shape
            Wp, al = B.pack_conv_weights(w), B.alpha_mean_abs(w)
            xp = B.pack_nchw(x, c["pad"])
            Ho, Wo = B.conv_out_hw(H, W, KH, KW, c["stride"], c["pad"])
            out = torch.empty((N, O, Ho, Wo), dtype=torch.float32, device="cuda")
            ws_report(what, lambda: B.binary_conv2d_packed(xp, C, Wp, O, KH, KW, c["stride"], c["pad"], alpha=al, out=out))
        else:
            raise SystemExit("unknown workload %r (fc1, fc2, config2, config4, config4s2)" % what)


if __name__ == "__main__":
    main(sys.argv[1:])
