"""Build libbmx.so (hand-written HIP for gfx950) in-tree with hipcc."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbmx.so")
SOURCES = ["bmx_api.hip", "pack.hip", "gemm.hip", "gemm_mfma.hip", "gemm_fp4.hip", "conv.hip", "conv_mfma.hip", "fc_small.hip", "probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed-fp32 VALU forms are kept out of generated code on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # host-pass errors inside kernel bodies are reported, not deferred (deferred, they leave the
         # kernel's host stub undefined without a word)
         "-fno-gpu-defer-diag",
         "-Wno-unused-command-line-argument"]


def _stale(out, deps):
    if not os.path.exists(out):
        return True
    t = os.path.getmtime(out)
    return any(os.path.getmtime(d) > t for d in deps)


def device_asm(src):
    """Path of the gfx950 assembly that -save-temps leaves next to the object of `src`."""
    return os.path.join(BUILD, os.path.splitext(src)[0] + "-hip-amdgcn-amd-amdhsa-gfx950.s")


def check_scalar_loads():
    """Scan the compiled device code of every source for registers of an inline-asm scalar
    load that are touched while the load is still in flight (see isa_check.py; the kernels have
    no such load, the scan guards against one coming back)."""
    try:
        from . import isa_check
    except ImportError:  # run as a script
        sys.path.insert(0, HERE)
        import isa_check
    for src in SOURCES:
        path = device_asm(src)
        s = os.path.join(CSRC, src)
        if _stale(path, [s]):  # e.g. a fresh checkout: emit the device assembly alone
            os.makedirs(BUILD, exist_ok=True)
            subprocess.check_call([HIPCC] + FLAGS + ["-S", "--cuda-device-only", s, "-o", path],
                                  stderr=subprocess.DEVNULL)
        bad = isa_check.scan(path)
        if bad:
            raise RuntimeError("in-flight scalar load hazard in %s:\n%s" % (src, isa_check.report(bad)))


def check_codegen():
    """Properties of the generated code that a harmless-looking source change can lose without
    any test failing, only the clock: no kernel spills vector registers (the 64 x 64 tile of the
    register-operand matrix-core GEMM aside, which parks a dozen loop-invariant values); no
    kernel touches scratch memory (the same kernel and one convolution form of the popcount
    GEMM aside: a small array indexed at run time lands there, and every scratch access also
    waits for all stores issued before it, which cost the K-split GEMM 0.7 us per launch); and
    the convolution kernel with its filters in LDS reads each MFMA's filter operand with one
    ds_read_b128 (split into dword pairs, the rows meet four ways on the banks)."""
    import re
    try:
        from . import isa_check
    except ImportError:
        sys.path.insert(0, HERE)
        import isa_check
    for src in SOURCES:
        for name, nbytes in isa_check.scratch_bytes(device_asm(src)).items():
            known = "gemm_mfma_kernelILi2ELi2E" in name or "gemm_kernelILi16ELi32ELb0ELb0ELb1E" in name
            if nbytes and not known:
                raise RuntimeError("%s: kernel %s uses %d bytes of scratch memory per lane" % (src, name, nbytes))
        for name, (spills, ops) in isa_check.kernel_stats(device_asm(src)).items():
            allowed = 16 if "gemm_mfma_kernelILi2ELi2E" in name else 0
            if spills > allowed:
                raise RuntimeError("%s: kernel %s spills %d vector registers" % (src, name, spills))
            m = re.search(r"conv_mfma_ws_kernelILi(\d+)ELi(\d+)E", name)
            if m and ops["ds_read_b128"] < int(m.group(1)) * int(m.group(2)):
                raise RuntimeError("%s: kernel %s reads its filter operands with %d ds_read_b128, "
                                   "expected %d" % (src, name, ops["ds_read_b128"],
                                                    int(m.group(1)) * int(m.group(2))))


def build(force=True, verbose=False):
    """Compile every translation unit, verify the hand-placed scalar loads in the generated
    code, and link the shared library.  Returns its path."""
    os.makedirs(BUILD, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".h", ".hpp"))]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "bmx.h"))

    def compile_one(src):
        s = os.path.join(CSRC, src)
        o = os.path.join(BUILD, src + ".o")
        if force or _stale(o, [s] + headers):
            cmd = [HIPCC] + FLAGS + ["-save-temps=obj", "-c", s, "-o", o]
            if verbose:
                print(" ".join(cmd), flush=True)
            r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            if r.returncode != 0:
                raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stdout))
            warn = [l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip()]
            if verbose and warn:
                print("\n".join(warn))
        return o

    with ThreadPoolExecutor(max_workers=min(4, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    check_scalar_loads()
    check_codegen()
    # (-z defs: an undefined symbol, e.g. a kernel stub the host pass dropped, fails the link here
    # instead of the first call)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,-z,defs"] + objs + ["-o", LIB]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
