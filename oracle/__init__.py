"""ctypes front end of the CPU oracle (``bmx_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by
the ``cpu_baseline`` leg of ``bench.py``.  Nothing in the product package imports it,
and it imports nothing from the product package.

All arrays are host numpy arrays; every function returns freshly allocated outputs.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bmx_oracle.cpp")


def _cpu_tag():
    """The oracle is compiled with -march=native, so the library is keyed by the host's
    instruction-set flags: a machine with another CPU builds its own copy."""
    import hashlib
    flags = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("flags"):
                flags = line
                break
    except OSError:
        pass
    return hashlib.sha1(flags.encode()).hexdigest()[:10]


# BMX_ORACLE_SANITIZE=1 builds and loads a second copy of the oracle with AddressSanitizer and
# UndefinedBehaviorSanitizer (host code only; run the CPU tests with
# LD_PRELOAD=$(gcc -print-file-name=libasan.so) so that the runtime is loaded first).
_SANITIZE = os.environ.get("BMX_ORACLE_SANITIZE", "") not in ("", "0")
_LIB = os.path.join(_HERE, "libbmx_oracle.%s%s.so" % (_cpu_tag(), ".san" if _SANITIZE else ""))
_lib = None

_i64 = ctypes.c_int64
_int = ctypes.c_int
_p = ctypes.c_void_p


def build(force=False):
    """Compile the oracle with the host compiler (g++, OpenMP)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["g++", "-O3", "-march=native", "-fopenmp", "-std=c++17", "-fPIC", "-shared",
           _SRC, "-o", _LIB]
    if _SANITIZE:
        cmd[1:2] = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    "-fno-omit-frame-pointer"]
    subprocess.check_call(cmd)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_num_threads.restype = _int
    return _lib


def _ptr(a):
    return _p(a.ctypes.data) if a is not None else _p(0)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _rows(a):
    """A 2-D float32 array and its leading dimension in elements.  A view whose rows are further
    apart than their length (x[:, :K] of a wider buffer) is passed as it is, so that the C
    functions' leading-dimension arguments are exercised; anything else is made contiguous."""
    a = np.asarray(a, dtype=np.float32)
    if a.ndim == 2 and a.shape[0] > 1 and a.strides[1] == 4 and a.strides[0] % 4 == 0 \
            and a.strides[0] >= 4 * a.shape[1]:
        return a, a.strides[0] // 4
    a = np.ascontiguousarray(a)
    return a, (a.shape[1] if a.ndim == 2 else a.size)


def num_threads():
    return int(lib().orc_num_threads())


def sign(x):
    x = _f32(x)
    out = np.empty_like(x)
    lib().orc_sign(_ptr(x), _i64(x.size), _ptr(out))
    return out


def binarize_pack(x, pack_dim=1, out_ld_words=None, fill=0):
    """x: 2-D float32.  Returns uint64 [R, out_ld_words]; words past ceil(K/64) keep ``fill``."""
    x, ldx = _rows(x)
    rows, cols = x.shape
    R, K = (rows, cols) if pack_dim else (cols, rows)
    Kw = (K + 63) // 64
    ld = Kw if out_ld_words is None else int(out_ld_words)
    out = np.full((R, ld), fill, dtype=np.uint64)
    lib().orc_binarize_pack(_ptr(x), _i64(rows), _i64(cols), _i64(ldx), _int(pack_dim),
                            _ptr(out), _i64(ld))
    return out


def unpack_pm1(p, K):
    p = np.ascontiguousarray(p, dtype=np.uint64)
    rows, ld = p.shape
    out = np.empty((rows, K), dtype=np.float32)
    lib().orc_unpack_pm1(_ptr(p), _i64(rows), _i64(K), _i64(ld), _ptr(out))
    return out


def xnor_gemm(A, B, K):
    """A: uint64 [M, lda_w], B: uint64 [N, ldb_w] packed along K.  Returns int32 [M, N]."""
    A = np.ascontiguousarray(A, dtype=np.uint64)
    B = np.ascontiguousarray(B, dtype=np.uint64)
    M, N = A.shape[0], B.shape[0]
    C = np.empty((M, N), dtype=np.int32)
    lib().orc_xnor_gemm(_ptr(A), _i64(A.shape[1]), _ptr(B), _i64(B.shape[1]), _ptr(C), _i64(N),
                        _i64(M), _i64(N), _i64(K))
    return C


def alpha_mean_abs(w):
    w = np.asarray(w, dtype=np.float32)
    w2, ldw = _rows(w if w.ndim == 2 else np.ascontiguousarray(w).reshape(w.shape[0], -1))
    alpha = np.empty(w2.shape[0], dtype=np.float32)
    lib().orc_alpha_mean_abs(_ptr(w2), _i64(w2.shape[0]), _i64(w2.shape[1]), _i64(ldw),
                             _ptr(alpha))
    return alpha


def binary_fc(x, w, alpha=None):
    """x: [batch, in], w: [out, in] float32.  Returns (int32 [batch,out], float32 [batch,out])."""
    (x, ldx), (w, ldw) = _rows(x), _rows(w)
    batch, fin = x.shape
    fout = w.shape[0]
    assert w.shape[1] == fin
    al = None if alpha is None else _f32(alpha)
    oi = np.empty((batch, fout), dtype=np.int32)
    of = np.empty((batch, fout), dtype=np.float32)
    lib().orc_binary_fc(_ptr(x), _i64(ldx), _ptr(w), _i64(ldw), _ptr(al), _i64(batch), _i64(fin),
                        _i64(fout), _ptr(oi), _ptr(of), _i64(fout))
    return oi, of


def conv_out_hw(H, W, KH, KW, stride, pad):
    return (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1


def im2col(x, KH, KW, stride, pad):
    x = _f32(x)
    N, C, H, W = x.shape
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    col = np.empty((N * Ho * Wo, C * KH * KW), dtype=np.float32)
    lib().orc_im2col(_ptr(x), _i64(N), _i64(C), _i64(H), _i64(W), _i64(KH), _i64(KW),
                     _i64(stride), _i64(pad), _ptr(col))
    return col


def binary_conv2d(x, w, stride=1, pad=0, alpha=None):
    """x: NCHW, w: OIHW float32.  Returns (int32 NCHW, float32 NCHW)."""
    x, w = _f32(x), _f32(w)
    N, C, H, W = x.shape
    O, C2, KH, KW = w.shape
    assert C2 == C
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    al = None if alpha is None else _f32(alpha)
    oi = np.empty((N, O, Ho, Wo), dtype=np.int32)
    of = np.empty((N, O, Ho, Wo), dtype=np.float32)
    lib().orc_binary_conv2d(_ptr(x), _i64(N), _i64(C), _i64(H), _i64(W), _ptr(w), _i64(O),
                            _i64(KH), _i64(KW), _i64(stride), _i64(pad), _ptr(al), _ptr(oi),
                            _ptr(of))
    return oi, of


def binary_conv2d_direct(x, w, stride=1, pad=0):
    x, w = _f32(x), _f32(w)
    N, C, H, W = x.shape
    O, _, KH, KW = w.shape
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    oi = np.empty((N, O, Ho, Wo), dtype=np.int32)
    lib().orc_binary_conv2d_direct(_ptr(x), _i64(N), _i64(C), _i64(H), _i64(W), _ptr(w), _i64(O),
                                   _i64(KH), _i64(KW), _i64(stride), _i64(pad), _ptr(oi))
    return oi


def quantize(x, bits):
    """Eq. 1.  Returns (int32 levels, float64 quantised values), same shape as x."""
    x = _f32(x)
    q = np.empty(x.shape, dtype=np.int32)
    v = np.empty(x.shape, dtype=np.float64)
    lib().orc_quantize(_ptr(x), _i64(x.size), _int(bits), _ptr(q), _ptr(v))
    return q, v


def quant_gemm(a, w, bits_a, bits_w=1):
    """a: [M,K] in [0,1], w: [N,K] (bits_w = 1: any sign; bits_w > 1: in [-1,1]).  Returns
    (S int32, out float64, out float32), all [M,N]."""
    (a, lda), (w, ldw) = _rows(a), _rows(w)
    if bits_w != 1:
        M, K = a.shape
        N = w.shape[0]
        assert w.shape[1] == K
        S = np.empty((M, N), dtype=np.int32)
        o64 = np.empty((M, N), dtype=np.float64)
        o32 = np.empty((M, N), dtype=np.float32)
        lib().orc_quant_gemm_kw(_ptr(a), _i64(lda), _int(bits_a), _ptr(w), _i64(ldw), _int(bits_w), _i64(M),
                                _i64(N), _i64(K), _ptr(S), _ptr(o64), _ptr(o32), _i64(N))
        return S, o64, o32
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] == K
    S = np.empty((M, N), dtype=np.int32)
    o64 = np.empty((M, N), dtype=np.float64)
    o32 = np.empty((M, N), dtype=np.float32)
    lib().orc_quant_gemm(_ptr(a), _i64(lda), _int(bits_a), _ptr(w), _i64(ldw), _i64(M), _i64(N),
                         _i64(K), _ptr(S), _ptr(o64), _ptr(o32), _i64(N))
    return S, o64, o32
