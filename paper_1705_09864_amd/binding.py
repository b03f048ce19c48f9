"""Thin ctypes binding over libbmx.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (PyTorch is used for
device memory and streams, nothing else), passes raw device pointers and sizes through
the C ABI declared in include/bmx.h and raises BmxError on a non-zero status.  There is
no CPU fallback: if the HIP library cannot be loaded the import of this module's
functions fails loudly on first use.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbmx.so")
_lib = None

OP_BINARY_FC, OP_BINARY_CONV2D, OP_QUANT_GEMM, OP_BINARY_CONV2D_BITS, OP_XNOR_GEMM_W32 = 1, 2, 3, 4, 5
EXPORTS = ["bmx_binarize_pack", "bmx_xnor_gemm", "bmx_binary_fc", "bmx_pack_conv_weights",
           "bmx_binary_conv2d", "bmx_quant_gemm", "bmx_alpha_mean_abs", "bmx_pack_nchw",
           "bmx_binary_conv2d_packed", "bmx_workspace_bytes", "bmx_status_string", "bmx_version",
           "bmx_conv_weight_row_words", "bmx_binary_fc_packed", "bmx_tune_set",
           "bmx_binary_conv2d_bits", "bmx_xnor_gemm_count", "bmx_unpack_pm1", "bmx_widen_words32",
           "bmx_xnor_gemm_w32", "bmx_binary_fc_static", "bmx_last_kernel",
           "bmx_probe_valu"]

_i64, _int, _p, _sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t


class BmxError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s failed: %s" % (what, status_string(status)))


def lib():
    """Load libbmx.so (building it first only if no built library is present)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(LIB_PATH)
        L.bmx_binarize_pack.argtypes = [_p, _i64, _i64, _i64, _int, _p, _i64, _p]
        L.bmx_xnor_gemm.argtypes = [_p, _i64, _p, _i64, _p, _i64, _int, _int, _int, _p]
        L.bmx_xnor_gemm_count.argtypes = L.bmx_xnor_gemm.argtypes
        L.bmx_unpack_pm1.argtypes = [_p, _i64, _i64, _i64, _p, _i64, _p]
        L.bmx_unpack_pm1.restype = _int
        L.bmx_xnor_gemm_count.restype = _int
        L.bmx_binary_fc.argtypes = [_p, _i64, _p, _i64, _p, _int, _int, _int, _p, _p, _i64, _p, _sz, _p]
        L.bmx_pack_conv_weights.argtypes = [_p, _int, _int, _int, _int, _p, _p]
        L.bmx_binary_conv2d.argtypes = [_p, _int, _int, _int, _int, _p, _int, _int, _int, _int, _int,
                                        _p, _p, _p, _p, _sz, _p]
        L.bmx_quant_gemm.argtypes = [_p, _i64, _int, _p, _i64, _int, _int, _int, _int, _p, _p, _i64,
                                     _p, _sz, _p]
        L.bmx_alpha_mean_abs.argtypes = [_p, _i64, _i64, _i64, _p, _p]
        L.bmx_workspace_bytes.argtypes = [_int, ctypes.POINTER(_i64), _int]
        L.bmx_workspace_bytes.restype = _sz
        L.bmx_status_string.argtypes = [_int]
        L.bmx_status_string.restype = ctypes.c_char_p
        L.bmx_version.restype = _int
        L.bmx_binary_fc_packed.argtypes = [_p, _i64, _p, _i64, _p, _int, _int, _int, _p, _p, _p, _p, _i64, _p]
        L.bmx_binary_fc_packed.restype = _int
        L.bmx_conv_weight_row_words.argtypes = [_int, _int, _int]
        L.bmx_conv_weight_row_words.restype = _i64
        L.bmx_pack_nchw.argtypes = [_p, _int, _int, _int, _int, _int, _p, _p]
        L.bmx_binary_conv2d_packed.argtypes = [_p, _int, _int, _int, _int, _p, _int, _int, _int, _int,
                                               _int, _p, _p, _p, _p]
        L.bmx_binary_conv2d_bits.argtypes = [_p, _int, _int, _int, _int, _p, _int, _int, _int, _int, _int,
                                             _p, _p, _p, _int, _p, _sz, _p]
        L.bmx_binary_conv2d_bits.restype = _int
        L.bmx_widen_words32.argtypes = [_p, _i64, _i64, _i64, _p, _i64, _p]
        L.bmx_widen_words32.restype = _int
        L.bmx_xnor_gemm_w32.argtypes = [_p, _i64, _p, _i64, _p, _i64, _int, _int, _int, _p, _sz, _p]
        L.bmx_xnor_gemm_w32.restype = _int
        L.bmx_binary_fc_static.argtypes = [_p, _i64, _p, _i64, _p, _int, _int, _int, _p, _p, _i64, _p]
        L.bmx_binary_fc_static.restype = _int
        L.bmx_last_kernel.restype = ctypes.c_char_p
        L.bmx_probe_valu.argtypes = [_int, _int, _p, ctypes.POINTER(_int), _p]
        L.bmx_probe_valu.restype = _int
        L.bmx_tune_set.argtypes = [_int, _int]
        L.bmx_tune_set.restype = _int
        for name in EXPORTS[:9]:
            getattr(L, name).restype = _int
        _lib = L
    return _lib


def status_string(status):
    return lib().bmx_status_string(int(status)).decode()


def last_kernel():
    """Name and launch shape of the last compute kernel this thread launched through the library."""
    return lib().bmx_last_kernel().decode()


def probe_valu(workgroups, iters, out3, stream=None):
    """Launch the register-only xor+popcount chain; returns the wall-clock rate in kHz.  out3 is
    an int64 device tensor of 3 elements (cycles, wall ticks, sink)."""
    _chk(out3, _U64, "probe_valu out3", dense=True)
    khz = _int(0)
    _check(lib().bmx_probe_valu(int(workgroups), int(iters), _ptr(out3), ctypes.byref(khz), _stream(stream)),
           "bmx_probe_valu")
    return int(khz.value)


def version():
    return int(lib().bmx_version())


def _ptr(t):
    return _p(0) if t is None else _p(t.data_ptr())


_F32, _I32, _U64 = (torch.float32,), (torch.int32,), (torch.int64,)


def _chk(t, dtypes, what, dense=False):
    """Host-side guard in front of the C ABI, which sees only a raw address: the tensor must
    live on the GPU, have the element type the call reads or writes, and unit stride along its
    last dimension (rows may be further apart: the leading dimension is passed on).  With
    `dense` the whole tensor must be contiguous (layouts the C call takes no strides for)."""
    if t is None:
        return None
    if not hasattr(t, "data_ptr") or not hasattr(t, "is_cuda"):
        raise ValueError("%s: expected a torch tensor, got %s" % (what, type(t).__name__))
    if not t.is_cuda:
        raise ValueError("%s: tensor must live on the GPU (device is %s)" % (what, t.device))
    if t.dtype not in dtypes:
        raise ValueError("%s: dtype %s, expected %s" % (what, t.dtype, " or ".join(str(d) for d in dtypes)))
    if dense:
        if not t.is_contiguous():
            raise ValueError("%s: tensor must be contiguous" % what)
    elif t.dim() >= 1 and t.numel() > 1 and t.shape[-1] > 1 and t.stride(-1) != 1:
        raise ValueError("%s: last dimension must have stride 1 (got %d)" % (what, t.stride(-1)))
    elif t.dim() > 2 and not t.is_contiguous():
        raise ValueError("%s: tensor must be contiguous" % what)
    return t


def _ld(t):
    """Row stride of a 2-D tensor in elements (its row length when it has a single row)."""
    return t.stride(0) if t.shape[0] > 1 else max(t.shape[1], 1)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return _p(stream.cuda_stream)


def _check(status, what):
    if status != 0:
        raise BmxError(status, what)


def workspace_bytes(op, dims):
    arr = (_i64 * len(dims))(*[int(d) for d in dims])
    return int(lib().bmx_workspace_bytes(int(op), arr, len(dims)))


def _workspace(op, dims, device, workspace):
    need = workspace_bytes(op, dims)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    elif not (isinstance(workspace, torch.Tensor) and workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous GPU tensor")
    return workspace, workspace.numel() * workspace.element_size()


def _u64_as_i64(shape, device):
    # torch has no general uint64 support; packed words are carried as int64 storage
    return torch.empty(shape, dtype=torch.int64, device=device)


def binarize_pack(x, pack_dim=1, out=None, stream=None):
    """x: fp32 [rows, cols] device tensor (row-major, stride(1) == 1).  Returns packed int64
    storage [R, ceil(K/64)] holding the uint64 words."""
    _chk(x, _F32, "binarize_pack x")
    rows, cols = x.shape
    R, K = (rows, cols) if pack_dim else (cols, rows)
    if out is None:
        out = _u64_as_i64((R, (K + 63) // 64), x.device)
    _chk(out, _U64, "binarize_pack out")
    _check(lib().bmx_binarize_pack(_ptr(x), rows, cols, _ld(x), pack_dim, _ptr(out), _ld(out),
                                   _stream(stream)), "bmx_binarize_pack")
    return out


def unpack_pm1(bits, K, out=None, stream=None):
    """bits: packed int64 storage [rows, words] -> fp32 [rows, K] of +1 / -1."""
    _chk(bits, _U64, "unpack_pm1 bits")
    rows = bits.shape[0]
    if out is None:
        out = torch.empty((rows, K), dtype=torch.float32, device=bits.device)
    _chk(out, _F32, "unpack_pm1 out")
    _check(lib().bmx_unpack_pm1(_ptr(bits), rows, K, _ld(bits), _ptr(out), _ld(out), _stream(stream)),
           "bmx_unpack_pm1")
    return out


def xnor_gemm(A, B, K, out=None, stream=None, count=False):
    """count: the xnor count (dot + K) / 2 of Eq. 2 instead of the dot product."""
    _chk(A, _U64, "xnor_gemm A")
    _chk(B, _U64, "xnor_gemm B")
    M, N = A.shape[0], B.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=A.device)
    _chk(out, _I32, "xnor_gemm out")
    f = lib().bmx_xnor_gemm_count if count else lib().bmx_xnor_gemm
    _check(f(_ptr(A), _ld(A), _ptr(B), _ld(B), _ptr(out), _ld(out), M, N, K, _stream(stream)),
           "bmx_xnor_gemm_count" if count else "bmx_xnor_gemm")
    return out


def widen_words32(rows32, K, out=None, stream=None):
    """rows32: int32 storage [rows, dwords] holding rows of 32-bit words (the 32-bit BINARY_WORD
    flavour) -> int64 storage [rows, ceil(K/64)] holding the same rows as 64-bit words."""
    _chk(rows32, _I32, "widen_words32 rows32")
    rows = rows32.shape[0]
    if out is None:
        out = _u64_as_i64((rows, (K + 63) // 64), rows32.device)
    _chk(out, _U64, "widen_words32 out")
    _check(lib().bmx_widen_words32(_ptr(rows32), rows, K, _ld(rows32), _ptr(out), _ld(out), _stream(stream)),
           "bmx_widen_words32")
    return out


def xnor_gemm_w32(A32, B32, K, out=None, workspace=None, stream=None):
    """bmx_xnor_gemm on operands stored as rows of 32-bit words (int32 storage)."""
    _chk(A32, _I32, "xnor_gemm_w32 A")
    _chk(B32, _I32, "xnor_gemm_w32 B")
    M, N = A32.shape[0], B32.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=A32.device)
    _chk(out, _I32, "xnor_gemm_w32 out")
    ws, ws_bytes = _workspace(OP_XNOR_GEMM_W32, (M, N, K), A32.device, workspace)
    _check(lib().bmx_xnor_gemm_w32(_ptr(A32), _ld(A32), _ptr(B32), _ld(B32), _ptr(out), _ld(out), M, N, K,
                                   _ptr(ws), ws_bytes, _stream(stream)), "bmx_xnor_gemm_w32")
    return out


def binary_fc(x, Wp, alpha=None, integer_out=False, out=None, workspace=None, stream=None):
    _chk(x, _F32, "binary_fc x")
    _chk(Wp, _U64, "binary_fc Wp")
    _chk(alpha, _F32, "binary_fc alpha", dense=True)
    batch, fin = x.shape
    fout = Wp.shape[0]
    if out is None:
        out = torch.empty((batch, fout), dtype=torch.int32 if integer_out else torch.float32,
                          device=x.device)
    _chk(out, _I32 if integer_out else _F32, "binary_fc out")
    ws, ws_bytes = _workspace(OP_BINARY_FC, (batch, fin, fout), x.device, workspace)
    oi, of = (out, None) if integer_out else (None, out)
    _check(lib().bmx_binary_fc(_ptr(x), _ld(x), _ptr(Wp), _ld(Wp), _ptr(alpha), batch, fin, fout,
                               _ptr(oi), _ptr(of), _ld(out), _ptr(ws), ws_bytes, _stream(stream)),
           "bmx_binary_fc")
    return out


def binary_fc_static(x, Wp, alpha=None, integer_out=False, out=None, stream=None):
    """bmx_binary_fc on the library's own scratch array: the call itself allocates nothing, so
    `out` must be given."""
    _chk(x, _F32, "binary_fc_static x")
    _chk(Wp, _U64, "binary_fc_static Wp")
    _chk(alpha, _F32, "binary_fc_static alpha", dense=True)
    if out is None:
        raise ValueError("binary_fc_static: pass the output tensor (the call allocates nothing)")
    _chk(out, _I32 if integer_out else _F32, "binary_fc_static out")
    batch, fin = x.shape
    fout = Wp.shape[0]
    oi, of = (out, None) if integer_out else (None, out)
    _check(lib().bmx_binary_fc_static(_ptr(x), _ld(x), _ptr(Wp), _ld(Wp), _ptr(alpha), batch, fin, fout,
                                      _ptr(oi), _ptr(of), _ld(out), _stream(stream)), "bmx_binary_fc_static")
    return out


def binary_fc_packed(xp, in_features, Wp, alpha=None, mode="f32", out=None, thr=None, stream=None):
    """xp: packed activations [batch, words].  mode: "f32", "i32" or "bits" (packed sign bits,
    against the per-feature threshold thr if given)."""
    _chk(xp, _U64, "binary_fc_packed xp")
    _chk(Wp, _U64, "binary_fc_packed Wp")
    _chk(alpha, _F32, "binary_fc_packed alpha", dense=True)
    _chk(thr, _F32, "binary_fc_packed thr", dense=True)
    batch, fout = xp.shape[0], Wp.shape[0]
    if out is None:
        if mode == "bits":
            out = _u64_as_i64((batch, (fout + 63) // 64), xp.device)
        else:
            out = torch.empty((batch, fout), dtype=torch.int32 if mode == "i32" else torch.float32,
                              device=xp.device)
    oi, of, ob = (out if mode == "i32" else None, out if mode == "f32" else None,
                  out if mode == "bits" else None)
    _chk(out, {"i32": _I32, "f32": _F32, "bits": _U64}[mode], "binary_fc_packed out")
    _check(lib().bmx_binary_fc_packed(_ptr(xp), _ld(xp), _ptr(Wp), _ld(Wp), _ptr(alpha), batch,
                                      in_features, fout, _ptr(oi), _ptr(of), _ptr(ob), _ptr(thr),
                                      _ld(out), _stream(stream)), "bmx_binary_fc_packed")
    return out


def pack_conv_weights(w, stream=None):
    _chk(w, _F32, "pack_conv_weights w", dense=True)
    O, C, KH, KW = w.shape
    ld = int(lib().bmx_conv_weight_row_words(C, KH, KW))
    if ld <= 0:
        raise BmxError(-5, "bmx_conv_weight_row_words")
    Wp = _u64_as_i64((O, ld), w.device)
    _check(lib().bmx_pack_conv_weights(_ptr(w), O, C, KH, KW, _ptr(Wp), _stream(stream)),
           "bmx_pack_conv_weights")
    return Wp


def conv_out_hw(H, W, KH, KW, stride, pad):
    return (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1


def binary_conv2d(x, Wp, O, KH, KW, stride=1, pad=0, alpha=None, integer_out=False, out=None,
                  workspace=None, stream=None):
    _chk(x, _F32, "binary_conv2d x", dense=True)
    _chk(Wp, _U64, "binary_conv2d Wp", dense=True)
    _chk(alpha, _F32, "binary_conv2d alpha", dense=True)
    N, C, H, W = x.shape
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    if out is None:
        out = torch.empty((N, O, Ho, Wo), dtype=torch.int32 if integer_out else torch.float32,
                          device=x.device)
    _chk(out, _I32 if integer_out else _F32, "binary_conv2d out", dense=True)
    ws, ws_bytes = _workspace(OP_BINARY_CONV2D, (N, C, H, W, O, KH, KW, stride, pad), x.device,
                              workspace)
    oi, of = (out, None) if integer_out else (None, out)
    _check(lib().bmx_binary_conv2d(_ptr(x), N, C, H, W, _ptr(Wp), O, KH, KW, stride, pad, _ptr(alpha),
                                   _ptr(oi), _ptr(of), _ptr(ws), ws_bytes, _stream(stream)),
           "bmx_binary_conv2d")
    return out


def pack_nchw(x, pad=0, out=None, stream=None):
    _chk(x, _F32, "pack_nchw x", dense=True)
    N, C, H, W = x.shape
    if out is None:
        out = _u64_as_i64((N, H + 2 * pad, W + 2 * pad, (C + 63) // 64), x.device)
    _chk(out, _U64, "pack_nchw out", dense=True)
    _check(lib().bmx_pack_nchw(_ptr(x), N, C, H, W, pad, _ptr(out), _stream(stream)), "bmx_pack_nchw")
    return out


def binary_conv2d_packed(xp, C, Wp, O, KH, KW, stride=1, pad=0, alpha=None, integer_out=False,
                         out=None, stream=None):
    _chk(xp, _U64, "binary_conv2d_packed xp", dense=True)
    _chk(Wp, _U64, "binary_conv2d_packed Wp", dense=True)
    _chk(alpha, _F32, "binary_conv2d_packed alpha", dense=True)
    N, H, W = xp.shape[0], xp.shape[1] - 2 * pad, xp.shape[2] - 2 * pad
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    if out is None:
        out = torch.empty((N, O, Ho, Wo), dtype=torch.int32 if integer_out else torch.float32,
                          device=xp.device)
    _chk(out, _I32 if integer_out else _F32, "binary_conv2d_packed out", dense=True)
    oi, of = (out, None) if integer_out else (None, out)
    _check(lib().bmx_binary_conv2d_packed(_ptr(xp), N, C, H, W, _ptr(Wp), O, KH, KW, stride, pad,
                                          _ptr(alpha), _ptr(oi), _ptr(of), _stream(stream)),
           "bmx_binary_conv2d_packed")
    return out


def binary_conv2d_bits(xp, C, Wp, O, KH, KW, stride=1, pad=0, alpha=None, thr=None, out_pad=1,
                       out=None, workspace=None, stream=None):
    """Convolution on a packed image whose result is the next convolution's packed image
    [N, Ho + 2*out_pad, Wo + 2*out_pad, ceil(O/64)] (int64 storage holding the uint64 words)."""
    _chk(xp, _U64, "binary_conv2d_bits xp", dense=True)
    _chk(Wp, _U64, "binary_conv2d_bits Wp", dense=True)
    _chk(alpha, _F32, "binary_conv2d_bits alpha", dense=True)
    _chk(thr, _F32, "binary_conv2d_bits thr", dense=True)
    N, H, W = xp.shape[0], xp.shape[1] - 2 * pad, xp.shape[2] - 2 * pad
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    if out is None:
        out = _u64_as_i64((N, Ho + 2 * out_pad, Wo + 2 * out_pad, (O + 63) // 64), xp.device)
    _chk(out, _U64, "binary_conv2d_bits out", dense=True)
    ws, ws_bytes = _workspace(OP_BINARY_CONV2D_BITS, (N, C, H, W, O, KH, KW, stride, pad, out_pad),
                              xp.device, workspace)
    _check(lib().bmx_binary_conv2d_bits(_ptr(xp), N, C, H, W, _ptr(Wp), O, KH, KW, stride, pad,
                                        _ptr(alpha), _ptr(thr), _ptr(out), out_pad, _ptr(ws), ws_bytes,
                                        _stream(stream)), "bmx_binary_conv2d_bits")
    return out


def quant_gemm(a, w, bits_a, bits_w=1, want_int=True, want_float=True, out_int=None, out_float=None,
               workspace=None, stream=None):
    _chk(a, _F32, "quant_gemm a")
    _chk(w, _F32, "quant_gemm w")
    M, K = a.shape
    N = w.shape[0]
    S = out_int if out_int is not None else (
        torch.empty((M, N), dtype=torch.int32, device=a.device) if want_int else None)
    of = out_float if out_float is not None else (
        torch.empty((M, N), dtype=torch.float32, device=a.device) if want_float else None)
    _chk(S, _I32, "quant_gemm out_int")
    _chk(of, _F32, "quant_gemm out_float")
    ldo = _ld(S if S is not None else of)
    if S is not None and of is not None and _ld(of) != ldo:
        raise ValueError("quant_gemm: out_int and out_float must share one row stride")
    ws, ws_bytes = _workspace(OP_QUANT_GEMM, (M, N, K, bits_a, bits_w), a.device, workspace)
    _check(lib().bmx_quant_gemm(_ptr(a), _ld(a), bits_a, _ptr(w), _ld(w), bits_w, M, N, K, _ptr(S),
                                _ptr(of), ldo, _ptr(ws), ws_bytes, _stream(stream)), "bmx_quant_gemm")
    return S, of


def alpha_mean_abs(w, stream=None):
    _chk(w, _F32, "alpha_mean_abs w", dense=True)
    rows = w.shape[0]
    cols = w.numel() // max(rows, 1)
    alpha = torch.empty((rows,), dtype=torch.float32, device=w.device)
    _check(lib().bmx_alpha_mean_abs(_ptr(w), rows, cols, cols, _ptr(alpha), _stream(stream)),
           "bmx_alpha_mean_abs")
    return alpha
