"""Host-side checks of the C-ABI library that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

from paper_1705_09864_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 0x7F0000001000  # a fake, well aligned, never dereferenced device address
NULL = None
OK, E_NULL, E_SHAPE, E_LD, E_ALIGN, E_UNSUP, E_WS = 0, -1, -2, -3, -4, -5, -6


def test_header_symbols_exported():
    text = open(os.path.join(ROOT, "include", "bmx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(bmx_[a-z0-9_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert B.version() >= 100


def test_status_strings():
    for code in range(-7, 1):
        assert B.status_string(code).startswith("BMX_")
    assert "unknown" in B.status_string(-99)


def test_tune_keys():
    """The measurement hook takes the keys the header documents and no others, and key 0 puts
    every choice back to automatic (no kernel runs here: the settings only steer later calls)."""
    L = B.lib()
    text = open(os.path.join(ROOT, "include", "bmx.h")).read()
    documented = {int(k) for k in re.findall(r"\bkey (\d+)\b", text[text.index("bmx_tune_set(0, 0)"):text.index("int bmx_tune_set")])}
    try:
        for key in range(1, 40):
            rc = L.bmx_tune_set(key, 1)
            assert rc == (OK if key in documented else E_UNSUP), key
        assert {1, 5, 7, 10, 13, 14, 15} <= documented
    finally:
        assert L.bmx_tune_set(0, 0) == OK


def test_workspace_query():
    assert B.workspace_bytes(B.OP_BINARY_FC, (256, 9216, 4096)) == 256 * 144 * 8
    assert B.workspace_bytes(B.OP_BINARY_FC, (5, 65, 3)) == 5 * 16 * 8 + 128  # 5 rows padded to 16 words, rounded up to 256 B
    assert B.workspace_bytes(B.OP_BINARY_CONV2D, (16, 64, 56, 56, 64, 3, 3, 1, 1)) == 16 * 58 * 58 * 8
    assert B.workspace_bytes(B.OP_BINARY_CONV2D, (1, 65, 5, 5, 2, 3, 3, 1, 1)) == 1024  # 49*2 words -> 784 B
    q = B.workspace_bytes(B.OP_QUANT_GEMM, (1024, 1024, 4096, 2, 1))
    assert q == 2 * 1024 * 64 * 8 + 1024 * 64 * 8 + 4096  # plane rows, weight bits, row sums
    assert B.workspace_bytes(B.OP_QUANT_GEMM, (4, 4, 64, 9, 1)) == 0      # bits_a out of range
    assert B.workspace_bytes(B.OP_QUANT_GEMM, (4, 4, 64, 2, 9)) == 0      # bits_w out of range
    # k-bit weights: both operands as planes, row sums, one int32 result per weight plane
    assert B.workspace_bytes(B.OP_QUANT_GEMM, (4, 4, 64, 2, 2)) == 2 * 4 * 16 * 8 + 2 * 4 * 16 * 8 + 256 + 256 + 256
    assert B.workspace_bytes(B.OP_BINARY_CONV2D, (1, 3, 8, 8, 2, 4, 4, 1, 0)) == 0  # even kernel
    # packed-bit convolution: nothing where the convolution kernel writes the bits itself (3 x 3
    # over at most 256 channels), else the fp32 result of the two-kernel route
    assert B.workspace_bytes(B.OP_BINARY_CONV2D_BITS, (16, 64, 56, 56, 64, 3, 3, 1, 1, 1)) == 0
    assert B.workspace_bytes(B.OP_BINARY_CONV2D_BITS, (2, 256, 14, 14, 40, 3, 3, 2, 1, 0)) == 0
    assert B.workspace_bytes(B.OP_BINARY_CONV2D_BITS, (2, 64, 8, 8, 5, 5, 5, 1, 2, 1)) == 0   # 25 words too
    assert B.workspace_bytes(B.OP_BINARY_CONV2D_BITS, (2, 129, 8, 8, 5, 5, 5, 1, 2, 1)) == 2 * 5 * 8 * 8 * 4
    assert B.workspace_bytes(B.OP_BINARY_CONV2D_BITS, (2, 300, 8, 8, 5, 3, 3, 1, 1, 1)) == 2 * 5 * 8 * 8 * 4
    assert B.workspace_bytes(B.OP_BINARY_CONV2D_BITS, (2, 150, 8, 8, 5, 3, 3, 1, 1, 1)) == 0   # 27 words
    assert B.workspace_bytes(B.OP_BINARY_CONV2D_BITS, (2, 64, 8, 8, 5, 3, 3, 1, 1, 7)) == 0   # out_pad out of range
    assert B.workspace_bytes(B.OP_BINARY_CONV2D_BITS, (2, 64, 8, 8, 5, 3, 3, 1, 1)) == 0      # too few dims
    assert B.workspace_bytes(99, (1, 2, 3)) == 0
    assert B.workspace_bytes(B.OP_BINARY_FC, (1, 2)) == 0


def test_binarize_pack_validation():
    f = B.lib().bmx_binarize_pack
    assert f(P, 4, 64, 64, 2, P, 1, NULL) == E_UNSUP
    assert f(P, -1, 64, 64, 1, P, 1, NULL) == E_SHAPE
    assert f(P, 4, 0, 64, 1, P, 1, NULL) == E_SHAPE         # K = 0
    assert f(NULL, 4, 64, 64, 1, P, 1, NULL) == E_NULL
    assert f(P, 4, 64, 64, 1, NULL, 1, NULL) == E_NULL
    assert f(P, 4, 65, 64, 1, P, 2, NULL) == E_LD           # ldx < cols
    assert f(P, 4, 65, 65, 1, P, 1, NULL) == E_LD           # out_ld < ceil(65/64)
    assert f(P + 2, 4, 64, 64, 1, P, 1, NULL) == E_ALIGN
    assert f(P, 4, 64, 64, 1, P + 4, 1, NULL) == E_ALIGN
    assert f(P, 0, 64, 64, 1, P, 1, NULL) == OK             # empty: no launch
    assert f(P, 64, 0, 1, 0, P, 1, NULL) == OK              # pack_dim 0 with zero columns
    assert f(P, 1 << 24, 4, 4, 0, P, 1 << 18, NULL) == E_SHAPE  # K too long


@pytest.mark.parametrize("name", ["bmx_xnor_gemm", "bmx_xnor_gemm_count"])
def test_xnor_gemm_validation(name):
    f = getattr(B.lib(), name)
    assert f(P, 1, P, 1, P, 8, 4, 8, 0, NULL) == E_SHAPE
    assert f(P, 1, P, 1, P, 8, -4, 8, 64, NULL) == E_SHAPE
    assert f(P, 1, P, 1, P, 8, 4, 8, 1 << 24, NULL) == E_SHAPE
    assert f(NULL, 1, P, 1, P, 8, 4, 8, 64, NULL) == E_NULL
    assert f(P, 1, P, 1, P, 8, 4, 8, 65, NULL) == E_LD
    assert f(P, 2, P, 2, P, 7, 4, 8, 65, NULL) == E_LD
    assert f(P + 4, 2, P, 2, P, 8, 4, 8, 65, NULL) == E_ALIGN
    assert f(P, 1, P, 1, P, 8, 0, 8, 64, NULL) == OK
    assert f(P, 1, P, 1, P, 8, 4, 0, 64, NULL) == OK


def test_binary_fc_validation():
    f = B.lib().bmx_binary_fc
    big = 1 << 20
    assert f(P, 64, P, 1, NULL, 4, 64, 8, NULL, NULL, 8, P, big, NULL) == E_NULL    # no output
    assert f(P, 64, P, 1, NULL, 4, 64, 8, P, P, 8, P, big, NULL) == E_NULL          # both outputs
    assert f(P, 64, P, 1, P, 4, 64, 8, P, NULL, 8, P, big, NULL) == E_UNSUP         # alpha + int out
    assert f(P, 63, P, 1, NULL, 4, 64, 8, NULL, P, 8, P, big, NULL) == E_LD
    assert f(P, 64, P, 1, NULL, 4, 64, 8, NULL, P, 7, P, big, NULL) == E_LD
    assert f(P, 64, P, 1, NULL, 4, 64, 8, NULL, P, 8, NULL, big, NULL) == E_WS
    assert f(P, 64, P, 1, NULL, 4, 64, 8, NULL, P, 8, P, 16, NULL) == E_WS
    assert f(P, 64, P, 1, NULL, 4, 64, 8, NULL, P, 8, P + 8, big, NULL) == E_ALIGN
    assert f(P, 64, P, 1, NULL, 0, 64, 8, NULL, P, 8, P, big, NULL) == OK
    assert f(P, 64, P, 1, NULL, 4, 0, 8, NULL, P, 8, P, big, NULL) == E_SHAPE


def test_conv_validation():
    f = B.lib().bmx_binary_conv2d
    big = 1 << 24
    args = dict(N=2, C=3, H=8, W=8, O=4, KH=3, KW=3, s=1, p=1)

    def call(x=P, Wp=P, alpha=NULL, oi=NULL, of=P, ws=P, wsb=big, **kw):
        a = dict(args, **kw)
        return f(x, a["N"], a["C"], a["H"], a["W"], Wp, a["O"], a["KH"], a["KW"], a["s"], a["p"],
                 alpha, oi, of, ws, wsb, NULL)

    assert call(KH=4, KW=4) == E_UNSUP
    assert call(KH=3, KW=5) == E_UNSUP
    assert call(KH=9, KW=9) == E_UNSUP
    assert call(s=3) == E_UNSUP
    assert call(p=3) == E_UNSUP
    assert call(p=-1) == E_UNSUP
    assert call(C=0) == E_SHAPE
    assert call(H=1, W=1, p=0) == E_SHAPE          # window larger than the image
    assert call(x=NULL) == E_NULL
    assert call(of=NULL) == E_NULL
    assert call(oi=P, of=P) == E_NULL
    assert call(oi=P, of=NULL, alpha=P) == E_UNSUP
    assert call(ws=NULL) == E_WS
    assert call(wsb=64) == E_WS
    assert call(N=0) == OK
    assert call(O=0) == OK
    g = B.lib().bmx_pack_conv_weights
    assert g(P, 4, 3, 3, 3, NULL, NULL) == E_NULL
    assert g(P, 4, 3, 2, 2, P, NULL) == E_UNSUP
    assert g(P, 0, 3, 3, 3, P, NULL) == OK


def test_conv_bits_validation():
    f = B.lib().bmx_binary_conv2d_bits
    big = 1 << 24
    args = dict(N=2, C=129, H=8, W=8, O=4, KH=5, KW=5, s=1, p=1, op=1)

    def call(xp=P, Wp=P, alpha=NULL, thr=NULL, out=P, ws=P, wsb=big, **kw):
        a = dict(args, **kw)
        return f(xp, a["N"], a["C"], a["H"], a["W"], Wp, a["O"], a["KH"], a["KW"], a["s"], a["p"],
                 alpha, thr, out, a["op"], ws, wsb, NULL)

    assert call(KH=4, KW=4) == E_UNSUP
    assert call(s=3) == E_UNSUP
    assert call(op=-1) == E_UNSUP
    assert call(op=7) == E_UNSUP
    assert call(C=0) == E_SHAPE
    assert call(O=0) == OK                         # zero counts launch nothing, like everywhere
    assert call(O=4 * 65535 + 1) == E_SHAPE
    assert call(xp=NULL) == E_NULL
    assert call(Wp=NULL) == E_NULL
    assert call(out=NULL) == E_NULL
    assert call(N=0) == OK
    # where the size query answers 0 (the kernel that writes the bits itself), the filter rows are
    # read in 16-byte pieces: an 8-byte aligned Wp is refused, not sent down the other route with
    # a workspace the query never asked for
    assert B.workspace_bytes(B.OP_BINARY_CONV2D_BITS, (2, 64, 8, 8, 4, 3, 3, 1, 1, 1)) == 0
    assert call(C=64, KH=3, KW=3, Wp=P + 8, ws=NULL, wsb=0) == E_ALIGN
    # 5 x 5 over three channel words goes through the fp32 result: the workspace is checked before any launch
    assert call(ws=NULL) == E_WS
    assert call(wsb=64) == E_WS


def test_quant_and_alpha_validation():
    f = B.lib().bmx_quant_gemm
    big = 1 << 24
    assert f(P, 64, 0, P, 64, 1, 4, 4, 64, P, P, 4, P, big, NULL) == E_UNSUP
    assert f(P, 64, 9, P, 64, 1, 4, 4, 64, P, P, 4, P, big, NULL) == E_UNSUP
    assert f(P, 64, 2, P, 64, 9, 4, 4, 64, P, P, 4, P, big, NULL) == E_UNSUP
    assert f(P, 64, 2, P, 64, 0, 4, 4, 64, P, P, 4, P, big, NULL) == E_UNSUP
    assert f(P, 1 << 20, 8, P, 1 << 20, 8, 4, 4, 1 << 20, P, P, 4, P, big, NULL) == E_SHAPE   # K * 255 * 255 >= 2^31
    assert f(P, 64, 2, P, 64, 1, 4, 4, 64, NULL, NULL, 4, P, big, NULL) == E_NULL
    assert f(P, 63, 2, P, 64, 1, 4, 4, 64, P, P, 4, P, big, NULL) == E_LD
    assert f(P, 64, 2, P, 64, 1, 4, 4, 64, P, P, 4, P, 100, NULL) == E_WS
    assert f(P, 64, 2, P, 64, 1, 0, 4, 64, P, P, 4, P, big, NULL) == OK
    g = B.lib().bmx_alpha_mean_abs
    assert g(P, 4, 0, 0, P, NULL) == E_SHAPE
    assert g(P, 4, 8, 7, P, NULL) == E_LD
    assert g(NULL, 4, 8, 8, P, NULL) == E_NULL
    assert g(P, 0, 8, 8, P, NULL) == OK


def test_words32_validation():
    L = B.lib()
    f = L.bmx_widen_words32
    assert f(P, -1, 96, 3, P, 2, NULL) == E_SHAPE
    assert f(P, 4, 0, 3, P, 2, NULL) == E_SHAPE
    assert f(P, 0, 96, 3, P, 2, NULL) == OK
    assert f(NULL, 4, 96, 3, P, 2, NULL) == E_NULL
    assert f(P, 4, 96, 2, P, 2, NULL) == E_LD          # 96 bits need 3 dwords
    assert f(P, 4, 96, 3, P, 1, NULL) == E_LD          # and 2 words
    assert f(P + 2, 4, 96, 3, P, 2, NULL) == E_ALIGN
    assert f(P, 4, 96, 3, P + 4, 2, NULL) == E_ALIGN
    g = L.bmx_xnor_gemm_w32
    assert g(P, 3, P, 3, P, 5, 0, 5, 96, NULL, 0, NULL) == OK
    assert g(P, 3, P, 3, P, 5, 4, 5, 0, NULL, 0, NULL) == E_SHAPE
    assert g(P, 2, P, 3, P, 5, 4, 5, 96, P, 1 << 20, NULL) == E_LD
    assert g(P, 3, P, 3, P, 4, 4, 5, 96, P, 1 << 20, NULL) == E_LD
    assert g(NULL, 3, P, 3, P, 5, 4, 5, 96, P, 1 << 20, NULL) == E_NULL
    assert g(P, 3, P, 3, P, 5, 4, 5, 96, NULL, 0, NULL) == E_WS       # odd dword rows must be widened
    assert g(P, 3, P, 3, P, 5, 4, 5, 96, P, 64, NULL) == E_WS
    assert g(P + 1, 3, P, 3, P, 5, 4, 5, 96, P, 1 << 20, NULL) == E_ALIGN
    assert B.workspace_bytes(B.OP_XNOR_GEMM_W32, (4, 5, 96)) == 256 + 256    # 4 x 2 and 5 x 2 words
    assert B.workspace_bytes(B.OP_XNOR_GEMM_W32, (4, 5, 0)) == 0


def test_fc_packed_validation():
    f = B.lib().bmx_binary_fc_packed
    ok = dict(xp=P, ldx=8, Wp=P, ldw=8, alpha=NULL, b=4, fin=512, fout=70, oi=NULL, of=NULL, ob=P, thr=NULL,
              ldo=2)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["xp"], a["ldx"], a["Wp"], a["ldw"], a["alpha"], a["b"], a["fin"], a["fout"], a["oi"],
                 a["of"], a["ob"], a["thr"], a["ldo"], NULL)

    assert call(b=0) == OK and call(fout=0) == OK                       # empty: no launch
    assert call(ob=NULL, of=P, ldo=70, thr=P) == E_UNSUP                # a threshold decides bits only
    assert call(thr=P + 2) == E_ALIGN
    assert call(b=-1) == E_SHAPE and call(fin=0) == E_SHAPE
    assert call(xp=NULL) == E_NULL and call(Wp=NULL) == E_NULL
    assert call(ob=NULL) == E_NULL                                      # no output at all
    assert call(of=P, ldo=70) == E_NULL                                 # two outputs
    assert call(oi=P, ob=NULL, alpha=P, ldo=70) == E_UNSUP              # int output with a scale
    assert call(ldx=7) == E_LD and call(ldw=7) == E_LD
    assert call(ldo=1) == E_LD                                          # 70 features need 2 words
    assert call(ob=NULL, of=P, ldo=69) == E_LD
    assert call(ob=P + 4) == E_ALIGN and call(xp=P + 4) == E_ALIGN


def test_binding_refuses_tensors_the_c_abi_would_misread():
    """The wrappers see tensors, the C ABI only addresses: a host tensor, a wrong element type or
    a transposed view must be refused on the host, before any address reaches the library."""
    import torch
    x = torch.zeros((4, 128), dtype=torch.float32)             # lives on the host
    with pytest.raises(ValueError, match="GPU"):
        B.binarize_pack(x, 1)
    with pytest.raises(ValueError, match="GPU"):
        B.xnor_gemm(torch.zeros((4, 2), dtype=torch.int64), torch.zeros((4, 2), dtype=torch.int64), 128)
    with pytest.raises(ValueError, match="GPU"):
        B.binary_conv2d(torch.zeros((1, 3, 5, 5)), torch.zeros((2, 10), dtype=torch.int64), 2, 3, 3)
    with pytest.raises(ValueError, match="torch tensor"):
        B.alpha_mean_abs([[1.0, 2.0]])
    # dtype and layout are checked on "meta" tensors here: no GPU in this test, and the checks
    # must fire before a data pointer is taken
    for bad, what in ((torch.zeros((4, 128), dtype=torch.float64), "dtype"),
                      (torch.zeros((128, 4), dtype=torch.float32).t(), "stride")):
        with pytest.raises(ValueError):
            B._chk(_FakeCuda(bad), B._F32, "x")
    ok = _FakeCuda(torch.zeros((4, 200), dtype=torch.float32)[:, :128])   # rows further apart: fine
    assert B._chk(ok, B._F32, "x") is ok and B._ld(ok) == 200


class _FakeCuda:
    """A host tensor that claims to live on the GPU, to reach the checks behind the device test."""

    def __init__(self, t):
        self._t = t
        self.is_cuda = True

    def __getattr__(self, name):
        return getattr(self._t, name)
