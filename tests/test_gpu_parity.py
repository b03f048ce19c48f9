"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs.

Bars: packed words and integer results bit-exact; fp32 results within 1e-6 relative of the
oracle (they are in practice bit-identical: one fp32 multiply or one IEEE division of an
exactly representable integer).  All calls go through paper_1705_09864_amd.binding, i.e.
through the C ABI of libbmx.so.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1705_09864_amd import binding as B
from paper_1705_09864_amd import synth

pytestmark = pytest.mark.gpu
RTOL = 1e-6
POISON = np.uint64(0xCDCDCDCDCDCDCDCD)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host_u64(t):
    return t.cpu().numpy().view(np.uint64)


def assert_f32_close(got, ref, atol=0.0):
    """|got - ref| <= 1e-6 * |ref| (+ atol).  atol is non-zero only against the oracle's
    double-precision sum of quantised values, whose own rounding noise (about K * 2^-53 * K,
    below 1e-9 for every K used here) is all that separates it from the exact rational."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(got - ref)
    assert (err <= RTOL * np.abs(ref) + atol).all(), "max rel err %g" % (err / np.maximum(np.abs(ref), 1e-30)).max()


# ------------------------------------------------------------------ binarize + pack
@pytest.mark.parametrize("rows,K", [(1, 1), (3, 63), (2, 64), (5, 65), (7, 500), (4, 576), (3, 1000),
                                    (9, 4095), (33, 512), (2, 8192), (130, 27)])
def test_pack_rows(rows, K):
    rng = np.random.default_rng(rows * 100003 + K)
    x = rng.standard_normal((rows, K)).astype(np.float32)
    x.flat[:: 7] = 0.0
    x.flat[3:: 11] = -0.0
    got = host_u64(B.binarize_pack(dev(x), 1))
    np.testing.assert_array_equal(got, oracle.binarize_pack(x, 1))


def test_pack_rows_special_values():
    v = np.array([0.0, -0.0, 1e-45, -1e-45, 1.1754942e-38, -1.1754942e-38, np.inf, -np.inf,
                  1.0, -1.0, 3e38, -3e38, np.nan, -np.nan, 2.5, -2.5], dtype=np.float32)
    x = np.tile(v, 16)[None, :].copy()
    got = host_u64(B.binarize_pack(dev(x), 1))
    np.testing.assert_array_equal(got, oracle.binarize_pack(x, 1))  # negative denormals stay -1
    # the pattern itself, from the reading of the sign function: (x >= 0) as an IEEE compare,
    # so +-0, positive denormals and +inf give 1, NaN of either sign gives 0
    assert got[0, 0] & np.uint64(0xFFFF) == np.uint64(0b0100_0101_0101_0111)
    # the same values down a strided column and through the channel pack of a convolution
    col = np.tile(v, 8)[:, None] * np.ones((1, 3), dtype=np.float32)
    np.testing.assert_array_equal(host_u64(B.binarize_pack(dev(col), 0)), oracle.binarize_pack(col, 0))


def test_conv_special_values_in_the_image():
    """NaN, +-0, denormals and infinities in a convolution input: the channel pack takes the same
    IEEE compare as the row pack, and the layer equals the oracle's (which binarises the
    zero-padded float image element by element)."""
    v = np.array([0.0, -0.0, 1e-45, -1e-45, np.inf, -np.inf, np.nan, -np.nan, 1.0, -1.0], dtype=np.float32)
    rng = np.random.default_rng(41)
    x = rng.choice(v, size=(2, 70, 9, 7)).astype(np.float32)
    w = rng.standard_normal((5, 70, 3, 3)).astype(np.float32)
    ri, _ = oracle.binary_conv2d(x, w, 1, 1)
    np.testing.assert_array_equal(run_conv(x, w, 1, 1, integer_out=True), ri)
    xp = host_u64(B.pack_nchw(dev(x), 0))
    rows = np.transpose(x, (0, 2, 3, 1)).reshape(-1, 70)
    np.testing.assert_array_equal(xp.reshape(-1, 2), oracle.binarize_pack(rows, 1))


def test_pack_rows_strided_and_poisoned():
    rng = np.random.default_rng(11)
    rows, K, ldx, ld = 6, 200, 260, 6
    buf = rng.standard_normal((rows, ldx)).astype(np.float32)
    xd = dev(buf)[:, :K]
    out = torch.from_numpy(np.full((rows, ld), POISON, dtype=np.uint64).view(np.int64)).cuda()
    B.binarize_pack(xd, 1, out=out)
    got = host_u64(out)
    ref = oracle.binarize_pack(buf[:, :K].copy(), 1, out_ld_words=ld, fill=POISON)
    np.testing.assert_array_equal(got, ref)       # tail bits 0, words past Kw untouched


@pytest.mark.parametrize("K,N", [(1, 1), (64, 64), (65, 3), (130, 7), (512, 256), (500, 300), (27, 1000)])
def test_pack_dim0(K, N):
    rng = np.random.default_rng(K * 7919 + N)
    x = rng.standard_normal((K, N)).astype(np.float32)
    got = host_u64(B.binarize_pack(dev(x), 0))
    np.testing.assert_array_equal(got, oracle.binarize_pack(x, 0))


# ------------------------------------------------------------------ xnor GEMM
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (4, 4, 64), (3, 5, 65), (17, 29, 333), (64, 256, 512),
                                   (70, 130, 1000), (33, 300, 2304), (129, 65, 4095), (8, 600, 576)])
def test_xnor_gemm(M, N, K):
    rng = np.random.default_rng(M * 31 + N * 17 + K)
    A = oracle.binarize_pack(rng.standard_normal((M, K)).astype(np.float32), 1)
    Bm = oracle.binarize_pack(rng.standard_normal((N, K)).astype(np.float32), 1)
    got = B.xnor_gemm(dev(A.view(np.int64)), dev(Bm.view(np.int64)), K).cpu().numpy()
    np.testing.assert_array_equal(got, oracle.xnor_gemm(A, Bm, K))


@pytest.mark.parametrize("engine", [1, 2, 3])
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (5, 7, 63), (33, 65, 500), (70, 130, 1100), (256, 300, 4096)])
def test_xnor_gemm_count_range(M, N, K, engine):
    """The other range of Eq. 2: the number of agreeing positions, counted from the definition on
    the unpacked +-1 values, from every GEMM engine (rows padded to an even word count so that
    the matrix-core kernels take the problem)."""
    rng = np.random.default_rng(M + N + K)
    a = rng.standard_normal((M, K)).astype(np.float32)
    b = rng.standard_normal((N, K)).astype(np.float32)
    want = (oracle.sign(a)[:, None, :] == oracle.sign(b)[None, :, :]).sum(axis=2).astype(np.int32)

    def even_rows(x):
        p = oracle.binarize_pack(x, 1)
        out = np.zeros((p.shape[0], (p.shape[1] + 1) // 2 * 2), dtype=np.uint64)
        out[:, :p.shape[1]] = p
        return dev(out.view(np.int64))

    with tuned(k7=engine):
        got = B.xnor_gemm(even_rows(a), even_rows(b), K, count=True).cpu().numpy()
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(2 * got - K, oracle.xnor_gemm(oracle.binarize_pack(a, 1), oracle.binarize_pack(b, 1), K))


def test_xnor_gemm_wide_rows_and_invariants():
    """Row stride wider than ceil(K/64): extra words are ignored (they hold garbage here)."""
    rng = np.random.default_rng(5)
    M, N, K = 20, 40, 200
    a = rng.standard_normal((M, K)).astype(np.float32)
    A = oracle.binarize_pack(a, 1, out_ld_words=6, fill=POISON)
    Bm = oracle.binarize_pack(rng.standard_normal((N, K)).astype(np.float32), 1, out_ld_words=5,
                              fill=POISON)
    got = B.xnor_gemm(dev(A.view(np.int64)), dev(Bm.view(np.int64)), K).cpu().numpy()
    np.testing.assert_array_equal(got, oracle.xnor_gemm(A, Bm, K))
    assert (np.abs(got) <= K).all() and ((got - K) % 2 == 0).all()
    same = B.xnor_gemm(dev(A.view(np.int64)), dev(A.view(np.int64)), K).cpu().numpy()
    assert (np.diag(same) == K).all()


class tuned:
    """Pin kernel choices through bmx_tune_set for a block of code (results must not depend on them)."""

    def __init__(self, **kv):
        self.kv = kv

    def __enter__(self):
        for k, v in self.kv.items():
            assert B.lib().bmx_tune_set(int(k[1:]), v) == 0
        return self

    def __exit__(self, *exc):
        for k in self.kv:
            B.lib().bmx_tune_set(int(k[1:]), 0)


# every GEMM engine: automatic (FP4 matrix cores), xor/popcount, int8 matrix cores
GEMM_ENGINES = [dict(), dict(k7=1), dict(k7=2)]


# ------------------------------------------------------------------ binary FC
def test_config1_fc_gemm_exact():
    c = synth.config1()
    a, w_kn = c["a"], c["w_kn"]                       # A [64,512], W stored [K=512, N=256]
    Wp = B.binarize_pack(dev(w_kn), 0)                # pack down the K rows -> [256, 8]
    np.testing.assert_array_equal(host_u64(Wp), oracle.binarize_pack(w_kn, 0))
    got = B.binary_fc(dev(a), Wp, integer_out=True).cpu().numpy()
    assert "fc_small_kernel" in B.last_kernel()       # the one-launch form of very small layers
    ref, _ = oracle.binary_fc(a, w_kn.T.copy())
    assert got.dtype == np.int32 and got.shape == (64, 256)
    np.testing.assert_array_equal(got, ref)
    with tuned(k15=1):                                 # the general path: pack, then the GEMM
        got = B.binary_fc(dev(a), Wp, integer_out=True).cpu().numpy()
        assert "fc_small_kernel" not in B.last_kernel()
        np.testing.assert_array_equal(got, ref)
    # the same through pack + xnor_gemm
    Ap = B.binarize_pack(dev(a), 1)
    np.testing.assert_array_equal(B.xnor_gemm(Ap, Wp, 512).cpu().numpy(), ref)


@pytest.mark.parametrize("small", [True, False])
def test_config3_fc_chain(small):
    c = synth.config3(small=small)
    x, w1, w2 = c["x"], c["w1"], c["w2"]
    a1, a2 = oracle.alpha_mean_abs(w1), oracle.alpha_mean_abs(w2)
    W1p, W2p = B.binarize_pack(dev(w1), 1), B.binarize_pack(dev(w2), 1)
    r1i, r1f = oracle.binary_fc(x, w1, a1)
    r2i, r2f = oracle.binary_fc(r1f, w2, a2)
    for engine in GEMM_ENGINES:
        with tuned(**engine):
            h1 = B.binary_fc(dev(x), W1p, alpha=dev(a1))
            h2 = B.binary_fc(h1, W2p, alpha=dev(a2))
            i1 = B.binary_fc(dev(x), W1p, integer_out=True)
            np.testing.assert_array_equal(i1.cpu().numpy(), r1i)
            assert_f32_close(h1.cpu().numpy(), r1f)
            np.testing.assert_array_equal(h1.cpu().numpy(), r1f)   # one fp32 multiply: bit-identical
            assert_f32_close(h2.cpu().numpy(), r2f)
            i2 = B.binary_fc(h1, W2p, integer_out=True)
            np.testing.assert_array_equal(i2.cpu().numpy(), r2i)


@pytest.mark.parametrize("batch,fin,fout", [(1, 1, 1), (64, 512, 256), (7, 65, 3), (100, 1000, 70), (4096, 64, 1),
                                            (3, 64 * 33 + 5, 7), (2, 65536, 16), (33, 4000, 257), (1, 130, 5000)])
def test_fc_small_layers_one_launch(batch, fin, fout):
    """bmx_binary_fc on layers small enough for its one-launch form (sign bits of a batch row in
    LDS, xor + popcount per output feature): K tails inside a word, more and fewer than four
    words per wave, more than 256 output features, rows of x and of the output further apart
    than their length with poison between them, special values in x; int32 and scaled fp32."""
    rng = np.random.default_rng(batch + 3 * fin + 7 * fout)
    x = rng.standard_normal((batch, fin)).astype(np.float32)
    x.flat[:: 7] = 0.0
    x.flat[3:: 11] = -0.0
    x.flat[5:: 13] = np.nan
    x.flat[1:: 17] = np.inf
    x.flat[2:: 19] = -np.inf
    w = rng.uniform(-1, 1, (fout, fin)).astype(np.float32)
    alpha = rng.standard_normal(fout).astype(np.float32)
    alpha[::3] = 0.0
    ri, rf = oracle.binary_fc(x, w, alpha)
    Wp = B.binarize_pack(dev(w), 1)
    xw = torch.full((batch, fin + 5), float("nan"), dtype=torch.float32, device="cuda")   # rows fin + 5 apart
    xw[:, :fin] = dev(x)
    oi = torch.full((batch, fout + 3), -7, dtype=torch.int32, device="cuda")
    of = torch.full((batch, fout + 3), 123.0, dtype=torch.float32, device="cuda")
    B.binary_fc(xw[:, :fin], Wp, integer_out=True, out=oi[:, :fout])
    assert "fc_small_kernel" in B.last_kernel()
    B.binary_fc(xw[:, :fin], Wp, alpha=dev(alpha), out=of[:, :fout])
    assert "fc_small_kernel" in B.last_kernel()
    np.testing.assert_array_equal(oi[:, :fout].cpu().numpy(), ri)
    np.testing.assert_array_equal(of[:, :fout].cpu().numpy(), rf)      # one fp32 multiply: bit-identical
    assert (oi[:, fout:] == -7).all() and (of[:, fout:] == 123.0).all()
    np.testing.assert_array_equal(B.binary_fc(dev(x), Wp).cpu().numpy(), ri.astype(np.float32))
    with tuned(k15=1):
        np.testing.assert_array_equal(B.binary_fc(dev(x), Wp, integer_out=True).cpu().numpy(), ri)
        assert "fc_small_kernel" not in B.last_kernel()


@pytest.mark.parametrize("batch,fin,fout", [(1, 1, 1), (5, 27, 3), (3, 180, 70), (66, 1000, 130)])
def test_fc_ragged(batch, fin, fout):
    rng = np.random.default_rng(batch + fin + fout)
    x = rng.standard_normal((batch, fin)).astype(np.float32)
    w = rng.uniform(-1, 1, (fout, fin)).astype(np.float32)
    alpha = oracle.alpha_mean_abs(w)
    Wp = B.binarize_pack(dev(w), 1)
    ri, rf = oracle.binary_fc(x, w, alpha)
    np.testing.assert_array_equal(B.binary_fc(dev(x), Wp, integer_out=True).cpu().numpy(), ri)
    assert_f32_close(B.binary_fc(dev(x), Wp, alpha=dev(alpha)).cpu().numpy(), rf)


# ------------------------------------------------------------------ binary conv2d
CONV_CASES = [
    # N, C, H, W, O, k, s, p
    (1, 1, 1, 1, 1, 1, 1, 0),
    (2, 3, 5, 5, 4, 3, 1, 1),
    (1, 20, 8, 5, 3, 3, 2, 1),
    (2, 64, 5, 8, 5, 3, 1, 1),
    (1, 65, 8, 8, 2, 5, 2, 2),
    (1, 3, 8, 8, 2, 5, 1, 0),
    (1, 2, 2, 2, 3, 3, 1, 1),
    (2, 4, 7, 7, 3, 1, 2, 0),
    (1, 5, 9, 9, 2, 7, 1, 3),
    (3, 130, 9, 11, 70, 3, 1, 1),
    (2, 64, 56, 56, 64, 3, 1, 1),
    (2, 128, 28, 28, 128, 3, 2, 1),
    (1, 256, 14, 14, 19, 3, 1, 2),
]


def run_conv(x, w, s, p, alpha=None, integer_out=False):
    O, C, KH, KW = w.shape
    Wp = B.pack_conv_weights(dev(w))
    out = B.binary_conv2d(dev(x), Wp, O, KH, KW, s, p, alpha=None if alpha is None else dev(alpha),
                          integer_out=integer_out)
    return out.cpu().numpy()


@pytest.mark.parametrize("N,C,H,W,O,k,s,p", CONV_CASES)
def test_conv_cases(N, C, H, W, O, k, s, p):
    rng = np.random.default_rng(N + 10 * C + 100 * H + 1000 * O + k + s + p)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((O, C, k, k)).astype(np.float32)
    alpha = oracle.alpha_mean_abs(w)
    ri, rf = oracle.binary_conv2d(x, w, s, p, alpha)
    np.testing.assert_array_equal(run_conv(x, w, s, p, integer_out=True), ri)
    got = run_conv(x, w, s, p, alpha=alpha)
    assert_f32_close(got, rf)


def test_conv_output_offsets_beyond_two_gib():
    """A convolution whose fp32 output is 3.3 GB (130 x 512 x 112 x 112): the short-K matrix-core
    kernel addresses its output with 32-bit byte offsets from a uniform base, which here pass
    2^31.  The first, one middle and the last image against the oracle (image by image: the
    oracle would need minutes for the whole batch), every other image against the popcount
    kernel on a sample of rows."""
    N, C, H, W, O = 130, 64, 112, 112, 512
    gen = torch.Generator(device="cuda").manual_seed(130)
    x = torch.randn((N, C, H, W), device="cuda", generator=gen)
    rng = np.random.default_rng(130)
    w = rng.standard_normal((O, C, 3, 3)).astype(np.float32)
    alpha = oracle.alpha_mean_abs(w)
    Wp = B.pack_conv_weights(dev(w))
    got = B.binary_conv2d(x, Wp, O, 3, 3, 1, 1, alpha=dev(alpha))
    assert "conv_mfma_ws_kernel" in B.last_kernel()
    assert got.shape == (N, O, H, W) and got.numel() * 4 > 2 ** 31
    for n in (0, 77, N - 1):
        _, rf = oracle.binary_conv2d(x[n:n + 1].cpu().numpy(), w, 1, 1, alpha)
        assert_f32_close(got[n:n + 1].cpu().numpy(), rf)
    with tuned(k5=1):
        ref = B.binary_conv2d(x, Wp, O, 3, 3, 1, 1, alpha=dev(alpha))
        assert "conv_stationary_kernel" in B.last_kernel()
    assert torch.equal(got[:, ::37], ref[:, ::37])
    del got, ref, x
    torch.cuda.empty_cache()


def test_conv_padding_closed_form_on_gpu():
    C, H, W, O = 5, 6, 6, 2
    K = 9 * C
    wp = np.ones((O, C, 3, 3), dtype=np.float32)
    assert (run_conv(np.ones((1, C, H, W), dtype=np.float32), wp, 1, 1, integer_out=True) == K).all()
    x = -np.ones((1, C, H, W), dtype=np.float32)
    np.testing.assert_array_equal(run_conv(x, wp, 1, 1, integer_out=True),
                                  oracle.binary_conv2d(x, wp, 1, 1)[0])


def test_config2_conv_full():
    c = synth.config2()
    alpha = oracle.alpha_mean_abs(c["w"])
    assert_f32_close(B.alpha_mean_abs(dev(c["w"])).cpu().numpy(), alpha)
    ri, rf = oracle.binary_conv2d(c["x"], c["w"], 1, 1, alpha)
    # automatic (the short-K FP4 matrix-core kernel with its filters in LDS; k5=5 names it),
    # register-stationary xor/popcount kernel, xor/popcount GEMM kernel, GEMM-shaped FP4 and
    # int8 matrix-core kernels
    for choice in (dict(), dict(k5=1), dict(k5=5), dict(k5=2), dict(k5=4), dict(k5=4, k7=2)):
        with tuned(**choice):
            got = run_conv(c["x"], c["w"], 1, 1, alpha=alpha)
            assert got.shape == (16, 64, 56, 56)
            assert_f32_close(got, rf)
            np.testing.assert_array_equal(run_conv(c["x"], c["w"], 1, 1, integer_out=True), ri)


@pytest.mark.parametrize("stride", [1, 2])
def test_config4_conv_full(stride):
    c = synth.config4(stride=stride)
    frac_pos = (c["x"] >= 0).mean()
    assert 0.60 < frac_pos < 0.635                     # skewed sign balance, P(|z| >= 0.5) = 0.617
    alpha = oracle.alpha_mean_abs(c["w"])
    ri, rf = oracle.binary_conv2d(c["x"], c["w"], stride, 1, alpha)
    # automatic (the short-K FP4 matrix-core kernel, 36 words of K), register-stationary
    # xor/popcount kernel, xor/popcount GEMM kernel, GEMM-shaped FP4 and int8 matrix-core kernels,
    # the 64 x 64 per wave FP4 kernel's convolution form
    for choice in (dict(), dict(k14=1), dict(k14=2), dict(k14=3), dict(k5=1), dict(k5=2), dict(k5=4), dict(k5=4, k7=2), dict(k5=6)):
        with tuned(**choice):
            got = run_conv(c["x"], c["w"], stride, 1, alpha=alpha)
            assert got.shape == (64, 256, 14 // stride, 14 // stride)
            assert_f32_close(got, rf)
            np.testing.assert_array_equal(run_conv(c["x"], c["w"], stride, 1, integer_out=True), ri)


# ------------------------------------------------------------------ alpha helper
@pytest.mark.parametrize("rows,cols", [(1, 1), (3, 7), (64, 576), (5, 9216)])
def test_alpha_mean_abs(rows, cols):
    rng = np.random.default_rng(rows + cols)
    w = rng.uniform(-1, 1, (rows, cols)).astype(np.float32)
    assert_f32_close(B.alpha_mean_abs(dev(w)).cpu().numpy(), oracle.alpha_mean_abs(w))


# ------------------------------------------------------------------ k-bit GEMM
@pytest.mark.parametrize("bits", [1, 2, 3, 4, 8])
def test_quant_gemm_small(bits):
    rng = np.random.default_rng(bits)
    M, N, K = 37, 70, 333
    a = rng.uniform(0, 1, (M, K)).astype(np.float32)
    a[0, :6] = [1 / 6, 5 / 6, 0.5, 0.0, 1.0, 0.25]      # tie inputs of the quantiser
    a[1, :4] = [-0.5, 1.5, -0.0, 2.0]                   # clamped
    w = rng.standard_normal((N, K)).astype(np.float32)
    S, of = B.quant_gemm(dev(a), dev(w), bits)
    rS, r64, r32 = oracle.quant_gemm(a, w, bits)
    np.testing.assert_array_equal(S.cpu().numpy(), rS)
    assert_f32_close(of.cpu().numpy(), r64, atol=1e-9)
    assert_f32_close(of.cpu().numpy(), r32)


@pytest.mark.parametrize("engine", [0, 1])
@pytest.mark.parametrize("ba,bw", [(1, 2), (2, 2), (2, 3), (3, 2), (4, 4), (8, 8), (2, 8)])
def test_quant_gemm_kbit_weights(ba, bw, engine):
    """k-bit weights: w in [-1, 1] through the affine pair around Eq. 1.  Integer S exact, the
    float within 1e-6; tie and clamp inputs on both operands, ragged shapes, the matrix-core and
    the xor/popcount engine."""
    rng = np.random.default_rng(10 * ba + bw)
    M, N, K = 37, 45, 333
    a = rng.uniform(0, 1, (M, K)).astype(np.float32)
    a[0, :6] = [1 / 6, 5 / 6, 0.5, 0.0, 1.0, 0.25]
    w = rng.uniform(-1, 1, (N, K)).astype(np.float32)
    w[0, :8] = [0.0, -0.0, 1.0, -1.0, 1.5, -2.0, 1 / 3, -1 / 3]      # ties of u = 1/2, clamps
    rS, r64, r32 = oracle.quant_gemm(a, w, ba, bw)
    with tuned(k7=engine):
        S, of = B.quant_gemm(dev(a), dev(w), ba, bits_w=bw)
    np.testing.assert_array_equal(S.cpu().numpy(), rS)
    assert_f32_close(of.cpu().numpy(), r32)
    assert_f32_close(of.cpu().numpy(), r64, atol=1e-9)


def test_config5_quant_gemm():
    c = synth.config5(small=True)
    S, of = B.quant_gemm(dev(c["a"]), dev(c["w"]), 2)
    rS, r64, r32 = oracle.quant_gemm(c["a"], c["w"], 2)
    np.testing.assert_array_equal(S.cpu().numpy(), rS)
    assert_f32_close(of.cpu().numpy(), r64, atol=1e-9)
    assert_f32_close(of.cpu().numpy(), r32)


def test_config5_quant_gemm_full_size():
    """Full 1024 x 1024 x 4096, 2-bit activations x 1-bit weights: every element of S and of the
    scaled output against the oracle, on every GEMM engine."""
    c = synth.config5()
    rS, r64, r32 = oracle.quant_gemm(c["a"], c["w"], 2)
    assert (np.abs(rS) <= 3 * 4096).all()
    for engine in GEMM_ENGINES:
        with tuned(**engine):
            S, of = B.quant_gemm(dev(c["a"]), dev(c["w"]), 2)
        np.testing.assert_array_equal(S.cpu().numpy(), rS)
        assert_f32_close(of.cpu().numpy(), r64, atol=1e-9)
        assert_f32_close(of.cpu().numpy(), r32)


def test_quant_gemm_long_k_leaves_fp4_range():
    """K * (2^bits - 1) >= 2^24: fp32 sums could round, so the launcher must take the int8 form
    (int32 accumulation); the result stays exact."""
    M, N, K = 2, 3, 5_700_000
    rng = np.random.default_rng(77)
    a = rng.uniform(0, 1, (M, K)).astype(np.float32)
    a[0] = 1.0                                  # q = 3 everywhere: the largest possible sums
    w = rng.standard_normal((N, K)).astype(np.float32)
    w[0] = 1.0
    S, of = B.quant_gemm(dev(a), dev(w), 2)
    rS, r64, r32 = oracle.quant_gemm(a, w, 2)
    assert rS[0, 0] == 3 * K and 3 * K > (1 << 24)
    np.testing.assert_array_equal(S.cpu().numpy(), rS)
    assert_f32_close(of.cpu().numpy(), r32)


# ------------------------------------------------------------------ determinism, empties
def test_repeatable_and_empty():
    c = synth.config2(small=True)
    alpha = oracle.alpha_mean_abs(c["w"])
    a = run_conv(c["x"], c["w"], 1, 1, alpha=alpha)
    b = run_conv(c["x"], c["w"], 1, 1, alpha=alpha)
    assert a.tobytes() == b.tobytes()
    e = B.binarize_pack(torch.empty((0, 64), dtype=torch.float32, device="cuda"), 1)
    assert e.shape == (0, 1)
    z = B.xnor_gemm(torch.empty((0, 1), dtype=torch.int64, device="cuda"),
                    torch.empty((5, 1), dtype=torch.int64, device="cuda"), 64)
    assert z.shape == (0, 5)


# ------------------------------------------------------------------ GEMM kernel shapes
@pytest.mark.parametrize("rows_per_wave", [8, 16, 32])
@pytest.mark.parametrize("ksplit", [1, 2, 3, 8])
def test_gemm_every_kernel_shape(rows_per_wave, ksplit):
    """Every (rows per wave, K split, workgroup order) the launcher can pick, forced through
    the tuning hook, on shapes with ragged rows, columns, K tails and bit planes."""
    L = B.lib()
    rng = np.random.default_rng(rows_per_wave * 10 + ksplit)
    try:
        assert L.bmx_tune_set(7, 1) == 0  # the xor/popcount engine
        for order in (0, 1):
            assert L.bmx_tune_set(2, rows_per_wave) == 0
            assert L.bmx_tune_set(3, ksplit) == 0
            assert L.bmx_tune_set(4, order) == 0
            for (M, N, K) in [(37, 70, 5000), (8, 64, 1024), (100, 129, 3072 + 64)]:
                A = oracle.binarize_pack(rng.standard_normal((M, K)).astype(np.float32), 1)
                Bm = oracle.binarize_pack(rng.standard_normal((N, K)).astype(np.float32), 1)
                got = B.xnor_gemm(dev(A.view(np.int64)), dev(Bm.view(np.int64)), K).cpu().numpy()
                np.testing.assert_array_equal(got, oracle.xnor_gemm(A, Bm, K))
            x = rng.standard_normal((19, 2500)).astype(np.float32)
            w = rng.uniform(-1, 1, (75, 2500)).astype(np.float32)
            alpha = oracle.alpha_mean_abs(w)
            ri, rf = oracle.binary_fc(x, w, alpha)
            Wp = B.binarize_pack(dev(w), 1)
            np.testing.assert_array_equal(B.binary_fc(dev(x), Wp, integer_out=True).cpu().numpy(), ri)
            assert_f32_close(B.binary_fc(dev(x), Wp, alpha=dev(alpha)).cpu().numpy(), rf)
            for bits in (1, 3):
                if rows_per_wave < bits:
                    continue
                a = rng.uniform(0, 1, (21, 2200)).astype(np.float32)
                wq = rng.standard_normal((70, 2200)).astype(np.float32)
                S, f = B.quant_gemm(dev(a), dev(wq), bits)
                rS, r64, r32 = oracle.quant_gemm(a, wq, bits)
                np.testing.assert_array_equal(S.cpu().numpy(), rS)
                assert_f32_close(f.cpu().numpy(), r32)
    finally:
        for key in (2, 3, 4, 7):
            L.bmx_tune_set(key, 0)


@pytest.mark.parametrize("engine", [2, 3])
@pytest.mark.parametrize("ksplit", [0, 1, 2, 3, 8])
def test_gemm_matrix_core_engine(ksplit, engine):
    """The matrix-core kernel (bits expanded in registers to int8, engine 2, or to FP4 nibbles,
    engine 3), forced through the tuning hook: ragged tiles in M and N, K tails inside and at
    the end of a 1024-bit step, every K split, every output kind."""
    L = B.lib()
    rng = np.random.default_rng(100 + ksplit)
    try:
        assert L.bmx_tune_set(7, engine) == 0
        assert L.bmx_tune_set(8, ksplit) == 0
        for (M, N, K) in [(37, 70, 5000), (8, 64, 1024), (100, 129, 3072 + 64), (1, 1, 1), (64, 64, 63),
                          (65, 33, 1025), (130, 200, 2048 + 128),
                          # enough tiles for the 64 x 64 per wave variant
                          (700, 801, 1100), (1031, 640, 2048 + 64)]:
            A = oracle.binarize_pack(rng.standard_normal((M, K)).astype(np.float32), 1)
            Bm = oracle.binarize_pack(rng.standard_normal((N, K)).astype(np.float32), 1)
            # rows padded to an even number of words: the kernel's 16-byte pieces need it
            ld = (A.shape[1] + 1) // 2 * 2
            Ad = np.zeros((M, ld), dtype=np.uint64); Ad[:, :A.shape[1]] = A
            Bd = np.zeros((N, ld), dtype=np.uint64); Bd[:, :A.shape[1]] = Bm
            got = B.xnor_gemm(dev(Ad.view(np.int64)), dev(Bd.view(np.int64)), K).cpu().numpy()
            np.testing.assert_array_equal(got, oracle.xnor_gemm(A, Bm, K))
        for (batch, fin, fout) in [(19, 2500, 75), (70, 4096, 130)]:
            x = rng.standard_normal((batch, fin)).astype(np.float32)
            w = rng.uniform(-1, 1, (fout, fin)).astype(np.float32)
            alpha = oracle.alpha_mean_abs(w)
            ri, rf = oracle.binary_fc(x, w, alpha)
            Wp = B.binarize_pack(dev(w), 1)
            np.testing.assert_array_equal(B.binary_fc(dev(x), Wp, integer_out=True).cpu().numpy(), ri)
            assert_f32_close(B.binary_fc(dev(x), Wp, alpha=dev(alpha)).cpu().numpy(), rf)
            assert_f32_close(B.binary_fc(dev(x), Wp).cpu().numpy(), ri.astype(np.float32))
        # k-bit activations (1 and 2 bit planes assembled into the int8 operand)
        for bits in (1, 2):
            for (M, N, K) in [(21, 70, 2200), (1, 1, 1), (33, 65, 1024), (100, 130, 4096 + 200)]:
                a = rng.uniform(0, 1, (M, K)).astype(np.float32)
                a[rng.random(a.shape) < 0.05] = 0.5  # a rounding tie of Eq. 1 for k = 2
                wq = rng.standard_normal((N, K)).astype(np.float32)
                Sg, fg = B.quant_gemm(dev(a), dev(wq), bits)
                rS, r64, r32 = oracle.quant_gemm(a, wq, bits)
                np.testing.assert_array_equal(Sg.cpu().numpy(), rS)
                assert_f32_close(fg.cpu().numpy(), r32)
    finally:
        L.bmx_tune_set(7, 0)
        L.bmx_tune_set(8, 0)


# ------------------------------------------------------------------ convolution kernel paths
BIG_K_CONV_CASES = [
    # K beyond the 36 words the register-stationary kernel holds: runs on the GEMM kernel
    # N, C, H, W, O, k, s, p
    (1, 320, 6, 7, 20, 3, 1, 1),      # 45 words, 24-dword chunks
    (2, 128, 9, 9, 33, 5, 2, 2),      # 50 words
    (1, 64, 12, 12, 5, 7, 1, 3),      # 49 words
    (2, 500, 5, 5, 70, 1, 1, 0),      # 8 words, 1x1, ragged channels
    (1, 1024, 4, 4, 17, 3, 1, 1),     # 144 words, many chunks
    (3, 200, 12, 12, 64, 5, 1, 0),    # the paper's efficiency shape (5x5, 64 filters, 8x8 out)
]


@pytest.mark.parametrize("N,C,H,W,O,k,s,p", BIG_K_CONV_CASES)
def test_conv_big_k(N, C, H, W, O, k, s, p):
    rng = np.random.default_rng(N + 10 * C + 100 * H + 1000 * O + k + s + p)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((O, C, k, k)).astype(np.float32)
    alpha = oracle.alpha_mean_abs(w)
    ri, rf = oracle.binary_conv2d(x, w, s, p, alpha)
    np.testing.assert_array_equal(run_conv(x, w, s, p, integer_out=True), ri)
    assert_f32_close(run_conv(x, w, s, p, alpha=alpha), rf)


@pytest.mark.parametrize("path", [1, 2, 3, 4])
def test_conv_every_path(path):
    """The four convolution kernels (register-stationary, GEMM kernel, one-thread-per-output,
    matrix cores), each forced through the tuning hook on the shapes it accepts, with every K
    split."""
    L = B.lib()
    try:
        assert L.bmx_tune_set(5, path) == 0
        for ksplit in ((0, 2, 3) if path in (2, 4) else (0,)):
            L.bmx_tune_set(3, ksplit)
            L.bmx_tune_set(8, ksplit)
            L.bmx_tune_set(7, 2 if (path == 4 and ksplit == 2) else 0)  # int8 form once, FP4 otherwise
            for (N, C, H, W, O, k, s, p) in (CONV_CASES if path == 4 else CONV_CASES[:10]) + BIG_K_CONV_CASES[:2]:
                rng = np.random.default_rng(N + 10 * C + 100 * H + 1000 * O + k + s + p + path)
                x = rng.standard_normal((N, C, H, W)).astype(np.float32)
                w = rng.standard_normal((O, C, k, k)).astype(np.float32)
                alpha = oracle.alpha_mean_abs(w)
                ri, rf = oracle.binary_conv2d(x, w, s, p, alpha)
                np.testing.assert_array_equal(run_conv(x, w, s, p, integer_out=True), ri)
                assert_f32_close(run_conv(x, w, s, p, alpha=alpha), rf)
    finally:
        L.bmx_tune_set(5, 0)
        L.bmx_tune_set(3, 0)
        L.bmx_tune_set(8, 0)
        L.bmx_tune_set(7, 0)


WS_CONV_CASES = [
    # N, C, H, W, O, s, p   (3x3 with 9, 18, 27 or 36 words of K: the short-K matrix-core kernel)
    (1, 1, 3, 3, 1, 1, 0),
    (2, 3, 5, 5, 4, 1, 1),
    (1, 20, 8, 5, 3, 2, 1),
    (2, 64, 5, 8, 5, 1, 1),
    (3, 33, 7, 9, 70, 1, 2),
    (2, 64, 56, 56, 64, 1, 1),
    (1, 32, 57, 57, 130, 2, 0),
    (2, 128, 28, 28, 128, 2, 1),
    (3, 100, 9, 11, 33, 1, 1),
    (1, 256, 14, 14, 19, 1, 2),
    (5, 200, 9, 9, 256, 1, 1),
    (64, 256, 14, 14, 40, 2, 1),
    (2, 192, 14, 14, 70, 1, 1),
    (3, 130, 9, 11, 33, 2, 1),
    (70, 200, 14, 14, 250, 1, 1),     # 429 blocks x 8 filter tiles: a wave per block at four waves per SIMD
]


@pytest.mark.parametrize("N,C,H,W,O,s,p", WS_CONV_CASES)
def test_conv_short_k_matrix_core(N, C, H, W, O, s, p):
    """The convolution kernel that reads pre-expanded FP4 filters from LDS and streams pixel
    blocks through the matrix cores, forced through the tuning hook: ragged filter and pixel
    tiles, both filter-tile heights, several blocks per wave (a fixed count, and an uneven deal
    of the blocks over 101 waves), every output kind."""
    L = B.lib()
    rng = np.random.default_rng(N + 10 * C + 100 * H + 1000 * O + s + p)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    x[rng.random(x.shape) < 0.05] = 0.0
    w = rng.standard_normal((O, C, 3, 3)).astype(np.float32)
    alpha = oracle.alpha_mean_abs(w)
    ri, rf = oracle.binary_conv2d(x, w, s, p, alpha)
    # (narrow = 1: pixel words fetched 8 bytes at a time also where an even number of channel
    # words lets the kernel fetch 16)
    # (narrow = 2: 16 at a time, but not in the form for channel-word counts that are multiples
    # of four, which those cases take by themselves)
    # (narrow = 3: never the form that holds one block per wave in 128 registers)
    for tile, per_wave, narrow in ((0, 0, 0), (2, 3, 0), (0, 7, 0), (0, 101, 0), (0, 0, 1), (0, 3, 1), (0, 0, 2), (0, 3, 2),
                                   (0, 0, 3)):
        with tuned(k5=5, k9=tile, k1=per_wave, k14=narrow):
            np.testing.assert_array_equal(run_conv(x, w, s, p, integer_out=True), ri)
            assert_f32_close(run_conv(x, w, s, p, alpha=alpha), rf)
            np.testing.assert_array_equal(run_conv(x, w, s, p), ri.astype(np.float32))


@pytest.mark.parametrize("N,C,H,W,O,s,p", [(1, 1, 5, 5, 1, 1, 0), (2, 64, 12, 12, 64, 1, 0), (3, 20, 9, 11, 70, 2, 2),
                                           (200, 64, 12, 12, 64, 1, 0), (2, 50, 30, 17, 33, 1, 4),
                                           (2, 100, 13, 9, 40, 1, 2), (200, 128, 12, 12, 64, 1, 0)])
def test_conv_short_k_matrix_core_5x5(N, C, H, W, O, s, p):
    """5 x 5 kernels over one or two channel words (K = 25 and 50 words, the first two points of
    the paper's Sec. 3.1 sweep) on the same kernel: an odd word count, several blocks per wave,
    every output kind."""
    rng = np.random.default_rng(N + 10 * C + 100 * H + 1000 * O + s + p)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((O, C, 5, 5)).astype(np.float32)
    alpha = oracle.alpha_mean_abs(w)
    ri, rf = oracle.binary_conv2d(x, w, s, p, alpha)
    for per_wave, narrow in ((0, 0), (3, 0), (101, 0), (0, 1), (3, 1)):
        with tuned(k5=5, k1=per_wave, k14=narrow):
            np.testing.assert_array_equal(run_conv(x, w, s, p, integer_out=True), ri)
            assert_f32_close(run_conv(x, w, s, p, alpha=alpha), rf)
    Wp, xp = B.pack_conv_weights(dev(w)), B.pack_nchw(dev(x), p)
    img = B.binary_conv2d_bits(xp, C, Wp, O, 5, 5, s, p, alpha=dev(alpha), out_pad=2)
    np.testing.assert_array_equal(host_u64(img), packed_image(rf >= 0.0, 2))


@pytest.mark.parametrize("N,C,H,W,O,s,p", [(1, 1, 7, 7, 1, 1, 0), (2, 64, 15, 14, 70, 1, 3), (3, 3, 40, 33, 64, 2, 3)])
def test_conv_short_k_matrix_core_7x7(N, C, H, W, O, s, p):
    """7 x 7 kernels over one channel word (K = 49 words; the first layer of a ResNet has this
    shape class) on the short-K kernel, forced, several blocks per wave."""
    rng = np.random.default_rng(N + 10 * C + 100 * H + 1000 * O + s + p)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((O, C, 7, 7)).astype(np.float32)
    alpha = oracle.alpha_mean_abs(w)
    ri, rf = oracle.binary_conv2d(x, w, s, p, alpha)
    for per_wave in (0, 2, 101):
        with tuned(k5=5, k1=per_wave):
            np.testing.assert_array_equal(run_conv(x, w, s, p, integer_out=True), ri)
            assert_f32_close(run_conv(x, w, s, p, alpha=alpha), rf)
    Wp, xp = B.pack_conv_weights(dev(w)), B.pack_nchw(dev(x), p)
    img = B.binary_conv2d_bits(xp, C, Wp, O, 7, 7, s, p, alpha=dev(alpha), out_pad=1)
    np.testing.assert_array_equal(host_u64(img), packed_image(rf >= 0.0, 1))


def test_conv_weight_rows_are_zero_padded():
    """Packed filter rows are as long as bmx_conv_weight_row_words says: the bits (zero past the
    data up to a whole register chunk), and for the K the short-K matrix-core kernel takes
    (9, 18, 25, 27, 36, 49 or 50 words) two more words holding the float K - 2 * popcount(filter)
    and zeros."""
    rng = np.random.default_rng(3)
    for (O, C, k) in [(3, 64, 3), (2, 256, 3), (2, 130, 5), (4, 1, 1), (5, 100, 3), (3, 40, 5), (3, 130, 3), (3, 70, 5), (2, 20, 7)]:
        w = rng.standard_normal((O, C, k, k)).astype(np.float32)
        Wp = host_u64(B.pack_conv_weights(dev(w)))
        kwords = k * k * ((C + 63) // 64)
        assert Wp.shape == (O, B.lib().bmx_conv_weight_row_words(C, k, k)) and Wp.shape[1] >= kwords
        ref = oracle.binarize_pack(np.transpose(w, (0, 2, 3, 1)).reshape(O * k * k, C), 1)
        ref = ref.reshape(O, kwords)
        np.testing.assert_array_equal(Wp[:, :kwords], ref)
        if kwords not in (9, 18, 25, 27, 36, 49, 50):
            assert (Wp[:, kwords:] == 0).all()
            continue
        ldb = Wp.shape[1] - 2
        assert ldb >= kwords and (Wp[:, kwords:ldb] == 0).all() and Wp.shape[1] % 2 == 0
        consts = Wp[:, ldb:].copy().view(np.float32)
        pc = np.array([[bin(int(v)).count("1") for v in row] for row in ref]).sum(axis=1)
        np.testing.assert_array_equal(consts[:, 0], (C * k * k - 2 * pc).astype(np.float32))
        assert (consts[:, 1:] == 0).all()


# ------------------------------------------------------------------ chained FC on packed bits
@pytest.mark.parametrize("small", [True, False])
def test_fc_packed_chain(small):
    """Two chained binary layers that hand packed sign bits to each other: the bits must be
    exactly what packing the first layer's fp32 output gives, and the second layer's output
    the same as through the fp32 route."""
    c = synth.config3(small=small)
    x, w1, w2 = c["x"], c["w1"], c["w2"]
    a1, a2 = oracle.alpha_mean_abs(w1), oracle.alpha_mean_abs(w2)
    r1i, r1f = oracle.binary_fc(x, w1, a1)
    r2i, r2f = oracle.binary_fc(r1f, w2, a2)
    W1p, W2p = B.binarize_pack(dev(w1), 1), B.binarize_pack(dev(w2), 1)
    Xp = B.binarize_pack(dev(x), 1)
    bits1 = B.binary_fc_packed(Xp, x.shape[1], W1p, alpha=dev(a1), mode="bits")
    np.testing.assert_array_equal(host_u64(bits1), oracle.binarize_pack(r1f, 1))
    np.testing.assert_array_equal(B.binary_fc_packed(Xp, x.shape[1], W1p, mode="i32").cpu().numpy(), r1i)
    h2 = B.binary_fc_packed(bits1, w1.shape[0], W2p, alpha=dev(a2), mode="f32")
    assert_f32_close(h2.cpu().numpy(), r2f)
    np.testing.assert_array_equal(B.binary_fc_packed(bits1, w1.shape[0], W2p, mode="i32").cpu().numpy(), r2i)


@pytest.mark.parametrize("engine", [1, 2, 3])
@pytest.mark.parametrize("batch,fin,fout", [(1, 1, 1), (5, 27, 3), (3, 180, 70), (66, 1000, 130), (9, 2100, 64),
                                            (300, 1100, 700)])
def test_fc_packed_bits_ragged(batch, fin, fout, engine):
    """Ragged shapes, poisoned output, and scales of either sign and zero: the bit is the
    IEEE compare (alpha * dot >= 0) of the fp32 product, as bmx_binarize_pack would see it.
    Every GEMM engine (xor/popcount, int8 and FP4 matrix cores), forced through the tuning hook; rows
    are padded to an even word count, which the matrix-core kernel needs to take the problem."""
    rng = np.random.default_rng(batch + fin + fout)
    x = rng.standard_normal((batch, fin)).astype(np.float32)
    w = rng.uniform(-1, 1, (fout, fin)).astype(np.float32)
    alpha = rng.standard_normal(fout).astype(np.float32)
    alpha[::3] = 0.0
    _, rf = oracle.binary_fc(x, w, alpha)

    def even_rows(a):
        p = oracle.binarize_pack(a, 1)
        out = np.zeros((p.shape[0], (p.shape[1] + 1) // 2 * 2), dtype=np.uint64)
        out[:, :p.shape[1]] = p
        return dev(out.view(np.int64))

    Xp, Wp = even_rows(x), even_rows(w)
    L = B.lib()
    try:
        assert L.bmx_tune_set(7, engine) == 0
        out = dev(np.full((batch, (fout + 63) // 64 + 1), -1, dtype=np.int64))   # one spare word
        B.binary_fc_packed(Xp, fin, Wp, alpha=dev(alpha), mode="bits", out=out)
        got = host_u64(out)
        np.testing.assert_array_equal(got[:, :-1], oracle.binarize_pack(rf, 1))
        assert (got[:, -1] == np.uint64(0xFFFFFFFFFFFFFFFF)).all()              # spare word untouched
        nob = B.binary_fc_packed(Xp, fin, Wp, mode="bits")                       # no scale: sign of dot
        ri, _ = oracle.binary_fc(x, w)
        np.testing.assert_array_equal(host_u64(nob), oracle.binarize_pack(ri.astype(np.float32), 1))
        # a folded BatchNorm threshold per feature: bit = (alpha * dot >= thr) in fp32
        thr = (rng.standard_normal(fout) * np.sqrt(fin)).astype(np.float32)
        thr[1::4] = 0.0
        tb = B.binary_fc_packed(Xp, fin, Wp, alpha=dev(alpha), mode="bits", thr=dev(thr))
        want = np.where(rf >= thr[None, :], 1.0, -1.0).astype(np.float32)
        np.testing.assert_array_equal(host_u64(tb), oracle.binarize_pack(want, 1))
    finally:
        L.bmx_tune_set(7, 0)


# ------------------------------------------------------------------ convolutions chained on packed images
def packed_image(bits_nchw, out_pad):
    """[N, O, Ho, Wo] booleans -> the packed image bmx_pack_nchw would hand the next layer:
    [N, Ho + 2*out_pad, Wo + 2*out_pad, ceil(O/64)] words, halo = every real channel set."""
    N, O, Ho, Wo = bits_nchw.shape
    rows = np.where(bits_nchw.transpose(0, 2, 3, 1).reshape(-1, O), 1.0, -1.0).astype(np.float32)
    words = oracle.binarize_pack(rows, 1)
    halo = oracle.binarize_pack(np.ones((1, O), dtype=np.float32), 1)[0]
    img = np.empty((N, Ho + 2 * out_pad, Wo + 2 * out_pad, words.shape[1]), dtype=np.uint64)
    img[:] = halo
    img[:, out_pad:out_pad + Ho, out_pad:out_pad + Wo, :] = words.reshape(N, Ho, Wo, -1)
    return img


CONV_BITS_CASES = [c + (op,) for c, op in zip(
    [(N, C, H, W, O, 3, s, p) for (N, C, H, W, O, s, p) in WS_CONV_CASES] + CONV_CASES,
    [1, 0, 2, 1, 3, 1, 0, 1, 2, 1, 1, 6, 1, 2, 1] + [1, 0, 1, 2, 1, 0, 1, 1, 3, 1, 1, 0, 2])]


@pytest.mark.parametrize("N,C,H,W,O,k,s,p,out_pad", CONV_BITS_CASES)
def test_conv_packed_bits(N, C, H, W, O, k, s, p, out_pad):
    """The convolution that hands the next one its packed image: bit o of a pixel is the fp32
    compare (alpha * dot >= thr), thr folded from a BatchNorm or absent, scales of either sign
    and zero; the halo carries the +1 of the next layer's zero padding; the image is written
    whole (poisoned beforehand).  3 x 3 kernels over up to 256 channels take the kernel that
    writes the bits itself, the rest go through the fp32 result and the channel pack."""
    rng = np.random.default_rng(7 + N + 10 * C + 100 * H + 1000 * O + k + s + p)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((O, C, k, k)).astype(np.float32)
    alpha = rng.standard_normal(O).astype(np.float32)
    alpha[::5] = 0.0
    thr = (rng.standard_normal(O) * np.sqrt(C * k * k)).astype(np.float32)
    thr[1::4] = 0.0
    ri, rf = oracle.binary_conv2d(x, w, s, p, alpha)
    Ho, Wo = ri.shape[2:]
    Wp = B.pack_conv_weights(dev(w))
    xp = B.pack_nchw(dev(x), p)
    shape = (N, Ho + 2 * out_pad, Wo + 2 * out_pad, (O + 63) // 64)
    # (four channel words: also the general form of the 16-byte pixel loads)
    for narrow in ((0, 2) if k == 3 and 192 < C <= 256 else (0,)):
        for al, th, ref in ((alpha, thr, rf >= thr[None, :, None, None]),
                            (alpha, None, rf >= 0.0),
                            (None, thr, ri.astype(np.float32) >= thr[None, :, None, None]),
                            (None, None, ri >= 0)):
            out = dev(np.full(shape, -1, dtype=np.int64))
            with tuned(k14=narrow):
                B.binary_conv2d_bits(xp, C, Wp, O, k, k, s, p, alpha=None if al is None else dev(al),
                                     thr=None if th is None else dev(th), out_pad=out_pad, out=out)
            np.testing.assert_array_equal(host_u64(out), packed_image(ref, out_pad))


@pytest.mark.parametrize("N,C,H,W,O1,O2,s1", [(2, 64, 20, 20, 64, 48, 1), (3, 100, 17, 13, 130, 70, 2),
                                               (16, 64, 56, 56, 64, 64, 1)])
def test_conv_chain_on_packed_images(N, C, H, W, O1, O2, s1):
    """Two binary blocks chained without an fp32 feature map in between: the second layer reads
    the image the first wrote, and matches the oracle run on the +-1 feature map (zero padded
    before the sign, like every layer input)."""
    rng = np.random.default_rng(N + C + H + O1 + O2)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w1 = rng.standard_normal((O1, C, 3, 3)).astype(np.float32)
    w2 = rng.standard_normal((O2, O1, 3, 3)).astype(np.float32)
    a1, a2 = oracle.alpha_mean_abs(w1), oracle.alpha_mean_abs(w2)
    thr = (rng.standard_normal(O1) * 5.0).astype(np.float32)
    _, r1 = oracle.binary_conv2d(x, w1, s1, 1, a1)
    h1 = np.where(r1 >= thr[None, :, None, None], 1.0, -1.0).astype(np.float32)
    r2i, r2f = oracle.binary_conv2d(h1, w2, 1, 1, a2)
    W1p, W2p = B.pack_conv_weights(dev(w1)), B.pack_conv_weights(dev(w2))
    xp = B.pack_nchw(dev(x), 1)
    img = B.binary_conv2d_bits(xp, C, W1p, O1, 3, 3, s1, 1, alpha=dev(a1), thr=dev(thr), out_pad=1)
    np.testing.assert_array_equal(host_u64(img), packed_image(h1 > 0, 1))
    got = B.binary_conv2d_packed(img, O1, W2p, O2, 3, 3, 1, 1, alpha=dev(a2))
    assert_f32_close(got.cpu().numpy(), r2f)
    goti = B.binary_conv2d_packed(img, O1, W2p, O2, 3, 3, 1, 1, integer_out=True)
    np.testing.assert_array_equal(goti.cpu().numpy(), r2i)


# ------------------------------------------------------------------ seeded random shapes
def _random_conv_shapes(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        k = int(rng.choice([1, 3, 3, 3, 5, 7]))
        s = int(rng.choice([1, 2]))
        p = int(rng.integers(0, k))
        C = int(rng.choice([1, 3, 31, 64, 65, 100, 128, 200, 256, 300]))
        H, W = int(rng.integers(1, 13)), int(rng.integers(1, 13))
        if H + 2 * p < k or W + 2 * p < k:
            continue
        out.append((int(rng.integers(1, 4)), C, H, W, int(rng.choice([1, 2, 31, 32, 33, 64, 70, 130])), k, s, p))
    return out


@pytest.mark.parametrize("N,C,H,W,O,k,s,p", _random_conv_shapes(2024, 48))
def test_conv_random_shapes(N, C, H, W, O, k, s, p):
    """Seeded random layer shapes across every kernel the dispatcher can pick (1x1 to 7x7, one
    to five channel words, ragged filter and pixel counts): integer output exact, scaled output
    within tolerance, and the packed-image output equal to packing the float one."""
    rng = np.random.default_rng(N + 7 * C + 11 * H + 13 * W + 17 * O + k + s + p)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((O, C, k, k)).astype(np.float32)
    alpha = oracle.alpha_mean_abs(w)
    ri, rf = oracle.binary_conv2d(x, w, s, p, alpha)
    np.testing.assert_array_equal(run_conv(x, w, s, p, integer_out=True), ri)
    assert_f32_close(run_conv(x, w, s, p, alpha=alpha), rf)
    Wp, xp = B.pack_conv_weights(dev(w)), B.pack_nchw(dev(x), p)
    img = B.binary_conv2d_bits(xp, C, Wp, O, k, k, s, p, alpha=dev(alpha), out_pad=1)
    np.testing.assert_array_equal(host_u64(img), packed_image(rf >= 0.0, 1))


@pytest.mark.parametrize("seed", range(24))
def test_fc_random_shapes(seed):
    """Seeded random fully connected layers through the fp32 entry point (pack + GEMM) and the
    packed one, every output kind."""
    rng = np.random.default_rng(900 + seed)
    batch, fin, fout = int(rng.integers(1, 300)), int(rng.integers(1, 3000)), int(rng.integers(1, 400))
    x = rng.standard_normal((batch, fin)).astype(np.float32)
    w = rng.standard_normal((fout, fin)).astype(np.float32)
    alpha = oracle.alpha_mean_abs(w)
    ri, rf = oracle.binary_fc(x, w, alpha)
    Wp = B.binarize_pack(dev(w), 1)
    np.testing.assert_array_equal(B.binary_fc(dev(x), Wp, integer_out=True).cpu().numpy(), ri)
    assert_f32_close(B.binary_fc(dev(x), Wp, alpha=dev(alpha)).cpu().numpy(), rf)
    Xp = B.binarize_pack(dev(x), 1)
    np.testing.assert_array_equal(B.binary_fc_packed(Xp, fin, Wp, mode="i32").cpu().numpy(), ri)
    bits = B.binary_fc_packed(Xp, fin, Wp, alpha=dev(alpha), mode="bits")
    np.testing.assert_array_equal(host_u64(bits), oracle.binarize_pack(rf, 1))


# ------------------------------------------------------------------ 32-bit BINARY_WORD rows
def words32(x, ld_dw=None, fill=0xCDCDCDCD):
    """Rows of 32-bit words straight from the definition (element k = bit k % 32 of dword k / 32,
    numpy.packbits, little bit order), ld_dw dwords apart, spare dwords poisoned."""
    bits = (x >= 0).astype(np.uint8)
    R, K = bits.shape
    Kd = (K + 31) // 32
    padded = np.zeros((R, Kd * 32), dtype=np.uint8)
    padded[:, :K] = bits
    w = np.packbits(padded, axis=1, bitorder="little").view("<u4").reshape(R, Kd)
    out = np.full((R, Kd if ld_dw is None else ld_dw), fill, dtype=np.uint32)
    out[:, :Kd] = w
    return out


@pytest.mark.parametrize("K", [1, 32, 33, 64, 96, 100, 333, 1000, 1024, 2048 + 32, 4096 + 96])
@pytest.mark.parametrize("layout", ["tight", "wide_odd", "wide_even", "offset"])
def test_words32_gemm_and_fc(K, layout):
    """Operands stored as rows of 32-bit words (Sec. 2.2.1, the 32-bit BINARY_WORD flavour): odd
    and even dword counts, odd and even strides with garbage behind the rows, and a base that is
    only 4-byte aligned.  The GEMM must equal the oracle's float layer on the unpacked signs."""
    rng = np.random.default_rng(K * 7 + len(layout))
    M, N = 37, 70
    a = rng.standard_normal((M, K)).astype(np.float32)
    b = rng.standard_normal((N, K)).astype(np.float32)
    alpha = oracle.alpha_mean_abs(b)
    ri, rf = oracle.binary_fc(a, b, alpha)
    Kd = (K + 31) // 32
    ld = {"tight": Kd, "wide_odd": Kd + 1 + (Kd & 1), "wide_even": Kd + 2 - (Kd & 1), "offset": Kd + 1}[layout]
    A32, B32 = words32(a, ld), words32(b, ld)

    def put(w):
        if layout != "offset":
            return dev(w.view(np.int32))
        flat = torch.empty(w.size + 1, dtype=torch.int32, device="cuda")   # rows start one dword in
        flat[1:] = dev(w.view(np.int32)).flatten()
        return flat[1:].view(w.shape)

    Ad, Bd = put(A32), put(B32)
    got = B.xnor_gemm_w32(Ad, Bd, K).cpu().numpy()
    np.testing.assert_array_equal(got, ri)
    # widened rows feed every call that takes packed operands
    Aw, Bw = B.widen_words32(Ad, K), B.widen_words32(Bd, K)
    np.testing.assert_array_equal(host_u64(Aw), oracle.binarize_pack(a, 1))
    np.testing.assert_array_equal(B.xnor_gemm(Aw, Bw, K).cpu().numpy(), ri)
    f = B.binary_fc_packed(Aw, K, Bw, alpha=dev(alpha), mode="f32").cpu().numpy()
    assert_f32_close(f, rf)
    bits = B.binary_fc_packed(Aw, K, Bw, alpha=dev(alpha), mode="bits")
    np.testing.assert_array_equal(host_u64(bits), oracle.binarize_pack(rf, 1))
    if Kd % 2 == 0 and layout in ("tight", "wide_even"):
        # whole 64-bit words already: the same memory read in place through the 64-bit entry point
        as64 = Ad.view(torch.int64) if layout == "tight" else None
        if as64 is not None:
            np.testing.assert_array_equal(B.xnor_gemm(as64, Bd.view(torch.int64), K).cpu().numpy(), ri)


# ------------------------------------------------------------------ 64 x 64 per wave FP4 kernel (LDS-staged operands)
def test_gemm_fp4_chip_filling_problem_exact():
    """A GEMM large enough to keep every SIMD busy with several waves for many segments
    (4096 x 4096 x 4096: 4096 tiles of 64 x 64, 8 segments each, no K split), repeated so that
    the LDS queues stay long: every element against the popcount engine (an independent kernel),
    96 sampled rows against the oracle.  A wave's staging area is overwritten by the next
    segment's loads; the kernel has to wait for its LDS reads to complete before it requests them,
    and under this load a missing wait shows as a few wrong counts."""
    rng = np.random.default_rng(4096)
    M = N = K = 4096
    A = rng.integers(0, 2 ** 63, size=(M, K // 64), dtype=np.int64) * 2 + rng.integers(0, 2, size=(M, K // 64), dtype=np.int64)
    Bm = rng.integers(0, 2 ** 63, size=(N, K // 64), dtype=np.int64) * 2 + rng.integers(0, 2, size=(N, K // 64), dtype=np.int64)
    Ad, Bd = dev(A), dev(Bm)
    with tuned(k7=1):
        ref = B.xnor_gemm(Ad, Bd, K)
        assert "gemm_kernel" in B.last_kernel()
    # tile order: automatic bands, ragged bands, none; tile: 64 x 64 per wave (the automatic
    # choice at this size) and 128 x 64
    for band, tall in ((0, 0), (3, 0), (1000, 0), (0, 2), (3, 2)):
        with tuned(k12=band, k13=tall):
            for rep in range(6):
                got = B.xnor_gemm(Ad, Bd, K)
                assert "gemm_fp4_kernel<%d,2,1" % (4 if tall else 2) in B.last_kernel() and "K split 1," in B.last_kernel()
                assert torch.equal(got, ref), "band %d tall %d repetition %d: %d elements differ" % (
                    band, tall, rep, int((got != ref).sum()))
    rows = np.sort(rng.choice(M, size=96, replace=False))
    want = oracle.xnor_gemm(A[rows].view(np.uint64), Bm.view(np.uint64), K)
    np.testing.assert_array_equal(ref[torch.from_numpy(rows).cuda()].cpu().numpy(), want)


def test_gemm_fp4_tall_tile():
    """The same kernel with 128 x 64 of C per wave (no K split; the automatic choice only for
    chip-filling products), forced on small and ragged problems: fewer rows than a tile, ragged
    tiles in M and N, rows that end inside a 64-byte segment, strides wider than the rows with
    garbage behind them, int32, xnor-count and scaled fp32 results."""
    rng = np.random.default_rng(1313)
    with tuned(k7=5, k10=1, k13=2):
        for (M, N, K) in [(1, 1, 1), (37, 70, 5000), (127, 64, 1024), (128, 129, 3072 + 64), (129, 64, 63),
                          (65, 33, 1025), (130, 200, 2048 + 128), (700, 801, 1100), (256, 512, 9216),
                          (300, 190, 64 * 7), (33, 65, 64 * 9), (513, 128, 64 * 10), (5, 300, 64 * 11),
                          (70, 70, 64 * 12 + 1), (257, 64, 64 * 13), (64, 65, 64 * 14), (191, 66, 64 * 15)]:
            a = rng.standard_normal((M, K)).astype(np.float32)
            b = rng.standard_normal((N, K)).astype(np.float32)
            A, Bm = oracle.binarize_pack(a, 1), oracle.binarize_pack(b, 1)
            ld = (A.shape[1] + 1) // 2 * 2 + 2 * (K % 3)            # even, sometimes wider than the row
            Ad = np.full((M, ld), POISON, dtype=np.uint64); Ad[:, :A.shape[1]] = A
            Bd = np.full((N, ld), POISON, dtype=np.uint64); Bd[:, :A.shape[1]] = Bm
            want = oracle.xnor_gemm(A, Bm, K)
            got = B.xnor_gemm(dev(Ad.view(np.int64)), dev(Bd.view(np.int64)), K).cpu().numpy()
            assert "gemm_fp4_kernel<4,2,1" in B.last_kernel()
            np.testing.assert_array_equal(got, want)
            cnt = B.xnor_gemm(dev(Ad.view(np.int64)), dev(Bd.view(np.int64)), K, count=True).cpu().numpy()
            np.testing.assert_array_equal(2 * cnt - K, want)
        for (batch, fin, fout) in [(19, 2500, 75), (200, 4096, 130), (256, 1100, 300)]:
            x = rng.standard_normal((batch, fin)).astype(np.float32)
            w = rng.uniform(-1, 1, (fout, fin)).astype(np.float32)
            alpha = rng.standard_normal(fout).astype(np.float32)
            alpha[::3] = 0.0
            ri, rf = oracle.binary_fc(x, w, alpha)
            Wp = B.binarize_pack(dev(w), 1)
            if Wp.shape[1] % 2:                                      # 16-byte rows for the matrix-core kernels
                Wp = torch.cat([Wp, torch.zeros_like(Wp[:, :1])], dim=1).contiguous()
            np.testing.assert_array_equal(B.binary_fc(dev(x), Wp, integer_out=True).cpu().numpy(), ri)
            assert "gemm_fp4_kernel<4,2,1" in B.last_kernel()
            assert_f32_close(B.binary_fc(dev(x), Wp, alpha=dev(alpha)).cpu().numpy(), rf)
            assert "gemm_fp4_kernel<4,2,1" in B.last_kernel()


@pytest.mark.parametrize("split,partials", [(0, 0), (1, 0), (2, 0), (3, 0), (5, 0), (7, 0), (8, 0), (8, 2), (3, 2)])
def test_gemm_fp4_lds_staged_kernel(split, partials):
    """The matrix-core GEMM kernel with 64 x 64 of C per wave, operands staged through LDS by the
    load unit and K split over the waves of a workgroup, forced through the tuning hook whatever
    the size: ragged tiles in M and N, rows that end inside a 64-byte segment (every residue of
    the word count mod 8), row strides wider than the rows with garbage behind them, every K
    split, partial tiles crossing LDS as fp16 pairs (where a wave's sums stay exact in them) and as
    fp32 (partials = 2 forces it), every output kind, and the plane form with 1 and 2 bit planes."""
    rng = np.random.default_rng(300 + split)
    with tuned(k7=5, k10=split, k11=partials):
        for (M, N, K) in [(1, 1, 1), (37, 70, 5000), (8, 64, 1024), (100, 129, 3072 + 64), (64, 64, 63),
                          (65, 33, 1025), (130, 200, 2048 + 128), (700, 801, 1100), (256, 512, 9216),
                          (31, 190, 64 * 7), (33, 65, 64 * 9), (64, 128, 64 * 10), (5, 300, 64 * 11),
                          (70, 70, 64 * 12 + 1), (129, 64, 64 * 13), (64, 65, 64 * 14), (66, 66, 64 * 15)]:
            a = rng.standard_normal((M, K)).astype(np.float32)
            b = rng.standard_normal((N, K)).astype(np.float32)
            A, Bm = oracle.binarize_pack(a, 1), oracle.binarize_pack(b, 1)
            ld = (A.shape[1] + 1) // 2 * 2 + 2 * (K % 3)            # even, sometimes wider than the row
            Ad = np.full((M, ld), POISON, dtype=np.uint64); Ad[:, :A.shape[1]] = A
            Bd = np.full((N, ld), POISON, dtype=np.uint64); Bd[:, :A.shape[1]] = Bm
            want = oracle.xnor_gemm(A, Bm, K)
            got = B.xnor_gemm(dev(Ad.view(np.int64)), dev(Bd.view(np.int64)), K).cpu().numpy()
            assert "gemm_fp4_kernel" in B.last_kernel()
            np.testing.assert_array_equal(got, want)
            cnt = B.xnor_gemm(dev(Ad.view(np.int64)), dev(Bd.view(np.int64)), K, count=True).cpu().numpy()
            np.testing.assert_array_equal(2 * cnt - K, want)
        for (batch, fin, fout) in [(19, 2500, 75), (70, 4096, 130), (256, 1100, 300)]:
            x = rng.standard_normal((batch, fin)).astype(np.float32)
            w = rng.uniform(-1, 1, (fout, fin)).astype(np.float32)
            alpha = rng.standard_normal(fout).astype(np.float32)
            alpha[::3] = 0.0
            ri, rf = oracle.binary_fc(x, w, alpha)
            Wp = B.binarize_pack(dev(w), 1)
            if Wp.shape[1] % 2:                                      # 16-byte rows for the matrix-core kernels
                Wp = torch.cat([Wp, torch.zeros_like(Wp[:, :1])], dim=1).contiguous()
            np.testing.assert_array_equal(B.binary_fc(dev(x), Wp, integer_out=True).cpu().numpy(), ri)
            assert "gemm_fp4_kernel" in B.last_kernel()
            assert_f32_close(B.binary_fc(dev(x), Wp, alpha=dev(alpha)).cpu().numpy(), rf)
            Xp = B.binarize_pack(dev(x), 1)
            if Xp.shape[1] % 2:
                Xp = torch.cat([Xp, torch.zeros_like(Xp[:, :1])], dim=1).contiguous()
            thr = (rng.standard_normal(fout) * np.sqrt(fin)).astype(np.float32)
            out = dev(np.full((batch, (fout + 63) // 64 + 1), -1, dtype=np.int64))
            B.binary_fc_packed(Xp, fin, Wp, alpha=dev(alpha), mode="bits", thr=dev(thr), out=out)
            assert "gemm_fp4_kernel" in B.last_kernel()
            want = np.where(rf >= thr[None, :], 1.0, -1.0).astype(np.float32)
            got = host_u64(out)
            np.testing.assert_array_equal(got[:, :-1], oracle.binarize_pack(want, 1))
            assert (got[:, -1] == np.uint64(0xFFFFFFFFFFFFFFFF)).all()
        for bits in (1, 2):
            for (M, N, K) in [(21, 70, 2200), (1, 1, 1), (33, 65, 1024), (100, 130, 4096 + 200), (256, 256, 64 * 9)]:
                a = rng.uniform(0, 1, (M, K)).astype(np.float32)
                a[rng.random(a.shape) < 0.05] = 0.5
                wq = rng.standard_normal((N, K)).astype(np.float32)
                Sg, fg = B.quant_gemm(dev(a), dev(wq), bits)
                # (the sign-packed weight rows of the workspace are ceil(K/64) words: an odd count is
                # not 16-byte aligned and goes to the xor/popcount kernel)
                assert "gemm_fp4_kernel" in B.last_kernel() or ((K + 63) // 64) % 2 == 1
                rS, r64, r32 = oracle.quant_gemm(a, wq, bits)
                np.testing.assert_array_equal(Sg.cpu().numpy(), rS)
                assert_f32_close(fg.cpu().numpy(), r32)


FP4_CONV_CASES = [
    # N, C, H, W, O, k, s, p   (an even number of channel words: 16-byte pieces never straddle two taps)
    (2, 128, 9, 9, 33, 5, 2, 2),
    (3, 100, 9, 11, 70, 3, 1, 1),
    (1, 256, 14, 14, 19, 3, 1, 2),
    (2, 500, 5, 5, 70, 1, 1, 0),
    (1, 1024, 4, 4, 17, 3, 1, 1),
    (3, 200, 12, 12, 64, 5, 1, 0),
    (2, 128, 28, 28, 128, 3, 2, 1),
    (2, 66, 9, 8, 3, 7, 1, 3),
    (5, 256, 14, 14, 256, 3, 1, 1),
    (1, 70, 1, 1, 1, 1, 1, 0),
]


@pytest.mark.parametrize("split", [0, 1, 2, 3, 8])
def test_conv_fp4_lds_staged_kernel(split):
    """The convolution form of the 64 x 64 per wave matrix-core kernel (im2col rows gathered piece
    by piece from the packed image by the load unit), forced through the tuning hook: ragged
    filter and pixel tiles, pixel tiles that straddle images, strides, halos, K that ends inside
    a 64-byte segment, every K split, both output kinds."""
    for (N, C, H, W, O, k, s, p) in FP4_CONV_CASES:
        rng = np.random.default_rng(N + 10 * C + 100 * H + 1000 * O + k + s + p + split)
        x = rng.standard_normal((N, C, H, W)).astype(np.float32)
        x[rng.random(x.shape) < 0.05] = 0.0
        w = rng.standard_normal((O, C, k, k)).astype(np.float32)
        alpha = rng.standard_normal(O).astype(np.float32)
        ri, rf = oracle.binary_conv2d(x, w, s, p, alpha)
        with tuned(k5=6, k10=split):
            got_i = run_conv(x, w, s, p, integer_out=True)
            assert "gemm_fp4_kernel" in B.last_kernel() and "conv" in B.last_kernel(), B.last_kernel()
            np.testing.assert_array_equal(got_i, ri)
            assert_f32_close(run_conv(x, w, s, p, alpha=alpha), rf)
            np.testing.assert_array_equal(run_conv(x, w, s, p), ri.astype(np.float32))
