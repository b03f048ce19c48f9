"""Pins for the oracle's alpha helper, Eq. 1 quantiser and k-bit GEMM (CPU only)."""
import os

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(5)


def test_alpha_closed_forms():
    w = RNG.uniform(-1, 1, (8, 20000)).astype(np.float32)
    a = oracle.alpha_mean_abs(w)
    np.testing.assert_allclose(a, np.abs(w.astype(np.float64)).mean(1), rtol=1e-7)
    assert np.abs(a - 0.5).max() < 0.01                      # E|U(-1,1)| = 1/2
    g = RNG.standard_normal((8, 20000)).astype(np.float32)
    assert np.abs(oracle.alpha_mean_abs(g) - np.sqrt(2 / np.pi)).max() < 0.02   # E|N(0,1)|
    # 4-D weights: mean over C*KH*KW per output channel
    w4 = RNG.standard_normal((3, 4, 3, 3)).astype(np.float32)
    np.testing.assert_allclose(oracle.alpha_mean_abs(w4),
                               np.abs(w4.astype(np.float64)).reshape(3, -1).mean(1), rtol=1e-7)
    assert oracle.alpha_mean_abs(np.array([[1.0, -3.0, 2.0]], dtype=np.float32))[0] == 2.0


def test_quantize_golden_k2(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "eq1_k2_levels.txt"))
            if l.strip() and not l.startswith("#")]
    x = np.array([float(r[0]) for r in rows], dtype=np.float32)
    q, v = oracle.quantize(x, 2)
    assert q.tolist() == [int(r[1]) for r in rows]
    np.testing.assert_allclose(v, q / 3.0, rtol=0, atol=0)


def test_quantize_properties():
    x = RNG.uniform(0, 1, 5000).astype(np.float32)
    for k in (1, 2, 3, 4, 8):
        L = 2 ** k - 1
        q, v = oracle.quantize(x, k)
        assert q.min() >= 0 and q.max() <= L
        assert np.abs(v - x).max() <= 0.5 / L + 1e-6            # nearest level
        q2, _ = oracle.quantize(v.astype(np.float32), k)        # idempotent
        np.testing.assert_array_equal(q, q2)
        xs = np.sort(x)
        assert (np.diff(oracle.quantize(xs, k)[0]) >= 0).all()  # monotone
    # k = 2 levels are {0, 1/3, 2/3, 1}
    _, v = oracle.quantize(x, 2)
    assert set(np.round(v * 3).astype(int).tolist()) == {0, 1, 2, 3}
    # ties round away from zero: fl(1/6)*3 = 0.5 -> 1, fl(5/6)*3 = 2.5 -> 3, 0.5*3 = 1.5 -> 2
    t = np.array([1 / 6, 5 / 6, 0.5], dtype=np.float32)
    assert (np.float32(3.0) * t).tolist() == [0.5, 2.5, 1.5]
    assert oracle.quantize(t, 2)[0].tolist() == [1, 3, 2]


@pytest.mark.parametrize("bits", [1, 2, 3, 8])
def test_quant_gemm_brute_force(bits):
    M, N, K = 5, 7, 130
    a = RNG.uniform(0, 1, (M, K)).astype(np.float32)
    w = RNG.standard_normal((N, K)).astype(np.float32)
    S, o64, o32 = oracle.quant_gemm(a, w, bits)
    L = 2 ** bits - 1
    q = np.floor(np.float32(L) * a + np.float32(0.5)).astype(np.int64)   # half-up == half-away for t >= 0
    sw = np.where(w >= 0, 1, -1).astype(np.int64)
    Sref = q @ sw.T
    np.testing.assert_array_equal(S, Sref)
    np.testing.assert_allclose(o64, Sref / L, rtol=0, atol=1e-9)
    np.testing.assert_allclose(o32, Sref / L, rtol=1e-6, atol=0)
    # bit-plane identity: S = 2 * sum_p 2^p pc(b_p & wb) - sum_p 2^p pc(b_p)
    wb = (w >= 0).astype(np.int64)
    acc = np.zeros((M, N), dtype=np.int64)
    for p in range(bits):
        bp = (q >> p) & 1
        acc += (1 << p) * (2 * (bp @ wb.T) - bp.sum(1, keepdims=True))
    np.testing.assert_array_equal(acc, Sref)


def test_quant_gemm_k1_reduces_to_and_count():
    a = RNG.uniform(0, 1, (3, 64)).astype(np.float32)
    w = RNG.standard_normal((4, 64)).astype(np.float32)
    S, _, _ = oracle.quant_gemm(a, w, 1)
    b = (a >= 0.5).astype(np.int64)                 # round(x) for k = 1
    b[a == 0.5] = 1
    wb = (w >= 0).astype(np.int64)
    np.testing.assert_array_equal(S, 2 * (b @ wb.T) - b.sum(1, keepdims=True))


# ------------------------------------------------------------------ k-bit weights
def test_kbit_weights_one_bit_is_the_sign_layer():
    """bits_w = 1 through the k-bit route (u = (w+1)/2, one level, threshold u = 1/2) is the
    sign layer for weights in [-1, 1] that are not within rounding of zero."""
    a = RNG.uniform(0, 1, (6, 150)).astype(np.float32)
    w = RNG.uniform(-1, 1, (9, 150)).astype(np.float32)
    w[np.abs(w) < 1e-3] = 0.25
    w[0, :5] = [1.0, -1.0, 0.0, 0.5, -0.5]
    for bits in (1, 2, 4):
        S1, f1, o1 = oracle.quant_gemm(a, w, bits)
        M, N, K = 6, 9, 150
        Sk = np.empty((M, N), dtype=np.int32); fk = np.empty((M, N)); ok = np.empty((M, N), dtype=np.float32)
        from oracle import lib, _ptr, _i64, _int
        lib().orc_quant_gemm_kw(_ptr(a), _i64(K), _int(bits), _ptr(w), _i64(K), _int(1), _i64(M), _i64(N),
                                _i64(K), _ptr(Sk), _ptr(fk), _ptr(ok), _i64(N))
        np.testing.assert_array_equal(Sk, S1)
        np.testing.assert_array_equal(ok, o1)
        np.testing.assert_allclose(fk, f1, rtol=1e-12)


def test_kbit_weights_closed_forms():
    K = 77
    ones = np.ones((2, K), dtype=np.float32)
    for ba, bw in [(1, 2), (2, 2), (3, 4), (8, 8)]:
        La, Lw = 2 ** ba - 1, 2 ** bw - 1
        S, f64, f32 = oracle.quant_gemm(ones, ones, ba, bw)           # 1 * 1 summed K times
        assert (S == K * La * Lw).all() and (f32 == K).all() and np.allclose(f64, K)
        S, _, f32 = oracle.quant_gemm(ones, -ones, ba, bw)
        assert (S == -K * La * Lw).all() and (f32 == -K).all()
        S, _, _ = oracle.quant_gemm(0 * ones, ones, ba, bw)
        assert (S == 0).all()
        # w = 0 -> u = 1/2 -> level round(Lw / 2) = (Lw + 1) / 2 (tie away) -> w_q = 1 / Lw
        S, f64, _ = oracle.quant_gemm(ones, 0 * ones, ba, bw)
        assert (S == K * La).all() and np.allclose(f64, K / Lw)
    # values outside [-1, 1] clamp
    S, _, _ = oracle.quant_gemm(ones, 5 * ones, 2, 2)
    assert (S == K * 9).all()


def test_kbit_weights_brute_force_in_exact_arithmetic():
    """Inputs on a dyadic grid, where every fp32 step is exact: Eq. 1 and the affine pair
    evaluated with fractions, ties away from zero."""
    from fractions import Fraction as F
    import math

    def rnd(v):  # half away from zero, v >= 0
        return math.floor(v + F(1, 2))

    M, N, K = 3, 4, 19
    a = RNG.integers(0, 17, (M, K)) / 16.0
    w = RNG.integers(-8, 9, (N, K)) / 8.0
    for ba, bw in [(2, 2), (1, 3), (4, 2)]:
        La, Lw = 2 ** ba - 1, 2 ** bw - 1
        S, f64, f32 = oracle.quant_gemm(a.astype(np.float32), w.astype(np.float32), ba, bw)
        for m in range(M):
            for n in range(N):
                acc = 0
                for k in range(K):
                    qa = rnd(La * F(a[m, k]))
                    qw = rnd(Lw * (F(w[n, k]) + 1) / 2)
                    acc += qa * (2 * qw - Lw)
                assert S[m, n] == acc
                assert abs(f64[m, n] - acc / (La * Lw)) < 1e-12
                assert f32[m, n] == np.float32(acc) / np.float32(La * Lw)
