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
