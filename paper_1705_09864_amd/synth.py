"""Seeded synthetic inputs for the binary-layer hot path.

This module only draws random numbers (numpy Philox streams) in the shapes and value
distributions of the benchmark configurations; it contains none of the method's
arithmetic (no sign, packing, popcount, quantisation or scaling) and is the one module
shared by the GPU tests, the benchmark and the CPU-oracle tests.
"""
import numpy as np

SEED_BASE = 1705098640  # arXiv number of the paper, times ten; config index is added


def _rng(config, stream):
    return np.random.Generator(np.random.Philox(key=SEED_BASE + int(config), counter=[0, 0, 0, int(stream)]))


def normal(shape, config, stream):
    return _rng(config, stream).standard_normal(size=shape, dtype=np.float32)


def uniform(shape, lo, hi, config, stream):
    r = _rng(config, stream).random(size=shape, dtype=np.float32)
    return (np.float32(lo) + (np.float32(hi) - np.float32(lo)) * r).astype(np.float32)


def relu_like(shape, config, stream):
    """|N(0,1)| - 0.5: about 62 % of the entries are non-negative (skewed sign balance)."""
    return (np.abs(normal(shape, config, stream)) - np.float32(0.5)).astype(np.float32)


# ---- the five benchmark configurations (shapes only; small=True gives a reduced case
# ---- with the same structure, for tests the oracle must finish quickly) ----

def config1():
    """Binary FC GEMM: A [64,512] N(0,1); W [512,256] N(0,1) stored K x N."""
    return {"a": normal((64, 512), 1, 0), "w_kn": normal((512, 256), 1, 1)}


def config2(small=False):
    """ResNet-18 stage conv 3x3 s1 p1: x [16,64,56,56] N(0,1); w [64,64,3,3] N(0,1)."""
    n, c, h, o = (2, 64, 14, 64) if small else (16, 64, 56, 64)
    return {"x": normal((n, c, h, h), 2, 0), "w": normal((o, c, 3, 3), 2, 1), "stride": 1, "pad": 1}


def config3(small=False):
    """AlexNet classifier: x [256,9216] N(0,1); W1 [4096,9216], W2 [4096,4096] uniform(-1,1)."""
    b, f0, f1, f2 = (32, 1152, 256, 192) if small else (256, 9216, 4096, 4096)
    return {"x": normal((b, f0), 3, 0), "w1": uniform((f1, f0), -1.0, 1.0, 3, 1),
            "w2": uniform((f2, f1), -1.0, 1.0, 3, 2)}


def config4(small=False, stride=1):
    """Deep conv stage: x [64,256,14,14] = |N(0,1)|-0.5; w [256,256,3,3] N(0,1); s1 or s2, p1."""
    n, c, h, o = (2, 256, 14, 32) if small else (64, 256, 14, 256)
    return {"x": relu_like((n, c, h, h), 4, 0), "w": normal((o, c, 3, 3), 4, 1), "stride": stride,
            "pad": 1}


def config5(small=False):
    """DoReFa GEMM: a [1024,4096] uniform[0,1] (2-bit); w [1024,4096] N(0,1) (sign)."""
    m, n, k = (96, 80, 1000) if small else (1024, 1024, 4096)
    return {"a": uniform((m, k), 0.0, 1.0, 5, 0), "w": normal((n, k), 5, 1), "bits_a": 2}
