"""Pins of the oracle's residual add + RMSNorm (the operator the per-token quantiser is fused behind, Sec. 6.1; the norm
is LLaMA's): closed forms, invariants and the rounding of the addition, none of which retype its formula."""
import numpy as np

import oracle


def _f16(a):
    return np.asarray(a, dtype=np.float16)


def test_constant_rows_have_closed_forms():
    K = 96
    g = _f16(np.linspace(0.5, 2.0, K))
    # eps = 0: a constant row c normalises to sign(c), whatever |c|
    for c in (3.0, -0.25, 1024.0):
        r, y64, y = oracle.add_rmsnorm(_f16(np.full((1, K), c)), None, g, 0.0)
        assert np.array_equal(r, _f16(np.full((1, K), c)))
        assert np.allclose(y64, np.sign(c) * g.astype(np.float64), rtol=1e-15, atol=0)
    # c = 2, eps = 5: 2 / sqrt(4 + 5) = 2/3
    _, y64, _ = oracle.add_rmsnorm(_f16(np.full((2, K), 2.0)), None, g, 5.0)
    assert np.allclose(y64, (2.0 / 3.0) * g.astype(np.float64), rtol=1e-15, atol=0)


def test_single_nonzero_element_carries_the_whole_norm():
    K = 64
    x = np.zeros((1, K), np.float16)
    x[0, 5] = -3.0
    g = _f16(np.ones(K) * 1.5)
    _, y64, _ = oracle.add_rmsnorm(x, None, g, 0.0)
    want = np.zeros(K)
    want[5] = -np.sqrt(K) * 1.5      # r / sqrt(r^2 / K) = sign(r) sqrt(K)
    assert np.allclose(y64[0], want, rtol=1e-15, atol=0)


def test_invariants_on_random_rows():
    rng = np.random.default_rng(5)
    M, K = 4, 160
    x = _f16(rng.standard_normal((M, K)))
    g = _f16(rng.uniform(0.5, 1.5, K))
    _, y64, y = oracle.add_rmsnorm(x, None, g, 0.0)
    # eps = 0: the normalised row has mean square 1
    assert np.allclose(np.mean((y64 / g.astype(np.float64)) ** 2, axis=1), 1.0, rtol=1e-12)
    # doubling the row (exact in fp16) changes nothing
    _, y64_2, _ = oracle.add_rmsnorm(_f16(x * np.float16(2)), None, g, 0.0)
    assert np.allclose(y64_2, y64, rtol=1e-15, atol=0)
    # a larger eps shrinks every element, and the sign follows r * g
    _, y64_e, _ = oracle.add_rmsnorm(x, None, g, 0.5)
    assert np.all(np.abs(y64_e) <= np.abs(y64)) and np.all(np.sign(y64_e) == np.sign(x.astype(np.float64)))
    # the fp16 output is the fp64 value rounded once, to nearest even (numpy's conversion as the independent routine)
    assert np.array_equal(y.view(np.uint16), y64.astype(np.float16).view(np.uint16))


def test_residual_addition_rounds_once_in_fp32_and_once_to_fp16():
    K = 32
    x = np.zeros((1, K), np.float16)
    res = np.zeros((1, K), np.float16)
    # fp16 spacing is 2 at 2048: 2049 and 2051 are ties, which go to the even neighbours 2048 and 2052
    res[0, :4] = [2048, 2048, 2048, -2048]
    x[0, :4] = [1, 3, 2, -1]
    # far apart: 1024 + 2^-14 is 1024 in fp32 already (and stays 1024 in fp16)
    res[0, 4], x[0, 4] = 1024, 2.0 ** -14
    # cancels exactly
    res[0, 5], x[0, 5] = 0.1, -0.1
    r, _, _ = oracle.add_rmsnorm(x, res, _f16(np.ones(K)), 1e-5)
    assert list(r[0, :6].astype(np.float64)) == [2048.0, 2052.0, 2050.0, -2048.0, 1024.0, 0.0]
    # without a residual r is x itself, bit for bit
    r2, _, _ = oracle.add_rmsnorm(x, None, _f16(np.ones(K)), 1e-5)
    assert np.array_equal(r2.view(np.uint16), x.view(np.uint16))
