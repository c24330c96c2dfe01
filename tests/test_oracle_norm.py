"""Pins for the oracle's RMS normalisation with the inverse scale folded in (AWQ Sec. 4.2 kernel
fusion of the normalisation; Sec. 3.2, Eq. 4: the diag(s)^-1 factor belongs to the producer of x)."""
import numpy as np

import oracle


def test_constant_rows_have_the_closed_form():
    K = 256
    gamma = np.full(K, 0.5, np.float16)
    s = np.full(K, 4.0, np.float32)
    for c in (3.0, -0.25):
        x = np.full((2, K), c, np.float16)
        y = oracle.rmsnorm_inv_scale(x, gamma, s, eps=0.0)
        assert np.all(y == np.float16(np.sign(c) * 0.5 / 4.0))
        y = oracle.rmsnorm_inv_scale(x, gamma, s, eps=c * c * 3)       # sqrt(c^2 + 3 c^2) = 2 |c|
        assert np.all(y == np.float16(np.sign(c) * 0.5 / 4.0 / 2))


def test_unit_rms_scale_invariance_and_per_channel_factors():
    g = np.random.default_rng(80)
    M, K = 5, 1408
    x = g.standard_normal((M, K)).astype(np.float16)
    ones = np.ones(K, np.float16)
    y = oracle.rmsnorm_inv_scale(x, ones, None, eps=0.0).astype(np.float64)
    assert np.allclose((y * y).mean(axis=1), 1.0, atol=2e-3)
    assert np.all(np.sign(y) == np.sign(x.astype(np.float64)))
    # exact powers of two commute with every rounding
    y4 = oracle.rmsnorm_inv_scale((x.astype(np.float32) * 4).astype(np.float16), ones, None, eps=0.0)
    assert np.array_equal(y4.view(np.uint16), oracle.rmsnorm_inv_scale(x, ones, None, eps=0.0).view(np.uint16))
    gamma = (2.0 ** g.integers(-2, 3, size=K)).astype(np.float16)
    s = (2.0 ** g.integers(-1, 3, size=K)).astype(np.float32)
    a = oracle.rmsnorm_inv_scale(x, gamma, s, eps=1e-5)
    b = oracle.rmsnorm_inv_scale(x, (gamma.astype(np.float32) / s).astype(np.float16), None, eps=1e-5)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    # against numpy, all different sizes, general factors
    gamma = g.uniform(0.5, 1.5, size=K).astype(np.float16)
    s = g.uniform(0.5, 4.0, size=K).astype(np.float32)
    want = (x.astype(np.float64) / np.sqrt((x.astype(np.float64) ** 2).mean(axis=1, keepdims=True) + 1e-5)
            * gamma.astype(np.float64) / s.astype(np.float64))
    got = oracle.rmsnorm_inv_scale(x, gamma, s, eps=1e-5).astype(np.float64)
    assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -11 + 1e-8)


def test_silu_mul_special_values():
    g = np.array([[0.0, 20.0, -20.0, 1.0, -1.0]], np.float16)
    u = np.array([[3.0, 2.0, 2.0, 1.0, 1.0]], np.float16)
    y = oracle.silu_mul(g, u).astype(np.float64)[0]
    assert y[0] == 0.0 and abs(y[1] - 40.0) < 0.05 and abs(y[2]) < 1e-6
    assert abs(y[3] - 0.7310585786) < 1e-3 and abs(y[4] + 0.2689414214) < 1e-3     # x * sigmoid(x)
    assert abs(y[3] + y[4] - 0.4621171573) < 1e-3                                      # silu(x) + silu(-x) = x tanh(x/2)


def test_scale_columns_rounds_once():
    x = np.array([[1.0, 3.0, 0.333251953125, 65504.0, 6e-8]], np.float16)
    w = np.array([0.5, 0.333251953125, 3.0, 0.5, 0.5], np.float16)
    y = oracle.scale_columns(x, w)[0]
    assert y[0] == np.float16(0.5) and y[3] == np.float16(32752.0)
    assert y[1] == y[2]                                         # commutative, one rounding
    assert abs(float(y[1]) - 0.999755859375) <= 2.0 ** -11      # 3 * fp16(1/3) rounded to fp16
    assert float(y[4]) in (0.0, 5.960464477539063e-08)         # subnormal result stays representable
