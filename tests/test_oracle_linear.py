"""Pins for the oracle's dequantize + matmul (AWQ Sec. 4.2) and for the
equivalent transform of Sec. 3.2 (Eq. 2 / Eq. 4)."""
import numpy as np

import oracle


def test_matmul_against_brute_force_python_floats():
    g = np.random.default_rng(20)
    for M, N, K in [(1, 16, 128), (3, 32, 256), (2, 16, 384)]:
        x = g.standard_normal((M, K)).astype(np.float16)
        Wdq = g.standard_normal((N, K)).astype(np.float32)
        y = oracle.matmul(x, Wdq)
        for m in range(M):
            for n in range(N):
                acc = 0.0
                for k in range(K):
                    acc += float(x[m, k]) * float(Wdq[n, k])
                assert abs(y[m, n] - acc) <= 1e-12 * max(1.0, abs(acc))


def test_matmul_against_numpy_float64_and_fp32_variant():
    g = np.random.default_rng(21)
    M, N, K = 5, 48, 1408                # all different: a swapped index changes the shape
    x = g.standard_normal((M, K)).astype(np.float16)
    Wdq = (g.standard_normal((N, K)) * 0.05).astype(np.float32)
    want = x.astype(np.float64) @ Wdq.astype(np.float64).T
    y = oracle.matmul(x, Wdq)
    assert y.shape == (M, N)
    assert np.allclose(y, want, rtol=0, atol=1e-11)
    y32 = oracle.matmul(x, Wdq, acc32=True)
    assert np.abs(y32 - want).max() < 1e-4 * np.abs(want).max()


def test_dequant_is_code_minus_zero_times_step():
    """One-hot constructions: a single code, a single zero point, a single step."""
    N, K = 16, 256
    codes = np.zeros((N, K), np.uint8)
    scales = np.ones((N, 2), np.float16)
    zeros = np.zeros((N, 2), np.uint8)
    codes[3, 130] = 9
    scales[3, 1] = 0.5
    zeros[7, 0] = 4
    scales[7, 0] = 2.0
    Wdq = oracle.dequant(codes, scales, zeros)
    want = np.zeros((N, K), np.float32)
    want[3, 130] = 4.5
    want[7, :128] = -8.0
    assert np.array_equal(Wdq, want)


def test_equivalent_transform_is_exact_without_quantization():
    """Eq. 4: (W diag(s)) (diag(s)^-1 x) == W x in exact arithmetic."""
    g = np.random.default_rng(22)
    M, N, K = 4, 32, 512
    W = (g.standard_normal((N, K)) * 0.02)
    x = g.standard_normal((M, K))
    s = g.uniform(0.25, 6.0, size=K)
    lhs = (x / s[None, :]) @ (W * s[None, :]).T
    rhs = x @ W.T
    assert np.allclose(lhs, rhs, rtol=0, atol=1e-13)


def test_scaled_quantized_layer_approximates_the_fp16_layer_better_on_outliers():
    """Sec. 3.2: protecting the channels with large activations lowers the
    output error of the quantized layer.  End to end through every oracle
    function: act_scale -> apply_inv_scale -> quantize -> pack -> unpack ->
    dequant -> matmul, compared with plain RTN (s = 1) on the same inputs."""
    g = np.random.default_rng(23)
    N, K, T, M = 256, 1024, 64, 16
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float16)
    out = g.choice(K, size=10, replace=False)
    X = g.standard_normal((T, K)).astype(np.float32)
    X[:, out] *= 20
    x = g.standard_normal((M, K)).astype(np.float32)
    x[:, out] *= 20
    X, x = X.astype(np.float16), x.astype(np.float16)
    y_fp = x.astype(np.float64) @ W.astype(np.float64).T

    s = oracle.act_scale(X, alpha=0.5).astype(np.float32)
    assert s.shape == (K,) and np.all(s[out] > 3.0) and np.all(np.delete(s, out) < 1.2)
    xs = oracle.apply_inv_scale(x, s)
    c, sc, z = oracle.quantize(W, s)
    c, sc, z = oracle.unpack(*oracle.pack(c, sc, z), N, K)
    y_awq = oracle.matmul(xs, oracle.dequant(c, sc, z))

    c0, sc0, z0 = oracle.quantize(W)
    y_rtn = oracle.matmul(x, oracle.dequant(c0, sc0, z0))
    e_awq = np.sqrt(((y_awq - y_fp) ** 2).mean())
    e_rtn = np.sqrt(((y_rtn - y_fp) ** 2).mean())
    assert e_awq < 0.85 * e_rtn
    assert e_awq < 0.1 * np.sqrt((y_fp ** 2).mean())


def test_act_scale_closed_form():
    """Eq. 5: s = s_X^alpha with s_X the per-channel mean magnitude."""
    X = np.zeros((4, 3), np.float16)
    X[:, 0] = [1, -1, 3, -3]           # mean |x| = 2
    X[:, 1] = [0.25, 0.25, -0.25, 0.25]
    X[:, 2] = 0                         # floored
    assert np.allclose(oracle.act_scale(X, 0.5, floor=1e-4), [2 ** 0.5, 0.5, 1e-2], rtol=1e-15)
    assert np.allclose(oracle.act_scale(X, 0.0), [1, 1, 1])
    assert np.allclose(oracle.act_scale(X, 1.0), [2, 0.25, 1e-4])
    xs = oracle.apply_inv_scale(np.array([[1.0, 3.0, 5.0]], np.float16),
                                np.array([2.0, 3.0, 0.3], np.float32))
    assert np.array_equal(xs, np.array([[0.5, 1.0, np.float32(5.0) / np.float32(0.3)]]).astype(np.float16))


def test_norm_error_metric():
    x = np.array([[3.0, 4.0]], np.float16)              # ||x|| = 5
    Wdq = np.array([[0.5, -2.0], [1.0, 0.0]], np.float32)   # max|W| = 2
    y_ref = np.array([[1.0, 2.0]])
    y_gpu = np.array([[1.5, 2.0]], np.float16)
    err = oracle.norm_error(y_gpu, y_ref, x, Wdq)
    assert np.allclose(err, [[0.5 / (10 + 1e-6), 0.0]])
