"""Pins for the oracle's scale search (AWQ Sec. 3.2, Eq. 4-5): the loss of a scaled, quantized
layer against the fp16 layer on cached calibration rows, and the grid search over alpha."""
import numpy as np

import oracle


def grid_weights(g, N, K, lo=-7, step=2.0 ** -6):
    """Weights on an exact 16-level grid per group with both end points present in every
    group: plain RTN (s = 1) reproduces them without error."""
    lv = g.integers(0, 16, size=(N, K))
    for grp in range(K // 128):
        lv[:, 128 * grp] = 0
        lv[:, 128 * grp + 1] = 15
    return ((lo + lv) * step).astype(np.float16), lv


def test_loss_is_zero_on_a_lossless_grid_and_has_the_closed_form_for_one_moved_weight():
    g = np.random.default_rng(40)
    N, K, T = 32, 256, 5
    W, lv = grid_weights(g, N, K)
    X = g.standard_normal((T, K)).astype(np.float16)
    ones = np.ones(K, np.float32)
    assert oracle.scale_search_loss(W, X, ones) == 0.0
    # move one interior weight a quarter step off the grid: range, step and every other code
    # stay, the moved weight rounds back to its level, so the layer output differs from the
    # fp16 layer by exactly e * X[:, k0] in column n0
    n0, k0 = 7, 130
    lv[n0, k0] = 5
    step = 2.0 ** -6
    W[n0, k0] = np.float16((-7 + 5 + 0.25) * step)
    e = -0.25 * step
    want = float(np.sum((e * X[:, k0].astype(np.float64)) ** 2))
    got = oracle.scale_search_loss(W, X, ones)
    assert abs(got - want) <= 1e-12 * want


def test_loss_matches_the_weight_error_form_in_exact_arithmetic():
    """(Q(W s) s^-1 - W) X summed in numpy float64 is the same quantity up to the fp16
    rounding of x / s, which the oracle keeps and this form does not."""
    g = np.random.default_rng(41)
    N, K, T = 48, 640, 33                       # all different: a transposed operand cannot pass
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float16)
    X = g.standard_normal((T, K)).astype(np.float32)
    X[:, g.choice(K, size=6, replace=False)] *= 20
    X = X.astype(np.float16)
    for alpha in (0.0, 0.35, 1.0):
        s = oracle.act_scale(X, alpha).astype(np.float32)
        codes, scales, zeros = oracle.quantize(W, s)
        E = oracle.dequant(codes, scales, zeros).astype(np.float64) / s.astype(np.float64)[None, :] \
            - W.astype(np.float64)
        want = float(np.sum((X.astype(np.float64) @ E.T) ** 2))
        got = oracle.scale_search_loss(W, X, s)
        assert abs(got / want - 1.0) < 2e-3
        assert got > 0


def test_loss_is_invariant_under_a_power_of_two_rescaling_of_s():
    """W (2s) doubles every scaled weight and every step exactly, x / (2s) halves exactly:
    the codes and the products are the same numbers."""
    g = np.random.default_rng(42)
    N, K, T = 32, 384, 9
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float16)
    X = g.standard_normal((T, K)).astype(np.float16)
    s = g.uniform(0.5, 3.0, size=K).astype(np.float32)
    a = oracle.scale_search_loss(W, X, s)
    for c in (2.0, 0.25):
        b = oracle.scale_search_loss(W, X, (s * np.float32(c)).astype(np.float32))
        assert abs(a - b) <= 1e-12 * a


def test_search_prefers_scaling_when_there_are_outlier_channels_and_not_otherwise():
    """Sec. 3.1-3.2: with a few input channels of large magnitude, protecting them (alpha > 0)
    lowers the output error; alpha = 0 is plain RTN.  Without such channels s_X is nearly flat
    and every alpha gives nearly the same loss."""
    g = np.random.default_rng(43)
    N, K, T = 128, 1024, 64
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float16)
    alphas = [i / 20 for i in range(20)]
    Xf = g.standard_normal((T, K)).astype(np.float32)
    flat = Xf.astype(np.float16)
    Xo = Xf.copy()
    Xo[:, g.choice(K, size=10, replace=False)] *= 20
    out = Xo.astype(np.float16)

    best, losses, s_best = oracle.search_scale(W, out, alphas)
    assert losses.shape == (20,) and best == int(np.argmin(losses))
    assert best > 0 and losses[best] < 0.8 * losses[0]
    assert np.array_equal(s_best, oracle.act_scale(out, alphas[best]).astype(np.float32))
    # the loss at alpha = 0 is the RTN loss (s = 1)
    assert losses[0] == oracle.scale_search_loss(W, out, np.ones(K, np.float32))

    best_f, losses_f, _ = oracle.search_scale(W, flat, alphas)
    assert losses_f.max() / losses_f.min() < 1.15
