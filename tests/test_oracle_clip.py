"""Pins for the oracle's weight clipping (AWQ Sec. 3.2, one sentence: clipping that minimises
the MSE of quantization; the reading taken is a per-group search over a grid of range ratios)."""
import numpy as np

import oracle

RATIOS = [1.0 - 0.05 * i for i in range(11)]        # 1.0 ... 0.5


def gauss(seed, N, K, sigma=0.02):
    g = np.random.default_rng(seed)
    return (g.standard_normal((N, K)) * sigma).astype(np.float16), g


def sq_err(W, s, codes, scales, zeros):
    """Squared quantization error per group, from the separately pinned dequantizer."""
    wp = W.astype(np.float32) * (np.ones(W.shape[1], np.float32) if s is None else s)[None, :]
    d = oracle.dequant(codes, scales, zeros).astype(np.float64) - wp.astype(np.float64)
    N, K = W.shape
    return (d * d).reshape(N, K // 128, 128).sum(axis=2)


def test_a_grid_of_one_is_the_plain_quantizer():
    W, g = gauss(50, 48, 512)
    s = g.uniform(0.5, 2.0, size=512).astype(np.float32)
    c0, s0, z0 = oracle.quantize(W, s)
    c1, s1, z1, ch = oracle.quantize_clip(W, s, [1.0])
    assert np.array_equal(c0, c1) and np.array_equal(s0.view(np.uint16), s1.view(np.uint16))
    assert np.array_equal(z0, z1) and not ch.any()


def test_one_ratio_shrinks_the_range_and_saturates_what_lies_outside():
    W, g = gauss(51, 32, 256)
    r = np.float32(0.7)
    codes, scales, zeros, _ = oracle.quantize_clip(W, None, [r])
    wp = W.astype(np.float32).reshape(32, 2, 128)
    mx, mn = wp.max(axis=2) * r, wp.min(axis=2) * r
    sc = ((mx - mn) / np.float32(15)).astype(np.float16)
    assert np.array_equal(scales.view(np.uint16), sc.view(np.uint16))
    scf = scales.astype(np.float32)
    assert np.array_equal(zeros, np.clip(np.rint(-mn / scf), 0, 15).astype(np.uint8))
    cg = codes.reshape(32, 2, 128).astype(np.int32)
    inside = (wp >= mn[..., None]) & (wp <= mx[..., None])
    want = np.rint(wp / scf[..., None]).astype(np.int32) + zeros[..., None].astype(np.int32)
    assert np.array_equal(cg[inside], np.clip(want, 0, 15)[inside])
    # above the shrunk range: the top level, below it: level 0 (the zero point is well inside
    # for these two-sided groups)
    assert (cg[wp > mx[..., None]] == 15).all() and (cg[wp < mn[..., None]] == 0).all()
    assert (~inside).sum() > 100                    # the case is not vacuous


def test_the_choice_is_the_first_minimum_of_independently_evaluated_errors():
    W, g = gauss(52, 64, 640)
    s = g.uniform(0.25, 4.0, size=640).astype(np.float32)
    codes, scales, zeros, choice = oracle.quantize_clip(W, s, RATIOS)
    errs = np.stack([sq_err(W, s, *oracle.quantize_clip(W, s, [r])[:3]) for r in RATIOS])
    want = errs.argmin(axis=0)                      # first index of the minimum
    # the per-ratio sums here come from fp64 numpy on the dequantized weights, the oracle's from
    # its own fp32 differences: choices may differ only where two ratios are within rounding
    diff = choice != want
    if diff.any():
        e_sorted = np.sort(errs, axis=0)
        assert np.all((e_sorted[1] - e_sorted[0])[diff] <= 1e-6 * e_sorted[0][diff])
    assert diff.mean() < 1e-3
    # and the returned codes are those of the chosen ratio
    got = sq_err(W, s, codes, scales, zeros)
    assert np.allclose(got, np.take_along_axis(errs, choice[None].astype(np.int64), 0)[0], rtol=1e-6)
    # clipping never does worse than not clipping, and on Gaussian groups it does better
    assert np.all(got <= errs[0] * (1 + 1e-6))
    assert got.sum() < 0.97 * errs[0].sum()
    assert 0 < choice.mean() < len(RATIOS) - 1


def test_a_lossless_grid_keeps_the_full_range_wherever_it_is_listed():
    g = np.random.default_rng(53)
    lv = g.integers(0, 16, size=(16, 256))
    lv[:, 0::128] = 0
    lv[:, 1::128] = 15
    W = ((lv - 7) * 2.0 ** -6).astype(np.float16)
    for ratios in ([1.0, 0.9, 0.8], [0.8, 0.9, 1.0], [0.9, 1.0, 1.0]):
        codes, scales, zeros, choice = oracle.quantize_clip(W, None, ratios)
        assert np.all(choice == ratios.index(1.0))   # zero error; the first of equal ratios
        assert np.array_equal(codes, lv.astype(np.uint8))


def test_activation_weighted_choice_against_independent_evaluation_and_its_special_cases():
    W, g = gauss(54, 48, 512)
    K, T = 512, 40
    X = g.standard_normal((T, K)).astype(np.float32)
    X[:, g.choice(K, size=5, replace=False)] *= 20
    X = X.astype(np.float16)
    s = oracle.act_scale(X, 0.4).astype(np.float32)
    xs = oracle.apply_inv_scale(X, s)
    codes, scales, zeros, choice = oracle.quantize_clip(W, s, RATIOS, xs=xs)
    # independent route: one full quantization per ratio, the group's output error in numpy
    wp = (W.astype(np.float32) * s[None, :]).astype(np.float64)
    xg = xs.astype(np.float64).reshape(T, K // 128, 128)
    errs, deq = [], []
    for r in RATIOS:
        c, sc, z, _ = oracle.quantize_clip(W, s, [r])
        D = oracle.dequant(c, sc, z).astype(np.float64)
        deq.append(D)
        proj = np.einsum("ngk,tgk->ngt", (D - wp).reshape(48, K // 128, 128), xg)
        errs.append((proj ** 2).sum(axis=2))
    errs = np.stack(errs)
    want = errs.argmin(axis=0)
    diff = choice != want
    if diff.any():
        e_sorted = np.sort(errs, axis=0)
        assert np.all((e_sorted[1] - e_sorted[0])[diff] <= 1e-9 * e_sorted[0][diff])
    assert diff.mean() < 1e-2
    got = oracle.dequant(codes, scales, zeros).astype(np.float64)
    for i in range(len(RATIOS)):
        m = np.repeat(choice == i, 128, axis=1)
        assert np.array_equal(got[m], deq[i][m])
    # it differs from the weight-space choice, and lowers the output error on those rows
    _, _, _, choice_w = oracle.quantize_clip(W, s, RATIOS)
    assert (choice != choice_w).mean() > 0.2
    y = xs.astype(np.float64) @ wp.T
    out_err = lambda D: np.sum((xs.astype(np.float64) @ D.T - y) ** 2)
    assert out_err(got) < out_err(deq[0])
    # rows that are zero outside one group leave every other group indifferent: first ratio
    xz = np.zeros_like(xs)
    xz[:, 128:256] = xs[:, 128:256]
    _, _, _, cz = oracle.quantize_clip(W, s, RATIOS[::-1], xs=xz)
    assert np.all(cz[:, [0, 2, 3]] == 0) and np.array_equal(cz[:, 1], len(RATIOS) - 1 - choice[:, 1])
    # one-hot rows on every column make it the weight-space error
    eye = np.zeros((128, 512), np.float16)
    eye[np.arange(128), 128 + np.arange(128)] = 1
    _, _, _, ce = oracle.quantize_clip(W, s, RATIOS, xs=eye)
    assert np.array_equal(ce[:, 1], choice_w[:, 1])
    # a power-of-two factor on the rows changes no choice
    _, _, _, c4 = oracle.quantize_clip(W, s, RATIOS, xs=(xs.astype(np.float32) * 4).astype(np.float16))
    assert np.array_equal(c4, choice)
