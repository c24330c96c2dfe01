"""Pins for the oracle's quantizer (AWQ Sec. 3.2, Eq. 1-3; asymmetric min/max form).

None of these retype the quantizer: they are invariants, closed forms and
constructed inputs with a known answer, chosen so that a dropped term, a wrong
sign, a wrong index or a transposed operand fails at least one of them.
"""
import numpy as np
import pytest

import oracle

G = 128


def gauss(N, K, sigma=0.02, seed=0):
    g = np.random.default_rng(seed)
    return (g.standard_normal((N, K), dtype=np.float32) * np.float32(sigma)).astype(np.float16)


def expand(a, K):
    """[N,G] per-group values -> [N,K]"""
    return np.repeat(a, G, axis=1)[:, :K]


def test_codes_and_zeros_are_uint4():
    W = gauss(64, 1024, seed=3)
    s = np.random.default_rng(4).uniform(0.3, 5.0, size=1024).astype(np.float32)
    codes, scales, zeros = oracle.quantize(W, s)
    assert codes.dtype == np.uint8 and zeros.dtype == np.uint8
    assert codes.min() >= 0 and codes.max() <= 15
    assert zeros.min() >= 0 and zeros.max() <= 15
    assert np.all(np.isfinite(scales.astype(np.float32))) and np.all(scales > 0)


def test_error_bound_half_step():
    """Eq. 1: Q(w) = Delta * Round(w / Delta)  =>  |w - Q(w)| <= Delta / 2.
    Gaussian groups straddle zero, so no element is clipped beyond the closed-form
    slack 15 * 2^-11 * Delta that rounding Delta to binary16 can add at the top end."""
    N, K = 96, 2048
    W = gauss(N, K, seed=5)
    s = np.random.default_rng(6).uniform(0.5, 4.0, size=K).astype(np.float32)
    codes, scales, zeros = oracle.quantize(W, s)
    wp = W.astype(np.float32) * s[None, :]                      # exact inputs of Q
    Wdq = oracle.dequant(codes, scales, zeros).astype(np.float64)
    delta = expand(scales.astype(np.float64), K)
    err = np.abs(wp.astype(np.float64) - Wdq)
    inner = (codes > 0) & (codes < 15)
    assert np.all(err[inner] <= delta[inner] * (0.5 + 1e-6))
    assert np.all(err <= delta * (0.5 + 15 * 2.0 ** -11 + 1e-6))
    # the bound is tight: the worst element is close to half a step
    assert (err / delta).max() > 0.49


def test_round_off_is_uniform_mean_quarter():
    """Sec. 3.2 observation (1): RoundErr ~ U[0, 0.5], mean 0.25."""
    N, K = 256, 4096
    W = gauss(N, K, seed=7)
    codes, scales, zeros = oracle.quantize(W)
    Wdq = oracle.dequant(codes, scales, zeros).astype(np.float64)
    r = np.abs(W.astype(np.float64) - Wdq) / expand(scales.astype(np.float64), K)
    assert abs(r.mean() - 0.25) < 0.002
    hist, _ = np.histogram(r, bins=10, range=(0.0, 0.5))
    assert np.all(np.abs(hist / r.size - 0.1) < 0.004)


def test_end_point_codes():
    """The group minimum maps to code 0 and dequantizes to -zero*scale; the maximum
    maps to 14 or 15 (rint is odd, (max-min)/scale = 15 up to binary16 rounding)."""
    N, K = 128, 1024
    W = gauss(N, K, seed=8)
    codes, scales, zeros = oracle.quantize(W)
    Wg = W.astype(np.float32).reshape(N, K // G, G)
    cg = codes.reshape(N, K // G, G)
    amin = Wg.argmin(axis=2)
    amax = Wg.argmax(axis=2)
    cmin = np.take_along_axis(cg, amin[..., None], axis=2)[..., 0]
    cmax = np.take_along_axis(cg, amax[..., None], axis=2)[..., 0]
    assert np.all(cmin == 0)
    assert np.all(cmax >= 14)
    assert np.all(cg.max(axis=2) == cmax) and np.all(cg.min(axis=2) == 0)


def test_exact_grid_round_trips_with_zero_error():
    """Plain RTN special case (s = None): a group whose values already lie on a
    16-level grid a + b*i with both end points present is reproduced exactly."""
    N, K = 16, 512
    g = np.random.default_rng(9)
    b = 2.0 ** g.integers(-9, -5, size=(N, K // G))          # binary16-exact steps
    z = g.integers(0, 16, size=(N, K // G))                   # intended zero points
    lv = g.integers(0, 16, size=(N, K // G, G))
    lv[..., 0] = 0
    lv[..., 1] = 15
    lv = g.permuted(lv, axis=2)
    W = ((lv - z[..., None]) * b[..., None]).reshape(N, K).astype(np.float16)
    assert np.array_equal(W.astype(np.float64).reshape(N, K // G, G), (lv - z[..., None]) * b[..., None])
    codes, scales, zeros = oracle.quantize(W)
    assert np.array_equal(scales.astype(np.float64), b)
    assert np.array_equal(zeros, z)
    assert np.array_equal(codes.reshape(N, K // G, G), lv)
    assert np.array_equal(oracle.dequant(codes, scales, zeros), W.astype(np.float32))


def test_group_parameters_land_at_their_own_row_and_group():
    """Index pin: every (row, group) gets a distinct power-of-two step; a transposed
    or shifted index would move it."""
    N, K = 48, 640                     # N != G, K not a power of two
    Gn = K // G
    e = -(np.arange(N)[:, None] % 6) - (np.arange(Gn)[None, :] % 5) - 2     # step 2^e
    step = 2.0 ** e
    ramp = (np.arange(G) % 16).astype(np.float64)                          # codes 0..15
    W = (step[..., None] * (ramp - 8.0)).reshape(N, K).astype(np.float16)
    codes, scales, zeros = oracle.quantize(W)
    assert np.array_equal(scales.astype(np.float64), step)
    assert np.all(zeros == 8)
    assert np.array_equal(codes, np.tile(ramp.astype(np.uint8), (N, K // G)))


def test_scale_s_is_applied_along_input_channels():
    """Eq. 2: Q(w * s) with s indexed by the input channel k (not the output row).
    W == 1 everywhere, so the codes are decided by s alone."""
    N, K = 32, 256
    W = np.ones((N, K), dtype=np.float16)
    s = np.tile((np.arange(16, dtype=np.float32) + 1.0) * 0.25, K // 16)     # 0.25 .. 4.0
    s = np.roll(s, 3)
    codes, scales, zeros = oracle.quantize(W, s)
    assert np.all(scales.astype(np.float32) == 0.25)
    assert np.all(zeros == 0)          # -min/scale = -1 -> clamps to 0
    want = np.clip(np.rint(s / 0.25), 0, 15).astype(np.uint8)
    assert np.array_equal(codes, np.tile(want, (N, 1)))
    # s = None is the same as s = 1
    a = oracle.quantize(gauss(16, 256, seed=10))
    b = oracle.quantize(gauss(16, 256, seed=10), np.ones(256, dtype=np.float32))
    assert all(np.array_equal(x, y) for x, y in zip(a, b))


def test_codes_use_the_stored_fp16_step():
    """The step is stored in binary16 ("Delta ... represented in FP16", Sec. 3.2), and
    the codes are taken with the stored value: re-deriving each code from the
    stored parameters in exact arithmetic gives back the same code."""
    N, K = 64, 1024
    W = gauss(N, K, seed=11)
    codes, scales, zeros = oracle.quantize(W)
    delta = expand(scales.astype(np.float64), K)
    z = expand(zeros.astype(np.float64), K)
    t = W.astype(np.float64) / delta + z
    # away from rounding ties the nearest integer is unambiguous
    far = np.abs(t - np.floor(t) - 0.5) > 1e-4
    assert far.mean() > 0.99
    assert np.array_equal(np.clip(np.rint(t), 0, 15)[far], codes[far].astype(np.float64))
    # and the stored step is the binary16 rounding of (max-min)/15
    Wg = W.astype(np.float32).reshape(N, K // G, G)
    rng_ = (Wg.max(axis=2) - Wg.min(axis=2)).astype(np.float32) / np.float32(15)
    assert np.array_equal(rng_.astype(np.float16), scales)


def test_degenerate_and_one_sided_groups():
    K = 384
    W = np.zeros((16, K), dtype=np.float16)
    W[1, :] = 0.5                                   # constant positive
    W[2, :] = -0.25                                 # constant negative
    W[3, :G] = np.linspace(1.0, 2.5, G)             # all positive group: min > 0
    W[4, :G] = -np.linspace(1.0, 2.5, G)            # all negative group
    codes, scales, zeros = oracle.quantize(W)
    tiny = np.float16(2.0 ** -14)
    # all-zero rows: floor step, zero point 0, codes 0, dequant 0
    assert np.all(scales[0] == tiny) and np.all(zeros[0] == 0) and np.all(codes[0] == 0)
    # constant groups: floor step; everything clips to one end
    assert np.all(scales[1] == tiny) and np.all(zeros[1] == 0) and np.all(codes[1] == 15)
    assert np.all(scales[2] == tiny) and np.all(zeros[2] == 15) and np.all(codes[2] == 0)
    # one-sided groups: formulas applied literally, far side clips
    assert scales[3, 0] == np.float16(0.1) and zeros[3, 0] == 0
    assert codes[3, :G].max() == 15 and codes[3, :G].min() == 10      # 1.0/0.1 -> 10
    assert zeros[4, 0] == 15 and codes[4, :G].max() == 5 and codes[4, :G].min() == 0
    assert np.all(np.isfinite(oracle.dequant(codes, scales, zeros)))


def test_huge_range_clamps_step_to_fp16_max():
    W = np.zeros((16, G), dtype=np.float16)
    W[:, 0] = 65504.0
    W[:, 1] = -65504.0
    s = np.full(G, 16.0, dtype=np.float32)          # range/15 = 139 742 > 65504
    codes, scales, zeros = oracle.quantize(W, s)
    assert np.all(scales == np.float16(65504.0))
    assert np.all(np.isfinite(oracle.dequant(codes, scales, zeros)))


def test_error_ratio_law():
    """Eq. 3: scaling one input channel by s > 1 multiplies that channel's
    quantization error by (Delta'/Delta) / s.  Where Delta is unchanged the
    ratio of mean errors is 1/s (statistical, +-10 %)."""
    N, K = 4096, 256
    W = gauss(N, K, seed=12)
    Wf = W.astype(np.float64)
    ch = np.array([5, 77, 130, 201])
    c0, s0, z0 = oracle.quantize(W)
    e0 = np.abs(oracle.dequant(c0, s0, z0).astype(np.float64) - Wf)[:, ch]
    d0 = s0.astype(np.float64)[:, ch // G]
    for sval in (1.25, 1.5, 2.0):
        sv = np.ones(K, dtype=np.float32)
        sv[ch] = sval
        c1, s1, z1 = oracle.quantize(W, sv)
        eff = oracle.dequant(c1, s1, z1).astype(np.float64) / sv[None, :]
        e1 = np.abs(eff - Wf)[:, ch]
        d1 = s1.astype(np.float64)[:, ch // G]
        same = d1 == d0
        assert same.mean() > 0.5
        ratio_same = e1[same].mean() / e0[same].mean()
        assert abs(ratio_same * sval - 1.0) < 0.10
        ratio_all = e1.mean() / e0.mean()
        predicted = (d1 / d0).mean() / sval
        assert abs(ratio_all / predicted - 1.0) < 0.10
        # the step never shrinks when a channel is scaled up
        assert np.all(d1 >= d0)


def test_rejects_bad_shapes():
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((16, 100), dtype=np.float16))
    with pytest.raises(ValueError):
        oracle.pack(np.zeros((8, 128), np.uint8), np.zeros((8, 1), np.float16),
                    np.zeros((8, 1), np.uint8))


def test_scale_study_table_structure_on_the_oracle():
    """The table of Sec. 3.2 (1 % salient channels multiplied by s): its printed rows obey
    Err ratio = (Delta'/Delta) / s of Eq. 3, and the oracle's quantizer shows the same structure
    on seeded weights: no step shrinks, the share of changed steps and the mean step ratio grow
    with s, the error of the salient channels falls as (mean step ratio) / s."""
    import os
    rows = [tuple(float(v) for v in ln.split()) for ln in
            open(os.path.join(os.path.dirname(__file__), "golden", "table2_scale_study.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert [r[0] for r in rows] == [1.0, 1.25, 1.5, 2.0, 4.0]
    for sval, changed, ratio, reduction in rows:
        assert abs(ratio / sval - reduction) <= 0.0015             # printed to three decimals
    assert all(a[1] < b[1] and a[2] < b[2] and a[3] > b[3] for a, b in zip(rows, rows[1:]))

    N, K = 2048, 1024
    W = gauss(N, K, seed=21)
    Wf = W.astype(np.float64)
    salient = np.sort(np.random.default_rng(22).choice(K, size=K // 100, replace=False))
    c0, s0, z0 = oracle.quantize(W)
    d0 = s0.astype(np.float64)
    e0 = np.abs(oracle.dequant(c0, s0, z0).astype(np.float64) - Wf)[:, salient].mean()
    prev = (0.0, 1.0)
    for sval, _, _, _ in rows:
        sv = np.ones(K, dtype=np.float32)
        sv[salient] = sval
        c1, s1, z1 = oracle.quantize(W, sv)
        d1 = s1.astype(np.float64)
        assert np.all(d1 >= d0)
        changed, ratio = float((d1 != d0).mean()), float((d1 / d0).mean())
        e1 = np.abs(oracle.dequant(c1, s1, z1).astype(np.float64) / sv[None, :] - Wf)[:, salient].mean()
        grp = salient // G
        predicted = (d1 / d0)[:, grp].mean() / sval
        if sval == 1.0:
            assert changed == 0.0 and ratio == 1.0 and e1 == e0
        else:
            assert changed > prev[0] and ratio > prev[1]
            assert abs((e1 / e0) / predicted - 1.0) < 0.10
        prev = (changed, ratio)
