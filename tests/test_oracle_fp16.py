"""Pins for the oracle's hand-written binary16 conversions: numpy's float16 is the
independent implementation (IEEE 754 round-to-nearest-even)."""
import numpy as np

import oracle


def test_f16_to_f32_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.f16_to_f32_scalar(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def _check_f32_to_f16(vals):
    vals = np.asarray(vals, dtype=np.float32)
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f32_to_f16_scalar(v) for v in vals], dtype=np.uint16)
    nan = np.isnan(vals)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7c00) == 0x7c00) and np.all((got[nan] & 0x3ff) != 0)


def test_f32_to_f16_random_bit_patterns():
    g = np.random.default_rng(1)
    bits = g.integers(0, 2 ** 32, size=200_000, dtype=np.uint64).astype(np.uint32)
    _check_f32_to_f16(bits.view(np.float32))


def test_f32_to_f16_ties_and_boundaries():
    # every half value, the midpoint to its successor, and one float either side of it
    hb = np.arange(0, 0x7c00, dtype=np.uint16)
    lo = hb.view(np.float16).astype(np.float64)
    hi = (hb + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    hi[-1] = 65536.0
    mid = ((lo + hi) / 2).astype(np.float32)          # exactly representable in fp32
    around = np.concatenate([mid, np.nextafter(mid, np.float32(np.inf)),
                             np.nextafter(mid, np.float32(-np.inf))])
    _check_f32_to_f16(around)
    _check_f32_to_f16(-around)
    _check_f32_to_f16([0.0, -0.0, 65504.0, 65519.99, 65520.0, 65536.0, 1e30, np.inf, -np.inf,
                       np.nan, 2.0 ** -24, 2.0 ** -25, np.nextafter(np.float32(2.0 ** -25), 1),
                       2.0 ** -14, 1e-45, 6.1e-5])
