"""Pins for the INT3-g128 variant of the oracle (AWQ Sec. 5: INT4/INT3, group size 128)."""
import numpy as np

import oracle


def test_codes_range_error_bound_and_round_off_statistic():
    g = np.random.default_rng(60)
    N, K = 64, 1024
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float16)
    s = g.uniform(0.5, 3.0, size=K).astype(np.float32)
    codes, scales, zeros = oracle.quantize_w3(W, s)
    assert codes.max() <= 7 and zeros.max() <= 7
    wp = W.astype(np.float32) * s[None, :]
    sc = np.repeat(scales.astype(np.float32), 128, axis=1)
    Wdq = oracle.dequant(codes, scales, zeros)
    lv = np.rint(wp / sc) + np.repeat(zeros, 128, axis=1)
    inside = (lv >= 0) & (lv <= 7)
    assert np.all(np.abs(Wdq - wp)[inside] <= sc[inside] * 0.5 * (1 + 1e-5))
    frac = np.abs(wp / sc - np.rint(wp / sc))
    assert abs(frac.mean() - 0.25) < 0.004                  # Sec. 3.2: expected round-off 0.25
    # the step is (max - min) / 7: about 15/7 of the 4-bit step of the same group
    _, s4, _ = oracle.quantize(W, s)
    ratio = scales.astype(np.float64) / s4.astype(np.float64)
    assert np.all(np.abs(ratio - 15 / 7) < 0.01)


def test_an_eight_level_grid_round_trips_exactly():
    g = np.random.default_rng(61)
    lv = g.integers(0, 8, size=(16, 384))
    lv[:, 0::128] = 0
    lv[:, 1::128] = 7
    W = ((lv - 3) * 2.0 ** -5).astype(np.float16)
    codes, scales, zeros = oracle.quantize_w3(W)
    assert np.array_equal(codes, lv.astype(np.uint8))
    assert np.all(scales == np.float16(2.0 ** -5)) and np.all(zeros == 3)
    assert np.array_equal(oracle.dequant(codes, scales, zeros), W.astype(np.float32))


def test_pack_round_trip_and_sizes():
    g = np.random.default_rng(62)
    N, K = 48, 640
    codes = g.integers(0, 8, size=(N, K), dtype=np.uint8)
    scales = g.uniform(0.001, 0.1, size=(N, K // 128)).astype(np.float16)
    zeros = g.integers(0, 8, size=(N, K // 128), dtype=np.uint8)
    q, sp, zp = oracle.pack_w3(codes, scales, zeros)
    assert (q.size, sp.size * 2, zp.size) == oracle.packed_sizes_w3(N, K) == (N * K * 3 // 8, N * 5 * 2, N * 5 // 2)
    c2, s2, z2 = oracle.unpack_w3(q, sp, zp, N, K)
    assert np.array_equal(c2, codes) and np.array_equal(z2, zeros)
    assert np.array_equal(s2.view(np.uint16), scales.view(np.uint16))
    # flipping one code changes exactly its three bits' worth of one slot
    codes2 = codes.copy()
    codes2[17, 300] ^= 7
    q2, _, _ = oracle.pack_w3(codes2, scales, zeros)
    changed = np.flatnonzero(q != q2)
    tile = (17 // 16) * 5 + 300 // 128
    slot = 17 % 16 + 16 * ((300 % 32) // 8)
    assert changed.size >= 1 and np.all(changed // 12 == tile * 64 + slot)
    assert sum(bin(int(a ^ b)).count("1") for a, b in zip(q[changed], q2[changed])) == 3


def test_hand_written_bytes_of_one_slot():
    """One tile, row 5, column block c = 2: codes i -> value (i % 8); every other code 0.
    Expected words written out by hand from the layout text."""
    codes = np.zeros((16, 128), np.uint8)
    for i in range(32):
        codes[5, 32 * (i // 8) + 8 * 2 + (i % 8)] = i % 8
    q, _, _ = oracle.pack_w3(codes, np.ones((16, 1), np.float16), np.zeros((16, 1), np.uint8))
    slot = 5 + 16 * 2
    words = q[slot * 12: slot * 12 + 12].view("<u4")
    # pairs p = (code 2p, code 2p+1) = values ((2p) % 8, (2p+1) % 8): (0,1),(2,3),(4,5),(6,7) repeating
    lo = [0, 2, 4, 6] * 4          # member h = 0 of pair p
    hi = [1, 3, 5, 7] * 4          # member h = 1
    want = [0, 0, 0]
    for p in range(15):
        want[p // 5] |= lo[p] << (3 * (p % 5))
        want[p // 5] |= hi[p] << (16 + 3 * (p % 5))
    for b in range(3):             # pair 15 = (6, 7): bit b of 6 at bit 15, of 7 at bit 31 of word b
        want[b] |= ((6 >> b) & 1) << 15
        want[b] |= ((7 >> b) & 1) << 31
    assert [int(w) for w in words] == want
    # word 0 by hand: low half fields (0,2,4,6,0) = 0 + 2<<3 + 4<<6 + 6<<9 + 0<<12 = 0x0D10, bit 15 = 0;
    # high half fields (1,3,5,7,1) = 1 + 3<<3 + 5<<6 + 7<<9 + 1<<12 = 0x1F59, bit 31 = 1 -> 0x9F59
    assert int(words[0]) == 0x9F590D10
    everything_else = np.delete(q, np.arange(slot * 12, slot * 12 + 12))
    assert not everything_else.any()
