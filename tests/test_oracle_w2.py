"""Pins for the INT2-g64 variant of the oracle (AWQ Sec. 5, extreme low-bit table: INT2, group 64)."""
import numpy as np
import pytest

import oracle


def test_codes_range_error_bound_and_round_off_statistic():
    g = np.random.default_rng(70)
    N, K = 64, 1024
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float16)
    s = g.uniform(0.5, 3.0, size=K).astype(np.float32)
    codes, scales, zeros = oracle.quantize_w2(W, s)
    assert codes.shape == (N, K) and scales.shape == zeros.shape == (N, K // 64)
    assert codes.max() <= 3 and zeros.max() <= 3
    wp = W.astype(np.float32) * s[None, :]
    sc = np.repeat(scales.astype(np.float32), 64, axis=1)
    Wdq = oracle.dequant(codes, scales, zeros, group=64)
    lv = np.rint(wp / sc) + np.repeat(zeros, 64, axis=1)
    inside = (lv >= 0) & (lv <= 3)
    assert np.all(np.abs(Wdq - wp)[inside] <= sc[inside] * 0.5 * (1 + 1e-5))
    # a clipped value is off by less than one step more (the zero point is rounded)
    assert np.all(np.abs(Wdq - wp) <= sc * 1.0 * (1 + 1e-3))
    # Sec. 3.2: the expected round-off of a value spread evenly over the steps is 0.25 (with four
    # levels a normal group is not spread evenly over a step, so the check uses uniform weights)
    Wu = g.uniform(-0.05, 0.05, size=(N, K)).astype(np.float16)
    _, su, _ = oracle.quantize_w2(Wu)
    ru = Wu.astype(np.float32) / np.repeat(su.astype(np.float32), 64, axis=1)
    assert abs(np.abs(ru - np.rint(ru)).mean() - 0.25) < 0.01
    # the step is (max - min) / 3 of the group of 64
    span = wp.reshape(N, K // 64, 64)
    want = (span.max(axis=2) - span.min(axis=2)) / 3
    assert np.all(np.abs(scales.astype(np.float64) / want - 1) < 2.0 ** -10)
    # the smallest value of a group has code 0 (rint(a) + rint(-a)); the largest has code 3, or 2
    # where the two roundings of the ends of the range both go down
    cg = codes.reshape(N, K // 64, 64)
    assert np.all(cg.min(axis=2) == 0) and np.all(cg.max(axis=2) >= 2)
    assert (cg.max(axis=2) == 3).mean() > 0.95


def test_a_four_level_grid_round_trips_exactly():
    g = np.random.default_rng(71)
    lv = g.integers(0, 4, size=(16, 512))
    lv[:, 0::64] = 0
    lv[:, 1::64] = 3
    W = ((lv - 1) * 2.0 ** -5).astype(np.float16)
    codes, scales, zeros = oracle.quantize_w2(W)
    assert np.array_equal(codes, lv.astype(np.uint8))
    assert np.all(scales == np.float16(2.0 ** -5)) and np.all(zeros == 1)
    assert np.array_equal(oracle.dequant(codes, scales, zeros, group=64), W.astype(np.float32))
    # the groups are 64 wide, not 128: two halves of a 128-column span with different ranges
    W2 = np.zeros((16, 256), np.float16)
    W2[:, :64] = ((lv[:, :64] - 1) * 2.0 ** -5)
    W2[:, 64:128] = ((lv[:, :64] - 2) * 2.0 ** -3)
    W2[:, 128:192] = W2[:, :64]
    W2[:, 192:] = W2[:, 64:128]
    c2, s2, z2 = oracle.quantize_w2(W2)
    assert np.array_equal(s2[0], np.array([2.0 ** -5, 2.0 ** -3] * 2, np.float16))
    assert np.array_equal(z2[0], np.array([1, 2, 1, 2], np.uint8))
    assert np.array_equal(oracle.dequant(c2, s2, z2, group=64), W2.astype(np.float32))


def test_pack_round_trip_and_sizes():
    g = np.random.default_rng(72)
    N, K = 48, 768
    G = K // 64
    codes = g.integers(0, 4, size=(N, K), dtype=np.uint8)
    scales = g.uniform(0.001, 0.1, size=(N, G)).astype(np.float16)
    zeros = g.integers(0, 4, size=(N, G), dtype=np.uint8)
    q, sp, zp = oracle.pack_w2(codes, scales, zeros)
    assert (q.size, sp.size * 2, zp.size) == oracle.packed_sizes_w2(N, K) == (N * K // 4, N * G * 2, N * G // 4)
    c2, s2, z2 = oracle.unpack_w2(q, sp, zp, N, K)
    assert np.array_equal(c2, codes) and np.array_equal(z2, zeros)
    assert np.array_equal(s2.view(np.uint16), scales.view(np.uint16))
    # flipping one code changes exactly its two bits, in the word of its column pair in its slot
    n, k = 17, 600
    codes2 = codes.copy()
    codes2[n, k] ^= 3
    q2, _, _ = oracle.pack_w2(codes2, scales, zeros)
    changed = np.flatnonzero(q != q2)
    block = (n // 16) * (K // 256) + k // 256
    slot = n % 16 + 16 * ((k % 32) // 8)
    word, half, field = (k % 8) // 2, k % 2, (k % 256) // 64 + 4 * ((k % 64) // 32)
    assert changed.size == 1 and changed[0] // 4 == (block * 64 + slot) * 4 + word
    assert changed[0] % 4 == (16 * half + 2 * field) // 8
    assert int(q[changed[0]] ^ q2[changed[0]]) == 3 << ((16 * half + 2 * field) % 8)
    # one scale and one zero point: their places
    scales2 = scales.copy()
    scales2[n, 9] = np.float16(7.0)
    zeros2 = zeros.copy()
    zeros2[n, 9] ^= 3
    _, sp2, zp2 = oracle.pack_w2(codes, scales2, zeros2)
    blk = (n // 16) * (K // 256) + 9 // 4
    assert np.flatnonzero(sp != sp2).tolist() == [(blk * 16 + n % 16) * 4 + 9 % 4]
    assert np.flatnonzero(zp != zp2).tolist() == [blk * 16 + n % 16]
    assert int(zp[blk * 16 + n % 16] ^ zp2[blk * 16 + n % 16]) == 3 << (2 * (9 % 4))
    with pytest.raises(Exception):
        oracle.pack_w2(codes[:, :640], scales[:, :10], zeros[:, :10])     # K not a multiple of 256


def test_hand_written_bytes_of_one_slot():
    """One block, row 5, column block c = 2, word i = 1 (columns 64t + 32j + 16 + 2 + h): the code
    of (t, j, h) is (t + j + h) % 4; every other code 0.  Expected word written out by hand from
    the layout text."""
    codes = np.zeros((16, 256), np.uint8)
    for t in range(4):
        for j in range(2):
            for h in range(2):
                codes[5, 64 * t + 32 * j + 8 * 2 + 2 * 1 + h] = (t + j + h) % 4
    q, _, _ = oracle.pack_w2(codes, np.ones((16, 4), np.float16), np.zeros((16, 4), np.uint8))
    slot = 5 + 16 * 2
    words = q[slot * 16: slot * 16 + 16].view("<u4")
    # low half (h = 0), fields f = t + 4j hold (t + j) % 4: f0..f7 = 0,1,2,3, 1,2,3,0
    #   = 1<<2 | 2<<4 | 3<<6 | 1<<8 | 2<<10 | 3<<12 = 4 + 32 + 192 + 256 + 2048 + 12288 = 0x39E4
    # high half (h = 1) holds (t + j + 1) % 4: f0..f7 = 1,2,3,0, 2,3,0,1
    #   = 1 | 2<<2 | 3<<4 | 2<<8 | 3<<10 | 1<<14 = 1 + 8 + 48 + 512 + 3072 + 16384 = 0x4E39
    assert [int(w) for w in words] == [0, 0x4E3939E4, 0, 0]
    everything_else = np.delete(q, np.arange(slot * 16, slot * 16 + 16))
    assert not everything_else.any()


def test_linear_of_the_two_bit_matrix_is_the_plain_product():
    g = np.random.default_rng(73)
    N, K, M = 32, 512, 3
    W = (g.standard_normal((N, K)) * 0.05).astype(np.float16)
    codes, scales, zeros = oracle.quantize_w2(W)
    x = g.standard_normal((M, K)).astype(np.float16)
    y = oracle.linear(x, codes, scales, zeros, group=64)
    Wdq = (codes.astype(np.float64) - np.repeat(zeros, 64, axis=1)) * np.repeat(scales.astype(np.float64), 64, axis=1)
    assert np.allclose(y, x.astype(np.float64) @ Wdq.T, rtol=1e-12, atol=1e-12)
