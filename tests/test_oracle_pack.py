"""Pins for the oracle's pack / unpack of the gfx950 byte layout (AWQ Sec. 4.2,
"SIMD-aware weight packing": a pure index permutation of the 4-bit codes).

The expected offsets below were worked out by hand from the layout text in the
library header (include/awq_mi355x.h), not computed by the oracle:
  tile (16 rows x 128 cols, 1024 B) index = (n // 16) * G + (k // 128)
  slot  = (n % 16) + 16 * ((k % 32) // 8), 16 B each; word j = (k % 128) // 32
  element e = k % 8 sits in nibble {0,4,1,5,2,6,3,7}[e] of the little-endian word
"""
import numpy as np

import oracle


def one_hot_pack(N, K, n, k, code=0xF, zero=None, g=None):
    codes = np.zeros((N, K), np.uint8)
    codes[n, k] = code
    scales = np.zeros((N, K // 128), np.float16)
    zeros = np.zeros((N, K // 128), np.uint8)
    if zero is not None:
        zeros[n, g] = zero
    return oracle.pack(codes, scales, zeros)


# (n, k) -> (byte offset in qweight, shift inside that byte), for N=32, K=256 (G=2)
HAND_PLACED = [
    ((0, 0), (0, 0)),                    # tile 0, slot 0, word 0, nibble 0
    ((0, 1), (2, 0)),                    # e=1 -> nibble 4 -> byte 2 low
    ((0, 2), (0, 4)),                    # e=2 -> nibble 1 -> byte 0 high
    ((0, 7), (3, 4)),                    # e=7 -> nibble 7 -> byte 3 high
    ((0, 8), (16 * 16, 0)),              # c=1 -> slot 16
    ((3, 17), (16 * (3 + 16 * 2) + 2, 0)),     # n=3, kk=17: j=0, c=2, e=1
    ((5, 100), (16 * (5 + 16 * 0) + 4 * 3 + 1, 0)),   # kk=100: j=3, c=0, e=4 -> nibble 2
    ((15, 127), (16 * (15 + 16 * 3) + 4 * 3 + 3, 4)), # last element of tile 0
    ((0, 128), (1024, 0)),               # next group of the same row block -> tile 1
    ((16, 0), (2048, 0)),                # next row block -> tile 2 (G = 2)
    ((31, 255), (3 * 1024 + 16 * 63 + 15, 4)),        # very last nibble
]


def test_hand_placed_nibbles():
    N, K = 32, 256
    for (n, k), (byte, shift) in HAND_PLACED:
        q, _, _ = one_hot_pack(N, K, n, k, code=0xB)
        want = np.zeros(N * K // 2, np.uint8)
        want[byte] = 0xB << shift
        assert np.array_equal(q, want), (n, k)


def test_scale_and_zero_placement():
    N, K = 32, 384                       # G = 3
    codes = np.zeros((N, K), np.uint8)
    scales = np.zeros((N, 3), np.float16)
    zeros = np.zeros((N, 3), np.uint8)
    scales[21, 2] = 1.5                  # row block 1, group 2, row 5
    zeros[21, 2] = 0xA
    zeros[20, 2] = 0x3
    _, sp, zp = oracle.pack(codes, scales, zeros)
    want_s = np.zeros(N * 3, np.float16)
    want_s[(1 * 3 + 2) * 16 + 5] = 1.5
    assert np.array_equal(sp.view(np.float16), want_s)
    want_z = np.zeros(N * 3 // 2, np.uint8)
    want_z[(1 * 3 + 2) * 8 + 2] = 0x3 | (0xA << 4)    # rows 4 (low) and 5 (high) of the block
    assert np.array_equal(zp, want_z)


def test_pack_is_a_bijection_on_nibbles():
    N, K = 32, 256
    seen = set()
    for n in range(N):
        for k in range(0, K, 5):
            q, _, _ = one_hot_pack(N, K, n, k, code=0xF)
            nz = np.flatnonzero(q)
            assert nz.size == 1 and q[nz[0]] in (0x0F, 0xF0)
            key = (int(nz[0]), int(q[nz[0]]))
            assert key not in seen
            seen.add(key)


def test_round_trip_random():
    g = np.random.default_rng(2)
    for N, K in [(16, 128), (48, 640), (64, 11008 // 2 + 128 * 1)]:
        codes = g.integers(0, 16, size=(N, K), dtype=np.uint8)
        scales = g.standard_normal((N, K // 128)).astype(np.float16)
        zeros = g.integers(0, 16, size=(N, K // 128), dtype=np.uint8)
        q, sp, zp = oracle.pack(codes, scales, zeros)
        assert (q.size, sp.size * 2, zp.size) == oracle.packed_sizes(N, K)
        c2, s2, z2 = oracle.unpack(q, sp, zp, N, K)
        assert np.array_equal(c2, codes) and np.array_equal(z2, zeros)
        assert np.array_equal(s2.view(np.uint16), scales.view(np.uint16))


def test_eight_codes_of_a_word_in_paper_order():
    """Sec. 4.2: each 8 weights are stored as w{0,2,4,6,1,3,5,7}: reading the
    nibbles of a word from low to high gives elements 0,2,4,6,1,3,5,7."""
    codes = np.zeros((16, 128), np.uint8)
    codes[0, :8] = np.arange(8) + 1      # element e has code e+1
    q, _, _ = oracle.pack(codes, np.zeros((16, 1), np.float16), np.zeros((16, 1), np.uint8))
    word = int.from_bytes(bytes(q[:4]), "little")
    nibbles = [(word >> (4 * p)) & 0xF for p in range(8)]
    assert nibbles == [1, 3, 5, 7, 2, 4, 6, 8]
