"""Pins for the oracle's decode attention with rotary embedding and cache update (AWQ Sec. 4.2,
kernel fusion of the attention layer)."""
import numpy as np

import oracle


def caches(g, Hkv, Lmax, D, filled):
    kc = np.zeros((Hkv, Lmax, D), np.float16)
    vc = np.zeros((Hkv, Lmax, D), np.float16)
    kc[:, :filled] = g.standard_normal((Hkv, filled, D)).astype(np.float16)
    vc[:, :filled] = g.standard_normal((Hkv, filled, D)).astype(np.float16)
    return kc, vc


def test_rotation_keeps_norms_is_the_identity_at_zero_and_depends_on_relative_position():
    g = np.random.default_rng(100)
    a, b = g.standard_normal((2, 3, 128))
    assert np.array_equal(oracle.rope_rotate(a, 0), a)
    for pos in (1, 17, 4000):
        assert np.allclose(np.linalg.norm(oracle.rope_rotate(a, pos), axis=-1), np.linalg.norm(a, axis=-1))
    d1 = (oracle.rope_rotate(a, 40) * oracle.rope_rotate(b, 33)).sum(-1)
    d2 = (oracle.rope_rotate(a, 1007) * oracle.rope_rotate(b, 1000)).sum(-1)
    assert np.allclose(d1, d2, atol=1e-9)
    # the first pair (i = 0) turns by exactly pos radians, the last one hardly at all
    e0 = np.zeros(128); e0[0] = 1.0
    r = oracle.rope_rotate(e0, 2)
    assert np.allclose([r[0], r[64]], [np.cos(2.0), np.sin(2.0)])
    e63 = np.zeros(128); e63[63] = 1.0
    r = oracle.rope_rotate(e63, 2)
    assert abs(r[63] - np.cos(2 * 10000.0 ** (-126 / 128))) < 1e-12 and r[63] > 0.999


def test_first_token_returns_its_value_and_fills_row_zero():
    g = np.random.default_rng(101)
    H, Hkv, D, Lmax = 8, 4, 128, 16
    q = g.standard_normal((H, D)).astype(np.float16)
    k = g.standard_normal((Hkv, D)).astype(np.float16)
    v = g.standard_normal((Hkv, D)).astype(np.float16)
    kc, vc = caches(g, Hkv, Lmax, D, 0)
    out, kc2, vc2 = oracle.decode_attention(q, k, v, kc, vc, 0)
    assert np.array_equal(out, np.repeat(v, 2, axis=0))          # head h reads kv head h // 2
    assert np.array_equal(kc2[:, 0], k) and np.array_equal(vc2[:, 0], v)
    assert not kc2[:, 1:].any() and not vc2[:, 1:].any()


def test_softmax_weights_uniform_keys_and_a_dominant_key():
    g = np.random.default_rng(102)
    H, Hkv, D, Lmax, pos = 4, 4, 128, 64, 37
    q = g.standard_normal((H, D)).astype(np.float16)
    k = g.standard_normal((Hkv, D)).astype(np.float16)
    v = g.standard_normal((Hkv, D)).astype(np.float16)
    kc, vc = caches(g, Hkv, Lmax, D, pos)
    # weights sum to one: all-ones values give ones
    out, _, _ = oracle.decode_attention(q, k, np.ones_like(v), kc, np.ones_like(vc), pos)
    assert np.all(out == np.float16(1.0))
    # zero queries: every position weighs the same, the result is the mean of the values
    out, _, vc2 = oracle.decode_attention(np.zeros_like(q), k, v, kc, vc, pos)
    want = vc2[:, : pos + 1].astype(np.float64).mean(axis=1)
    assert np.all(np.abs(out.astype(np.float64) - want) <= np.abs(want) * 2.0 ** -10 + 1e-6)
    # a cached key equal to 100 x the rotated query direction takes all the weight
    qr = oracle.rope_rotate(q.astype(np.float64), pos)
    kc3 = kc.copy()
    kc3[:, 5] = (qr * 8).astype(np.float16)
    out, _, _ = oracle.decode_attention(q, k, v, kc3, vc, pos)
    assert np.all(np.abs(out.astype(np.float64) - vc[:, 5].astype(np.float64)) < 1e-2)


def test_against_a_direct_numpy_evaluation_with_grouped_heads():
    g = np.random.default_rng(103)
    H, Hkv, D, Lmax, pos = 8, 2, 128, 300, 257
    q = g.standard_normal((H, D)).astype(np.float16)
    k = g.standard_normal((Hkv, D)).astype(np.float16)
    v = g.standard_normal((Hkv, D)).astype(np.float16)
    kc, vc = caches(g, Hkv, Lmax, D, pos)
    out, kc2, vc2 = oracle.decode_attention(q, k, v, kc, vc, pos)
    assert np.array_equal(kc2[:, :pos], kc[:, :pos]) and np.array_equal(vc2[:, pos], v)
    i = np.arange(64)
    ang = pos * 10000.0 ** (-2.0 * i / 128)
    def rot(x):
        x = x.astype(np.float64)
        return np.concatenate([x[:, :64] * np.cos(ang) - x[:, 64:] * np.sin(ang),
                               x[:, 64:] * np.cos(ang) + x[:, :64] * np.sin(ang)], axis=1)
    qr, kr = rot(q), rot(k)
    assert np.all(np.abs(kc2[:, pos].astype(np.float64) - kr) <= np.abs(kr) * 2.0 ** -10 + 1e-7)
    for h in range(H):
        keys = np.concatenate([kc[h // 4, :pos].astype(np.float64), kr[h // 4][None]])
        vals = np.concatenate([vc[h // 4, :pos].astype(np.float64), v[h // 4][None].astype(np.float64)])
        w = np.exp(keys @ qr[h] / np.sqrt(128))
        want = (w / w.sum()) @ vals
        assert np.all(np.abs(out[h].astype(np.float64) - want) <= 1e-3)
