"""Pins for the oracle's rotary embedding.  The pairing convention itself (half-split) is a
choice the paper does not fix; what is pinned here is that the function is that rotation."""
import numpy as np

from oracle import kvra_oracle as orc


def test_position_zero_is_identity():
    x = np.random.default_rng(0).standard_normal((1, 3, 8))
    np.testing.assert_array_equal(orc.rope(x, np.array([0]), 10000.0), x)


def test_head_dim_two_is_a_plane_rotation():
    # d = 2: one pair, theta_0 = 1, so (1, 0) at position t becomes (cos t, sin t)
    t = np.array([0, 1, 2, 100])
    x = np.tile(np.array([1.0, 0.0]), (4, 1, 1))
    y = orc.rope(x, t, 10000.0)
    np.testing.assert_allclose(y[:, 0, 0], np.cos(t), atol=1e-15)
    np.testing.assert_allclose(y[:, 0, 1], np.sin(t), atol=1e-15)


def test_equals_complex_multiplication_with_half_split_pairs():
    r = np.random.default_rng(1)
    T, H, d, base = 9, 2, 8, 10000.0
    x = r.standard_normal((T, H, d))
    pos = np.array([0, 1, 2, 3, 50, 1000, 4095, 16383, 32767])
    y = orc.rope(x, pos, base)
    for i in range(d // 2):
        theta = base ** (-(2 * i) / d)
        z = (x[..., i] + 1j * x[..., i + d // 2]) * np.exp(1j * pos * theta).reshape(T, 1)
        np.testing.assert_allclose(y[..., i], z.real, atol=1e-12)
        np.testing.assert_allclose(y[..., i + d // 2], z.imag, atol=1e-12)


def test_frequencies_fall_geometrically_from_one():
    # a unit vector in pair i at position 1 turns by base**(-2i/d): pair 0 by 1 rad, last pair by base**(-(d-2)/d)
    d, base = 8, 10000.0
    for i in range(d // 2):
        x = np.zeros((1, 1, d))
        x[0, 0, i] = 1.0
        y = orc.rope(x, np.array([1]), base)
        ang = np.arctan2(y[0, 0, i + d // 2], y[0, 0, i])
        np.testing.assert_allclose(ang, base ** (-2 * i / d), atol=1e-15)


def test_norm_preserving():
    r = np.random.default_rng(2)
    x = r.standard_normal((6, 2, 16))
    y = orc.rope(x, np.array([3, 77, 1234, 9999, 20000, 32767]), 10000.0)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)


def test_inner_product_depends_on_relative_position_only():
    r = np.random.default_rng(3)
    q, k = r.standard_normal((1, 1, 16)), r.standard_normal((1, 1, 16))
    def ip(m, n):
        return float(np.sum(orc.rope(q, np.array([m]), 10000.0) * orc.rope(k, np.array([n]), 10000.0)))
    assert abs(ip(10, 3) - ip(110, 103)) < 1e-10
    assert abs(ip(10, 3) - ip(7, 0)) < 1e-12
    # direction matters: with q = e_0, k = e_1 in d = 2 the product is sin(m - n)
    e0, e1 = np.array([[[1.0, 0.0]]]), np.array([[[0.0, 1.0]]])
    for m, n in [(10, 3), (3, 10), (5, 5)]:
        got = float(np.sum(orc.rope(e0, np.array([m]), 10000.0) * orc.rope(e1, np.array([n]), 10000.0)))
        assert abs(got - np.sin(m - n)) < 1e-14


def test_attention_is_invariant_to_a_common_position_shift():
    r = np.random.default_rng(4)
    C, H, d = 24, 2, 8
    q, k, v = r.standard_normal((C, H, d)), r.standard_normal((C, H, d)), r.standard_normal((C, H, d))
    base = orc.causal_attention(q, k, v, 0.3, rope_base=10000.0)
    # same attention computed on tokens sitting at positions 500..523: rotate by hand, no rope inside
    qs = orc.rope(q, 500 + np.arange(C), 10000.0)
    ks = orc.rope(k, 500 + np.arange(C), 10000.0)
    shifted = orc.causal_attention(qs, ks, v, 0.3, rope_base=None)
    np.testing.assert_allclose(shifted, base, atol=1e-9)


def test_append_rotates_keys_and_queries_by_absolute_position():
    r = np.random.default_rng(5)
    cap, c, prefix, Hkv, H, d = 40, 6, 21, 1, 2, 8
    kc, vc = np.full((cap, Hkv, d), 5.0), np.full((cap, Hkv, d), -5.0)
    k, v, q = r.standard_normal((c, Hkv, d)), r.standard_normal((c, Hkv, d)), r.standard_normal((c, H, d))
    qr = orc.append_kv(kc, vc, k, v, prefix, 10000.0, q=q)
    pos = prefix + np.arange(c)
    np.testing.assert_array_equal(kc[prefix:prefix + c], orc.rope(k, pos, 10000.0))
    np.testing.assert_array_equal(vc[prefix:prefix + c], v)
    np.testing.assert_array_equal(qr, orc.rope(q, pos, 10000.0))
    assert np.all(kc[:prefix] == 5.0) and np.all(kc[prefix + c:] == 5.0)
    assert np.all(vc[:prefix] == -5.0) and np.all(vc[prefix + c:] == -5.0)
