"""Pins for the oracle's attention: hand-computed rationals, closed forms, invariants and
torch's CPU scaled_dot_product_attention.  None of these retypes the oracle's formula."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import kvra_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_fixture(name):
    rows = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            rows[key] = vals
    return rows


def _rng(*key):
    return np.random.default_rng(list(key))


def test_hand_computed_rationals():
    fx = _read_fixture("softmax_rationals.txt")
    ln2 = np.log(2.0)
    q = np.array([[1.0, 0.0]] * 3).reshape(3, 1, 2)
    k = np.array([[0 * ln2, 7.0], [1 * ln2, 7.0], [2 * ln2, 7.0]]).reshape(3, 1, 2)
    v = np.array([[1.0, 0.0], [0.0, 1.0], [3.0, 3.0]]).reshape(3, 1, 2)
    w = orc.attention_weights(q[:, 0], k[:, 0], 1.0)
    out = orc.causal_attention(q, k, v, 1.0)
    for t in range(3):
        want_w = [float(Fraction(x)) for x in fx[f"weights_row{t}"]]
        want_o = [float(Fraction(x)) for x in fx[f"out_row{t}"]]
        np.testing.assert_allclose(w[t], want_w, rtol=0, atol=1e-15)
        np.testing.assert_allclose(out[t, 0], want_o, rtol=0, atol=1e-14)


def test_scale_enters_the_exponent():
    # q.k = 2 ln 2 for the second key; with scale 1/2 its weight is 2, not 4.
    ln2 = np.log(2.0)
    q = np.array([[1.0], [1.0]])
    k = np.array([[0.0], [2 * ln2]])
    w = orc.attention_weights(q, k, 0.5)
    np.testing.assert_allclose(w[1], [1 / 3, 2 / 3], atol=1e-15)


def test_first_row_sees_only_itself():
    r = _rng(1)
    q, k, v = r.standard_normal((5, 2, 4)), r.standard_normal((5, 2, 4)), r.standard_normal((5, 2, 4))
    out = orc.causal_attention(q, k, v, 0.37)
    np.testing.assert_allclose(out[0], v[0], atol=1e-15)


def test_zero_queries_give_running_mean_of_values():
    r = _rng(2)
    C, H, d = 17, 3, 8
    q = np.zeros((C, H, d))
    k, v = r.standard_normal((C, H, d)), r.standard_normal((C, H, d))
    out = orc.causal_attention(q, k, v, 1.0)
    want = np.cumsum(v, axis=0) / np.arange(1, C + 1).reshape(C, 1, 1)
    np.testing.assert_allclose(out, want, atol=1e-13)


def test_equal_keys_give_running_mean_of_values():
    r = _rng(3)
    C, H, d = 11, 1, 4
    q = r.standard_normal((C, H, d))
    k = np.broadcast_to(r.standard_normal((1, H, d)), (C, H, d)).copy()
    v = r.standard_normal((C, H, d))
    out = orc.causal_attention(q, k, v, 0.5, rope_base=None)
    want = np.cumsum(v, axis=0) / np.arange(1, C + 1).reshape(C, 1, 1)
    np.testing.assert_allclose(out, want, atol=1e-13)


def test_weights_are_row_stochastic_and_causal():
    r = _rng(4)
    q, k = r.standard_normal((40, 16)) * 3, r.standard_normal((52, 16)) * 3
    w = orc.attention_weights(q, k, 0.25, first_pos=12)
    assert np.all(w >= 0)
    np.testing.assert_allclose(w.sum(axis=1), 1.0, atol=1e-12)
    for t in range(40):
        assert np.all(w[t, 12 + t + 1:] == 0.0)
        assert w[t, 12 + t] > 0.0


def test_brute_force_triple_loop():
    r = _rng(5)
    C, H, Hkv, d, scale = 7, 4, 2, 6, 0.41
    q, k, v = r.standard_normal((C, H, d)), r.standard_normal((C, Hkv, d)), r.standard_normal((C, Hkv, d))
    out = orc.causal_attention(q, k, v, scale)
    for t in range(C):
        for h in range(H):
            g = h // 2
            num = np.zeros(d)
            den = 0.0
            for j in range(t + 1):
                e = np.exp(scale * sum(q[t, h, i] * k[j, g, i] for i in range(d)))
                num += e * v[j, g]
                den += e
            np.testing.assert_allclose(out[t, h], num / den, atol=1e-13)


@pytest.mark.parametrize("scale", [1.0, 0.125])
def test_against_torch_sdpa_cpu_fp64(scale):
    r = _rng(6)
    C, H, d = 33, 3, 16
    q, k, v = r.standard_normal((C, H, d)), r.standard_normal((C, H, d)), r.standard_normal((C, H, d))
    out = orc.causal_attention(q, k, v, scale)
    tq, tk, tv = (torch.from_numpy(x).permute(1, 0, 2).unsqueeze(0) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    np.testing.assert_allclose(out, ref[0].permute(1, 0, 2).numpy(), atol=1e-12)


def test_gqa_equals_mha_on_repeated_heads():
    r = _rng(7)
    C, H, Hkv, d = 19, 6, 2, 8
    q, k, v = r.standard_normal((C, H, d)), r.standard_normal((C, Hkv, d)), r.standard_normal((C, Hkv, d))
    a = orc.causal_attention(q, k, v, 0.3, rope_base=10000.0)
    b = orc.causal_attention(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1), 0.3, rope_base=10000.0)
    np.testing.assert_allclose(a, b, atol=1e-14)
    # head 2 must read kv head 0 and head 3 kv head 1: perturbing kv head 1 leaves heads 0..2 alone
    k2, v2 = k.copy(), v.copy()
    k2[:, 1] += 1.0
    v2[:, 1] -= 1.0
    c = orc.causal_attention(q, k2, v2, 0.3, rope_base=10000.0)
    np.testing.assert_array_equal(a[:, :3], c[:, :3])
    assert np.abs(a[:, 3:] - c[:, 3:]).max() > 1e-3


@pytest.mark.parametrize("bounds", [[0, 160, 256], [0, 256], [0, 1, 2, 3, 256], [0, 100, 101, 255, 256],
                                    list(range(0, 257, 32))])
def test_partition_invariance(bounds):
    # "does not alter any task accuracy" (Sec. 5): chunked result == full-context result
    r = _rng(8)
    C, H, Hkv, d = 256, 2, 1, 16
    q, k, v = r.standard_normal((C, H, d)), r.standard_normal((C, Hkv, d)), r.standard_normal((C, Hkv, d))
    full = orc.causal_attention(q, k, v, 0.25, rope_base=10000.0)
    out, kc, vc = orc.chunked_prefill(q, k, v, bounds, 0.25, rope_base=10000.0)
    np.testing.assert_allclose(out, full, atol=1e-12)
    np.testing.assert_array_equal(vc, v)
    np.testing.assert_allclose(kc, orc.rope(k, np.arange(C), 10000.0), atol=1e-15)


def test_chunks_of_one_token():
    r = _rng(9)
    C, H, d = 12, 1, 4
    q, k, v = r.standard_normal((C, H, d)), r.standard_normal((C, H, d)), r.standard_normal((C, H, d))
    full = orc.causal_attention(q, k, v, 0.5)
    out, _, _ = orc.chunked_prefill(q, k, v, list(range(C + 1)), 0.5)
    np.testing.assert_allclose(out, full, atol=1e-13)


def test_chunk_ignores_cache_rows_beyond_its_end():
    r = _rng(10)
    cap, H, d = 20, 2, 4
    kc, vc = r.standard_normal((cap, H, d)), r.standard_normal((cap, H, d))
    q = r.standard_normal((5, H, d))
    a = orc.chunk_attention(q, kc, vc, 7, 5, 0.5)
    kc[12:] = 1e9
    vc[12:] = -1e9
    b = orc.chunk_attention(q, kc, vc, 7, 5, 0.5)
    np.testing.assert_array_equal(a, b)


def test_attention_rows_matches_full():
    r = _rng(11)
    C, H, Hkv, d = 50, 4, 2, 8
    q, k, v = r.standard_normal((C, H, d)), r.standard_normal((C, Hkv, d)), r.standard_normal((C, Hkv, d))
    full = orc.causal_attention(q, k, v, 0.35, rope_base=10000.0)
    rows = [0, 1, 17, 49]
    got = orc.attention_rows(q, k, v, rows, 0.35, rope_base=10000.0)
    np.testing.assert_allclose(got, full[rows], atol=1e-13)


def test_bf16_round_trip_and_ties():
    # exact bf16 values survive; ties go to even; agrees with torch's conversion
    x = np.array([1.0, -1.0, 0.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, 3.14159, -2.71828e-3, 65280.0])
    bits = orc.f64_to_bf16_bits(x)
    back = orc.bf16_bits_to_f64(bits)
    assert back[0] == 1.0 and back[1] == -1.0 and back[2] == 0.0
    assert back[3] == 1.0                       # tie -> even mantissa (1.0)
    assert back[4] == 1.0 + 2 ** -6             # tie -> even mantissa (1 + 4/256)
    assert back[5] == 1.0 + 2 ** -7             # just above the tie -> up
    r = _rng(12)
    y = r.standard_normal(4096) * np.exp(r.uniform(-8, 8, 4096))
    want = torch.from_numpy(y.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    # float32 first then bf16 can double-round only on exact float32 ties, absent in random data
    np.testing.assert_array_equal(orc.f64_to_bf16_bits(y.astype(np.float32).astype(np.float64)), want)
