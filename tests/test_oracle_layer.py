"""Pins for the oracle's decoder layer: library routines on special cases, closed forms, an
independent composition out of torch's CPU operators, and invariants."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import kvra_oracle as orc


def _weights(rng, hidden, H, Hkv, d, ffn, std=0.05):
    def w(*shape):
        return rng.standard_normal(shape) * std
    return {"norm1": 1.0 + 0.1 * rng.standard_normal(hidden), "norm2": 1.0 + 0.1 * rng.standard_normal(hidden),
            "wq": w(H * d, hidden), "wk": w(Hkv * d, hidden), "wv": w(Hkv * d, hidden), "wo": w(hidden, H * d),
            "w_gate": w(ffn, hidden), "w_up": w(ffn, hidden), "w_down": w(hidden, ffn)}


def test_rms_norm_against_torch_and_closed_forms():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 48))
    g = rng.standard_normal(48)
    want = F.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-6).numpy()
    np.testing.assert_allclose(orc.rms_norm(x, g, 1e-6), want, rtol=1e-13, atol=1e-13)
    # constant rows: a / sqrt(a^2 + eps)
    a = 3.0
    y = orc.rms_norm(np.full((2, 5), a), np.ones(5), 0.25)
    np.testing.assert_allclose(y, a / math.sqrt(a * a + 0.25), rtol=1e-15)
    # without eps the output does not depend on the scale of the input and has unit mean square
    y1 = orc.rms_norm(x, np.ones(48), 0.0)
    np.testing.assert_allclose(orc.rms_norm(17.0 * x, np.ones(48), 0.0), y1, rtol=1e-13)
    np.testing.assert_allclose(np.mean(y1 * y1, axis=-1), 1.0, rtol=1e-13)


def test_silu_and_linear_against_torch():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 12)) * 4
    np.testing.assert_allclose(orc.silu(x), F.silu(torch.from_numpy(x)).numpy(), rtol=1e-13, atol=1e-15)
    assert orc.silu(np.zeros(3)).tolist() == [0.0, 0.0, 0.0]
    np.testing.assert_allclose(orc.silu(x) - orc.silu(-x), x, rtol=1e-13, atol=1e-13)   # x s(x) + x s(-x)... = x
    w = rng.standard_normal((9, 12))                       # [out, in], not square: a transposed use fails
    np.testing.assert_allclose(orc.linear(x, w), F.linear(torch.from_numpy(x), torch.from_numpy(w)).numpy(),
                               rtol=1e-13, atol=1e-13)
    assert orc.linear(x, w).shape == (5, 9)


def _torch_layer(x, wt, H, Hkv, d, scale, base, eps):
    """The same layer composed from torch's CPU operators; rotary embedding written with complex
    numbers on (x_i, x_{i+d/2}) pairs so that it shares nothing with the oracle's formulation."""
    t = {k: torch.from_numpy(np.asarray(v)) for k, v in wt.items()}
    X = torch.from_numpy(x)
    C, hidden = X.shape

    def rot(u):                                               # u [C, heads, d]
        half = d // 2
        z = torch.complex(u[..., :half], u[..., half:])
        theta = base ** (-2.0 * torch.arange(half, dtype=torch.float64) / d)
        ang = torch.arange(C, dtype=torch.float64)[:, None] * theta[None, :]
        z = z * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    h1 = F.rms_norm(X, (hidden,), t["norm1"], eps=eps)
    q = rot(F.linear(h1, t["wq"]).view(C, H, d)).transpose(0, 1)
    k = rot(F.linear(h1, t["wk"]).view(C, Hkv, d)).transpose(0, 1).repeat_interleave(H // Hkv, dim=0)
    v = F.linear(h1, t["wv"]).view(C, Hkv, d).transpose(0, 1).repeat_interleave(H // Hkv, dim=0)
    a = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True, scale=scale)[0]
    a = a.transpose(0, 1).reshape(C, H * d)
    x2 = X + F.linear(a, t["wo"])
    h2 = F.rms_norm(x2, (hidden,), t["norm2"], eps=eps)
    y = x2 + F.linear(F.silu(F.linear(h2, t["w_gate"])) * F.linear(h2, t["w_up"]), t["w_down"])
    return y.numpy()


@pytest.mark.parametrize("H,Hkv,d,hidden,ffn,C", [(4, 4, 16, 64, 96, 23), (4, 2, 8, 32, 80, 17), (6, 1, 8, 40, 56, 12)])
def test_decoder_layer_against_torch_composition(H, Hkv, d, hidden, ffn, C):
    rng = np.random.default_rng(5)
    wt = _weights(rng, hidden, H, Hkv, d, ffn, std=0.2)
    x = rng.standard_normal((C, hidden))
    scale = d ** -0.5
    y, kc, vc = orc.decoder_layer(x, wt, H, Hkv, d, scale, 10000.0, 1e-6)
    np.testing.assert_allclose(y, _torch_layer(x, wt, H, Hkv, d, scale, 10000.0, 1e-6), rtol=1e-11, atol=1e-11)


def test_decoder_layer_partition_invariance_and_cache():
    rng = np.random.default_rng(6)
    H, Hkv, d, hidden, ffn, C = 4, 2, 8, 32, 48, 29
    wt = _weights(rng, hidden, H, Hkv, d, ffn, std=0.2)
    x = rng.standard_normal((C, hidden))
    whole, k0, v0 = orc.decoder_layer(x, wt, H, Hkv, d, d ** -0.5, 10000.0, 1e-6)
    for bounds in ([0, 10, 20, 29], [0, 1, 2, 28, 29], [0, 29]):
        part, k1, v1 = orc.decoder_layer(x, wt, H, Hkv, d, d ** -0.5, 10000.0, 1e-6, boundaries=bounds)
        np.testing.assert_allclose(part, whole, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(k1, k0, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(v1, v0, rtol=1e-12, atol=1e-12)


def test_decoder_layer_special_cases():
    rng = np.random.default_rng(7)
    H, Hkv, d, hidden, ffn, C = 2, 2, 8, 16, 24, 9
    wt = _weights(rng, hidden, H, Hkv, d, ffn, std=0.3)
    x = rng.standard_normal((C, hidden))
    # both output projections zero: the residual path alone survives
    z = dict(wt, wo=np.zeros_like(wt["wo"]), w_down=np.zeros_like(wt["w_down"]))
    y, _, _ = orc.decoder_layer(x, z, H, Hkv, d, d ** -0.5, 10000.0, 1e-6)
    np.testing.assert_array_equal(y, x)
    # MLP off: y = x + attention branch; the first token attends to itself, so its branch is wo v_0
    z = dict(wt, w_down=np.zeros_like(wt["w_down"]))
    y, kc, vc = orc.decoder_layer(x, z, H, Hkv, d, d ** -0.5, 10000.0, 1e-6)
    np.testing.assert_allclose(y[0], x[0] + wt["wo"] @ vc[0].reshape(-1), rtol=1e-12, atol=1e-12)
    # gate weights zero: silu(0) = 0 switches the MLP off whatever the other weights are
    z2 = dict(wt, w_gate=np.zeros_like(wt["w_gate"]))
    y2, _, _ = orc.decoder_layer(x, z2, H, Hkv, d, d ** -0.5, 10000.0, 1e-6)
    np.testing.assert_allclose(y2, y, rtol=1e-12, atol=1e-12)


def test_storage_rounding_hook():
    rng = np.random.default_rng(8)
    H, Hkv, d, hidden, ffn, C = 2, 1, 8, 16, 24, 11
    wt = {k: orc.round_to_bf16(v) for k, v in _weights(rng, hidden, H, Hkv, d, ffn, std=0.3).items()}
    x = orc.round_to_bf16(rng.standard_normal((C, hidden)))
    exact, _, _ = orc.decoder_layer(x, wt, H, Hkv, d, d ** -0.5, 10000.0, 1e-6)
    stored, kc, vc = orc.decoder_layer(x, wt, H, Hkv, d, d ** -0.5, 10000.0, 1e-6, rnd=orc.round_to_bf16)
    for t in (stored, kc, vc):                               # everything that is kept is a bf16 value
        np.testing.assert_array_equal(orc.round_to_bf16(t), t)
    assert np.max(np.abs(stored - exact)) < 0.05             # a handful of 2^-9 relative roundings
    assert np.max(np.abs(stored - exact)) > 0.0
    v = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -(1.0 + 2 ** -8 + 2 ** -20)])
    assert orc.round_to_bf16(v).tolist() == [1.0, 1.0, 1.0 + 2 ** -6, -(1.0 + 2 ** -7)]


def test_rows_evaluation_against_the_torch_composition_and_the_whole_layer():
    """decoder_layer_rows / layer_kv_cache (the forms used on long contexts): the sampled rows equal the rows of
    the layer composed from torch's operators and of decoder_layer run whole and in chunks; the cache equals
    the one the chunked run leaves behind."""
    rng = np.random.default_rng(21)
    C, hidden, H, Hkv, d, ffn = 57, 48, 4, 2, 16, 80
    wt = _weights(rng, hidden, H, Hkv, d, ffn, std=0.15)
    x = rng.standard_normal((C, hidden))
    rows = [0, 1, 19, 20, 56]
    want = _torch_layer(x, wt, H, Hkv, d, 0.25, 10000.0, 1e-6)
    tr = {}
    whole, kc, vc = orc.decoder_layer(x, wt, H, Hkv, d, 0.25, 10000.0, 1e-6, boundaries=[0, 20, 21, 57], trace=tr)
    y, x2 = orc.decoder_layer_rows(x, wt, H, Hkv, d, 0.25, 10000.0, 1e-6, rows)
    np.testing.assert_allclose(y, want[rows], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(y, whole[rows], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(x2, tr["x2"][rows], rtol=1e-11, atol=1e-12)
    k, v = orc.layer_kv_cache(x, wt, Hkv, d, 10000.0, 1e-6)
    np.testing.assert_allclose(k, kc, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(v, vc, rtol=1e-12, atol=1e-13)
    # a cache handed in is used as it is
    y2, _ = orc.decoder_layer_rows(x, wt, H, Hkv, d, 0.25, 10000.0, 1e-6, rows, cache=(k, v))
    np.testing.assert_allclose(y2, y, rtol=1e-13, atol=1e-14)
    # without rotary embedding
    y3, _ = orc.decoder_layer_rows(x, wt, H, Hkv, d, 0.25, None, 1e-6, rows)
    np.testing.assert_allclose(y3, orc.decoder_layer(x, wt, H, Hkv, d, 0.25, None, 1e-6)[0][rows], rtol=1e-11, atol=1e-12)


def test_rows_evaluation_with_storage_rounding_follows_the_whole_layer():
    """With bf16 storage of every intermediate the row-at-a-time sums differ from the batched ones in the last
    bits of fp64, which can flip a rounding now and then: all but a few elements are identical, the rest
    differ by what one flipped rounding upstream can cause."""
    rng = np.random.default_rng(22)
    C, hidden, H, Hkv, d, ffn = 40, 64, 4, 4, 16, 96
    wt = _weights(rng, hidden, H, Hkv, d, ffn, std=0.1)
    x = orc.round_to_bf16(rng.standard_normal((C, hidden)))
    rows = list(range(0, C, 3))
    whole, _, _ = orc.decoder_layer(x, wt, H, Hkv, d, 0.25, 10000.0, 1e-6, rnd=orc.round_to_bf16)
    y, _ = orc.decoder_layer_rows(x, wt, H, Hkv, d, 0.25, 10000.0, 1e-6, rows, rnd=orc.round_to_bf16)
    diff = np.abs(y - whole[rows])
    assert (diff > 0).mean() < 0.02
    assert diff.max() <= 2.0 ** -6 * np.abs(whole).max()
