"""Pins of the rounding model that sets the GPU parity bars for large-score ("peaky") inputs.

The model (tests/rounding_model.py) predicts, to first order, the spread of the difference between
the exact attention output and one computed from operands rounded the way the precision reading
says: rotated Q and K stored in bf16, the Q fragment times scale*log2(e) rounded to bf16 again, P
rounded to bf16 before P.V with the row sum taken over the unrounded weights, bf16 output.  Here that
recipe is carried out on the CPU with the oracle's own functions, and the observed differences are
compared with the prediction: if the model dropped a term, the normalised error would be spread
wider than 1; if it over-counted, the bars built on it would be slack."""
import math

import numpy as np
import pytest

from oracle import kvra_oracle as orc
from paper_2405_05329_amd import synth

import rounding_model as rm


def _rounded_path(q, k, v, scale, rope_base):
    """The attention with every rounding of the precision reading applied, in fp64 otherwise."""
    f, b = orc.bf16_bits_to_f64, orc.f64_to_bf16_bits
    C, H, d = q.shape
    Hkv = k.shape[1]
    pos = np.arange(C)
    qr = f(b(orc.rope(f(q), pos, rope_base))) if rope_base is not None else f(q)
    kr = f(b(orc.rope(f(k), pos, rope_base))) if rope_base is not None else f(k)
    c = float(np.float32(scale) * np.float32(1.4426950408889634))
    q2 = f(b(qr * c))
    vv = f(v)
    out = np.empty((C, H, d))
    for h in range(H):
        g = h // (H // Hkv)
        s = q2[:, h] @ kr[:, g].T                         # base-2 scores
        s = np.where(np.arange(C)[None, :] <= pos[:, None], s, -np.inf)
        # against a reference that is not the row maximum itself but trails it by an amount that varies from
        # row to row, as the kernel's exponent reference does: with the maximum itself the largest weight
        # of every row would be exactly 1 and escape the rounding
        p = np.exp2(s - s.max(axis=1, keepdims=True) - np.random.default_rng(h).uniform(0.0, 1.0, size=(C, 1)))
        p_rounded = np.where(p > 1e-30, f(b(np.maximum(p, 1e-30))), 0.0)
        out[:, h] = (p_rounded @ vv[:, g]) / p.sum(axis=1, keepdims=True)
    return out


@pytest.mark.parametrize("gain,d,rope", [(1.0, 128, True), (4.0, 128, True), (8.0, 128, False), (4.0, 64, True)])
def test_model_predicts_the_spread_of_the_rounded_path(gain, d, rope):
    C, H, Hkv = 320, 2, 1
    rope_base = synth.ROPE_BASE if rope else None
    q, k, v = synth.make_qkv(11, 70, C, H, Hkv, d, q_gain=gain)
    scale = synth.default_scale(d)
    f = orc.bf16_bits_to_f64
    sig, want = rm.sigma(f(q), f(k), f(v), scale, rope_base)
    np.testing.assert_allclose(want, orc.causal_attention(f(q), f(k), f(v), scale, rope_base=rope_base), atol=1e-12)
    got = _rounded_path(q, k, v, scale, rope_base)
    z = (got - want)[8:] / sig[8:]                        # the first rows see a handful of keys: few terms, not Gaussian
    rms = float(np.sqrt(np.mean(z * z)))
    assert 0.85 <= rms <= 1.15, rms
    assert np.abs(z).max() <= 5.5
    # after the output rounding, every element sits inside the bar the GPU tests use
    final = f(orc.f64_to_bf16_bits(got))
    ratio, mean_abs, mean_bar = rm.check(final, want, sig, f"gain {gain}")
    assert ratio <= 0.9 and mean_abs >= 0.5 * mean_bar / rm.MEAN_FACTOR


def test_cheap_q_term_is_an_upper_bound():
    C, H, Hkv, d = 200, 2, 2, 64
    q, k, v = synth.make_qkv(12, 71, C, H, Hkv, d, q_gain=4.0)
    f = orc.bf16_bits_to_f64
    exact, _ = rm.sigma(f(q), f(k), f(v), synth.default_scale(d), synth.ROPE_BASE)
    bound, _ = rm.sigma(f(q), f(k), f(v), synth.default_scale(d), synth.ROPE_BASE, exact_q_term=False)
    assert np.all(bound >= exact * (1 - 1e-9))


def test_rows_and_heads_selection_agrees_with_the_full_evaluation():
    C, H, Hkv, d = 90, 4, 2, 64
    q, k, v = synth.make_qkv(13, 72, C, H, Hkv, d, q_gain=2.0)
    f = orc.bf16_bits_to_f64
    full, out = rm.sigma(f(q), f(k), f(v), 0.1, synth.ROPE_BASE)
    rows, heads = [0, 5, 17, 89], [1, 3]
    part, out_part = rm.sigma(f(q), f(k), f(v), 0.1, synth.ROPE_BASE, rows=rows, heads=heads)
    np.testing.assert_allclose(part, full[rows][:, heads], rtol=1e-9, atol=1e-15)
    np.testing.assert_allclose(out_part, out[rows][:, heads], rtol=1e-12, atol=1e-15)


def test_a_planted_mistake_in_the_rounded_path_breaks_the_bar():
    """The bar is tight enough to see an error of a few bf16 units: the same path with P rounded to 7
    significant bits instead of 8 no longer passes."""
    C, H, Hkv, d = 320, 2, 1, 128
    q, k, v = synth.make_qkv(11, 70, C, H, Hkv, d, q_gain=4.0)
    scale = synth.default_scale(d)
    f = orc.bf16_bits_to_f64
    sig, want = rm.sigma(f(q), f(k), f(v), scale, synth.ROPE_BASE)
    got = _rounded_path(q, k, v, scale, synth.ROPE_BASE)
    worse = want + 3.0 * (got - want)
    with pytest.raises(AssertionError):
        rm.check(f(orc.f64_to_bf16_bits(worse)), want, sig, "planted")
