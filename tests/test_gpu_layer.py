"""Parity of the decoder-layer kernels (through the C-ABI) with the fp64 oracle on the same seeded
bf16 inputs.

Bars.  A single operator (RMSNorm, linear layer) computes in fp32 and rounds once to bf16: it must
lie within one bf16 unit in the last place of the oracle value, |err| <= 2^-8 |want| + 1e-4.  The
whole layer stores six intermediate tensors in bf16 and is compared with the oracle run with the
same storage roundings.  The two sides disagree by one unit in the last place on part of the stored
elements (the attention kernel rounds P to bf16, fp32 versus fp64 accumulation flips roundings);
each linear stage passes such a perturbation on with gain weight_std * sqrt(fan_in) (1.3 - 2.1 at
the LLaMA-7B shape), a flip of x2 = x + attention branch reaches the output directly through the
residual, and the output's own rounding adds one more unit.  Measured noise at the LLaMA-7B shape:
mean 6.5e-3, max 6.3e-2 for |x2| + |y| of 2.9 on average.  Bars (about twice that):
|err| <= 4e-2 + 2^-6 (|x2| + |y|), mean-abs <= 1e-3 + 2^-8 mean(|x2| + |y|); against the exact oracle
(no storage rounding) |err| <= 8e-2 + 2^-5 (|x2| + |y|).  A structural mistake (dropped residual or
gain, wrong head mapping, transposed weight) shows as errors of order 1.
"""
import numpy as np
import pytest
import torch

from oracle import kvra_oracle as orc
from paper_2405_05329_amd import kvra, synth
from gpu_pipeline import to_bits, to_dev

pytestmark = pytest.mark.gpu


def _f64(bits):
    return orc.bf16_bits_to_f64(bits)


def _one_rounding(got_bits, want, label):
    got = _f64(got_bits)
    assert np.all(np.isfinite(got)), label
    err = np.abs(got - want)
    bound = 2.0 ** -8 * np.abs(want) + 1e-4
    worst = np.max(err - bound)
    assert worst <= 0, f"{label}: exceeds one-rounding bound by {worst:.3e} (max err {err.max():.3e})"


def _empty(*shape):
    return torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")


@pytest.mark.parametrize("rows,hidden", [(1, 64), (37, 4096), (130, 4544), (5, 8192), (300, 256)])
def test_rms_norm(rows, hidden):
    x = synth.normal_bf16(0, 20, 0, (rows, hidden), std=1.7)
    g = synth.normal_bf16(0, 20, 1, (hidden,), std=1.0)
    y = _empty(rows, hidden)
    kvra.kvra_rms_norm(to_dev(x), to_dev(g), y, rows, hidden, 1e-6)
    torch.cuda.synchronize()
    _one_rounding(to_bits(y), orc.rms_norm(_f64(x), _f64(g), 1e-6), f"rms_norm {rows}x{hidden}")


@pytest.mark.parametrize("m,n,k", [(1, 32, 64), (300, 512, 256), (257, 1056, 320), (513, 96, 4096), (64, 4352, 128),
                                   (1000, 768, 1024)])
@pytest.mark.parametrize("mode", ["plain", "residual", "swiglu"])
def test_linear(m, n, k, mode):
    x = synth.normal_bf16(1, 21, 0, (m, k))
    w = synth.normal_bf16(1, 21, 1, (n, k), std=k ** -0.5)
    xd, wd = to_dev(x), to_dev(w)
    out = _empty(m, n)
    xf, wf = _f64(x), _f64(w)
    if mode == "plain":
        kvra.kvra_linear(xd, wd, None, None, out, m, n, k)
        want = orc.linear(xf, wf)
    elif mode == "residual":
        r = synth.normal_bf16(1, 21, 2, (m, n))
        kvra.kvra_linear(xd, wd, None, to_dev(r), out, m, n, k)
        want = orc.linear(xf, wf) + _f64(r)
    else:
        w2 = synth.normal_bf16(1, 21, 3, (n, k), std=k ** -0.5)
        kvra.kvra_linear(xd, wd, to_dev(w2), None, out, m, n, k)
        want = orc.silu(orc.linear(xf, wf)) * orc.linear(xf, _f64(w2))
    torch.cuda.synchronize()
    _one_rounding(to_bits(out), want, f"linear {mode} {m}x{n}x{k}")


def test_linear_residual_in_place():
    m, n, k = 200, 256, 128
    x = synth.normal_bf16(2, 21, 0, (m, k))
    w = synth.normal_bf16(2, 21, 1, (n, k), std=k ** -0.5)
    r = synth.normal_bf16(2, 21, 2, (m, n))
    buf = to_dev(r)
    kvra.kvra_linear(to_dev(x), to_dev(w), None, buf, buf, m, n, k)
    torch.cuda.synchronize()
    _one_rounding(to_bits(buf), orc.linear(_f64(x), _f64(w)) + _f64(r), "linear residual in place")


@pytest.mark.parametrize("m,H,Hkv,d,k", [(300, 4, 4, 64, 256), (129, 4, 2, 128, 192), (70, 3, 1, 64, 128),
                                         (33, 71, 1, 64, 4544)])
def test_qkv_proj_segments(m, H, Hkv, d, k):
    n = (H + 2 * Hkv) * d
    x = synth.normal_bf16(3, 22, 0, (m, k))
    w = synth.normal_bf16(3, 22, 1, (n, k), std=k ** -0.5)
    q, kk, v = _empty(m, H, d), _empty(m, Hkv, d), _empty(m, Hkv, d)
    kvra.kvra_qkv_proj(to_dev(x), to_dev(w), q, kk, v, m, H, Hkv, d, k)
    torch.cuda.synchronize()
    want = orc.linear(_f64(x), _f64(w))
    _one_rounding(to_bits(q).reshape(m, H * d), want[:, :H * d], "q")
    _one_rounding(to_bits(kk).reshape(m, Hkv * d), want[:, H * d:(H + Hkv) * d], "k")
    _one_rounding(to_bits(v).reshape(m, Hkv * d), want[:, (H + Hkv) * d:], "v")


def test_argument_checks_do_not_launch():
    t = _empty(64, 64)
    with pytest.raises(kvra.KvraError):
        kvra.kvra_linear(t, t, None, None, t, 64, 48, 64)          # n not a multiple of 32
    with pytest.raises(kvra.KvraError):
        kvra.kvra_linear(t, t, None, None, t, 64, 64, 96)          # k not a multiple of 64
    with pytest.raises(kvra.KvraError):
        kvra.kvra_linear(t, t, t, t, t, 64, 64, 64)                # gate/up and residual together
    with pytest.raises(kvra.KvraError):
        kvra.kvra_rms_norm(t, t, t, 64, 60, 1e-6)                  # hidden not a multiple of 8
    with pytest.raises(kvra.KvraError):
        kvra.kvra_rms_norm(t, t, t, 1, 16384, 1e-6)                # beyond the register-resident width
    torch.cuda.synchronize()
    assert bool(torch.isnan(t.float()).all())                      # nothing was written


def _run_layer(cfg_id, seed, C, hidden, ffn, H, Hkv, d, weight_std, boundaries):
    wt = synth.make_layer_weights(seed, cfg_id, hidden, ffn, H, Hkv, d, weight_std)
    x = synth.normal_bf16(seed, cfg_id, 0, (C, hidden))
    dev = {k: to_dev(v) for k, v in wt.items()}
    scale = synth.default_scale(d)
    layer = kvra.make_layer(hidden, ffn, H, Hkv, d, synth.RMS_EPS, synth.ROPE_BASE, scale, dev["norm1"], dev["wqkv"],
                            dev["wo"], dev["norm2"], dev["w_gate"], dev["w_up"], dev["w_down"])
    xd = to_dev(x)
    y = _empty(C, hidden)
    k_cache, v_cache = _empty(C, Hkv, d), _empty(C, Hkv, d)
    cmax = max(b - a for a, b in zip(boundaries[:-1], boundaries[1:]))
    nbytes = kvra.kvra_layer_workspace_bytes(layer, cmax)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    for lo, hi in zip(boundaries[:-1], boundaries[1:]):
        kvra.kvra_layer_chunk(layer, xd[lo:hi], y[lo:hi], k_cache, v_cache, lo, hi - lo, C, ws, nbytes)
    torch.cuda.synchronize()
    f = {k: _f64(v) for k, v in wt.items()}
    q_rows = H * d
    weights = {"norm1": f["norm1"], "norm2": f["norm2"], "wq": f["wqkv"][:q_rows],
               "wk": f["wqkv"][q_rows:q_rows + Hkv * d], "wv": f["wqkv"][q_rows + Hkv * d:], "wo": f["wo"],
               "w_gate": f["w_gate"], "w_up": f["w_up"], "w_down": f["w_down"]}
    return _f64(x), weights, scale, _f64(to_bits(y)), _f64(to_bits(k_cache)), _f64(to_bits(v_cache))


@pytest.mark.parametrize("C,hidden,ffn,H,Hkv,d,std,bounds", [
    (300, 256, 448, 4, 2, 64, 0.06, [0, 130, 300]),
    (200, 512, 1024, 4, 4, 128, 0.045, [0, 1, 65, 200]),
    (160, 4096, 11008, 32, 32, 128, 0.02, [0, 96, 160]),
])
def test_layer_chunked(C, hidden, ffn, H, Hkv, d, std, bounds):
    x, weights, scale, got, kc, vc = _run_layer(30, 0, C, hidden, ffn, H, Hkv, d, std, bounds)
    assert np.all(np.isfinite(got))
    tr = {}
    stored, ks, vs = orc.decoder_layer(x, weights, H, Hkv, d, scale, synth.ROPE_BASE, synth.RMS_EPS,
                                       boundaries=bounds, rnd=orc.round_to_bf16, trace=tr)
    exact, _, _ = orc.decoder_layer(x, weights, H, Hkv, d, scale, synth.ROPE_BASE, synth.RMS_EPS)
    mag = np.abs(tr["x2"]) + np.abs(stored)
    err = np.abs(got - stored)
    print(f"layer {hidden}/{ffn} C={C}: vs stored-rounding oracle max {err.max():.3e} mean {err.mean():.3e}; "
          f"vs exact max {np.abs(got - exact).max():.3e} mean {np.abs(got - exact).mean():.3e}; "
          f"|x2|+|y| mean {mag.mean():.2f}")
    assert np.max(err - (4e-2 + 2.0 ** -6 * mag)) <= 0
    assert err.mean() <= 1e-3 + 2.0 ** -8 * mag.mean()
    assert np.max(np.abs(got - exact) - (8e-2 + 2.0 ** -5 * mag)) <= 0
    # the cache rows the layer wrote: V within one rounding of the projection, K likewise after rotation
    assert np.max(np.abs(vc - vs) - (2.0 ** -7 * np.abs(vs) + 1e-3)) <= 0
    assert np.max(np.abs(kc - ks) - (2.0 ** -6 * np.abs(ks) + 2e-2)) <= 0
