"""First-order model of what the bf16 roundings of the HIP path do to an attention output.

Test infrastructure: it turns the precision reading (bf16 storage of the rotated Q and K, one more
bf16 rounding of the Q fragment that carries scale * log2(e), P rounded to bf16 before P.V, bf16
output; everything else fp32 with negligible error) into a tolerance for comparing the kernel with
the exact fp64 oracle on inputs whose scores are much larger than the unit-scale workloads', where
fixed bars say nothing.  Built on the oracle's own weights; shares nothing with the library.

For one query row with weights w_j = softmax(s)_j, output o_e = sum_j w_j v_je:
    d o_e / d s_j = w_j (v_je - o_e)
    s_j = scale <q, k_j>, so a perturbation of the operands gives
    delta s_j = scale (<dq, k_j> + <q, dk_j>)
A value x stored in bf16 (8 significant bits, round to nearest) is off by a quantity spread evenly
over +-ulp(x)/2, variance ulp(x)^2 / 12, ulp(x) = 2^(floor(log2 |x|) - 7).  Then
    Var_K[e] = scale^2 sum_j w_j^2 (v_je - o_e)^2 sum_i q_i^2 var(k_ji)          (independent per key)
    Var_Q[e] = scale^2 sum_i var(q_i) (sum_j w_j (v_je - o_e) k_ji)^2           (shared by all keys)
    Var_P[e] = rho^2 sum_j w_j^2 v_je^2   (each weight rounded on its own, the row sum is not)
    output rounding: at most half a bf16 ulp of the result, variance ulp(o)^2 / 12
with var(q_i) = ulp(q_i)^2/12 + ulp(c q_i)^2/(12 c^2) for the two roundings of Q (c = scale*log2 e);
with the rotary embedding off the stored Q and K are the exact inputs and only the second term is left.
"""
import math

import numpy as np

from oracle import kvra_oracle as orc

# mean of (ulp(x)/x)^2 / 12 for significands spread log-uniformly over [1, 2): 2^-14 / 12 * (3/8) / ln 2
RHO2 = 2.0 ** -14 / 12.0 * 0.375 / math.log(2.0)


def bf16_ulp(x):
    """Spacing of bf16 numbers at |x| (0 for x == 0)."""
    ax = np.abs(np.asarray(x, dtype=np.float64))
    out = np.zeros_like(ax)
    nz = ax > 0
    out[nz] = np.exp2(np.floor(np.log2(ax[nz])) - 7.0)
    return out


def _operand_variances(qr, kr, scale, stored_exactly):
    """Variances of the operand errors.  stored_exactly: the rotation was the identity (rotary embedding
    off), so Q and K reach the kernel as the exact bf16 inputs and only the Q fragment is rounded."""
    c = scale * math.log2(math.e)
    var_q = bf16_ulp(c * qr) ** 2 / (12.0 * c * c)
    if stored_exactly:
        return var_q, np.zeros_like(kr)
    return var_q + bf16_ulp(qr) ** 2 / 12.0, bf16_ulp(kr) ** 2 / 12.0


def head_sigma(qr, kr, v, scale, first_pos=0, stored_exactly=False, exact_q_term=True):
    """Predicted standard deviation of (kernel output before its final rounding - exact output) for ONE
    head: qr [n,d] rotated queries at positions first_pos.., kr [m,d] rotated keys, v [m,d].  Returns
    (sigma [n,d], exact output [n,d]).  With exact_q_term=False the Q term is replaced by its
    Cauchy-Schwarz upper bound  scale^2 (sum_j w_j (v_je - o_e)^2) (sum_i var(q_i) sum_j w_j k_ji^2),
    which costs no more than the attention itself."""
    qr, kr, v = (np.asarray(a, dtype=np.float64) for a in (qr, kr, v))
    w = orc.attention_weights(qr, kr, scale, first_pos=first_pos)          # [n, m]
    o = w @ v
    var_q, var_k = _operand_variances(qr, kr, scale, stored_exactly)
    b = (w * w) * ((qr * qr) @ var_k.T)                                    # [n, m]
    var_kpart = b @ (v * v) - 2.0 * o * (b @ v) + o * o * b.sum(axis=1, keepdims=True)
    if exact_q_term:
        wk = w @ kr                                                       # [n, d]
        var_qpart = np.empty_like(o)
        for t in range(qr.shape[0]):
            m_t = (v * w[t][:, None]).T @ kr - np.outer(o[t], wk[t])      # [e, i]
            var_qpart[t] = (m_t * m_t) @ var_q[t]
    else:
        spread = np.maximum(w @ (v * v) - o * o, 0.0)                      # [n, d]
        var_qpart = spread * np.sum(var_q * (w @ (kr * kr)), axis=1, keepdims=True)
    var_p = RHO2 * ((w * w) @ (v * v))
    var = scale * scale * (np.maximum(var_kpart, 0.0) + var_qpart) + var_p
    return np.sqrt(var), o


def sigma(q, k, v, scale, rope_base, rows=None, heads=None, exact_q_term=True):
    """The same for un-rotated q [C,H,d], k, v [C,Hkv,d] (full context, causal), on the given absolute
    rows (default: all) and query heads (default: all).  Returns (sigma, exact output), each
    [len(rows), len(heads), d]."""
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    C, H, d = q.shape
    Hkv = k.shape[1]
    rows = list(range(C)) if rows is None else [int(r) for r in rows]
    heads = list(range(H)) if heads is None else [int(h) for h in heads]
    if rope_base is not None:
        pos = np.arange(C)
        q = orc.rope(q, pos, rope_base)
        k = orc.rope(k, pos, rope_base)
    sig = np.empty((len(rows), len(heads), d))
    out = np.empty_like(sig)
    contiguous = rows == list(range(rows[0], rows[0] + len(rows)))
    for a, h in enumerate(heads):
        g = h // (H // Hkv)
        if contiguous:
            last = rows[-1] + 1
            s_, o_ = head_sigma(q[rows[0]:last, h], k[:last, g], v[:last, g], scale, rows[0], rope_base is None, exact_q_term)
            sig[:, a], out[:, a] = s_, o_
        else:
            for n, t in enumerate(rows):
                s_, o_ = head_sigma(q[t:t + 1, h], k[:t + 1, g], v[:t + 1, g], scale, t, rope_base is None, exact_q_term)
                sig[n, a], out[n, a] = s_[0], o_[0]
    return sig, out


K_SIGMA = 6.0          # elementwise bar, in predicted standard deviations (plus the output's half ulp)
MEAN_FACTOR = 1.25     # mean-abs bar over the expected mean-abs of the predicted distribution


def check(got, want, sig, label=""):
    """got: the kernel's bf16 outputs widened to fp64; want, sig: exact outputs and predicted standard
    deviations.  Elementwise |got - want| <= K_SIGMA sig + half a bf16 ulp of the result; mean-abs
    <= MEAN_FACTOR * mean of sqrt(2/pi) * sqrt(sig^2 + ulp^2/12).  Returns (worst ratio, mean-abs, mean bar)."""
    got, want, sig = (np.asarray(a, dtype=np.float64) for a in (got, want, sig))
    assert np.all(np.isfinite(got)), f"{label}: non-finite output"
    err = np.abs(got - want)
    half_ulp = 0.5 * bf16_ulp(np.maximum(np.abs(got), np.abs(want)))
    bar = K_SIGMA * sig + half_ulp + 1e-9
    ratio = float((err / bar).max())
    assert ratio <= 1.0, f"{label}: error {ratio:.2f} x the elementwise bar at {np.unravel_index(np.argmax(err / bar), err.shape)}"
    mean_bar = MEAN_FACTOR * float(np.mean(math.sqrt(2.0 / math.pi) * np.sqrt(sig * sig + bf16_ulp(want) ** 2 / 12.0)))
    assert err.mean() <= mean_bar, f"{label}: mean-abs {err.mean():.3e} above {mean_bar:.3e}"
    return ratio, float(err.mean()), mean_bar
