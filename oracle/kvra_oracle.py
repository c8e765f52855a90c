"""Plain fp64 CPU oracle of KV-Runahead's per-chunk hot path.

TEST INFRASTRUCTURE ONLY.  Slow, unblocked, unfused numpy written from the paper's
statement of the computation; it shares no code with the HIP library, does not import
it, and must not be called from the product path.

What it defines
  * causal attention of one layer on one process: softmax of the scaled Q.K^T map
    with the upper triangle masked to -inf, times V (Fig. 1(b); App. C listing,
    attention-weights and attention-output steps);
  * the KV-cache form each KV-Runahead process runs: concatenate the received cache
    with the local K,V, then attend the local queries to prefix+chunk keys
    (Sec. 4.1; Fig. 5; App. C listing, cache concatenation steps);
  * rotary position embedding (not in the paper; it comes from the LLaMA / Falcon
    models of Sec. 5 and is fixed here as the half-split "rotate-half" pairing);
  * the dot-product and traffic counts of Sec. 3 / Sec. 4.1 (Eq. 1-6, Fig. 4, Fig. 5);
  * the context-level load-balancing objective of Sec. 4.2 reduced to per-chunk costs:
    makespan of a partition, even split, exhaustive search; and its search tools: the
    one-dimensional scan for two processes, the hierarchical grid search, the lookup table
    with linear interpolation; and the time to first token of the chain of processes when
    every layer waits for the precedent's cache (Sec. 4 overview, Fig. 5(b));
  * the decoder layer a process runs around the attention block (App. C listing: q/k/v and
    output projections; RMSNorm and the SwiGLU MLP come from the LLaMA models of Sec. 5),
    exact or with bf16 storage rounding of every intermediate tensor; and the same layer evaluated for a
    few rows of a long context only (layer_kv_cache: K, V of every token; decoder_layer_rows: the rest of
    the layer for the chosen rows), which is the definition again with the rows that are not asked for
    left out, pinned against decoder_layer on a small case.

Pinned by tests/test_oracle_*.py against hand-computed rationals, closed forms,
torch's CPU scaled_dot_product_attention / rms_norm / silu / linear, the paper's worked
9-token example, its search example, brute force and (chain timing) closed forms.  Parity status: the rotary pairing convention (half-split versus
interleaved) is unpinned by the paper; everything else is pinned.
"""
from __future__ import annotations

import itertools
import math

import numpy as np


# --------------------------------------------------------------------------- bf16 helpers
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) exactly to float64."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float64 to the nearest bf16 (ties to even) and return the bit patterns.

    Done on the exact binary expansion of the double: keep 8 significant bits, look at
    the rest as guard/sticky.  Values are assumed finite and inside bf16's normal range
    (true for every tensor this repository generates).
    """
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros(x.shape, dtype=np.uint16)
    nz = x != 0.0
    m, e = np.frexp(np.abs(x[nz]))           # |x| = m * 2**e, 0.5 <= m < 1
    sig = m * 256.0                           # 8 significant bits live in [128, 256)
    lo = np.floor(sig)
    frac = sig - lo
    up = (frac > 0.5) | ((frac == 0.5) & (np.mod(lo, 2.0) == 1.0))
    lo = lo + up
    carry = lo == 256.0
    lo = np.where(carry, 128.0, lo)
    e = e + carry
    # value = lo * 2**(e-8), lo in [128,256): biased exponent = (e-1)+127, mantissa = lo-128
    bexp = (e - 1 + 127).astype(np.int64)
    if np.any(bexp <= 0) or np.any(bexp >= 255):
        raise ValueError("value outside bf16 normal range")
    bits = (bexp << 7) | (lo.astype(np.int64) - 128)
    bits = bits | (np.signbit(x[nz]).astype(np.int64) << 15)
    out[nz] = bits.astype(np.uint16)
    out[~nz] = (np.signbit(x[~nz]).astype(np.uint16) << np.uint16(15))
    return out


# --------------------------------------------------------------------------- rotary embedding
def rope(x: np.ndarray, positions: np.ndarray, base: float) -> np.ndarray:
    """Rotate x[t, h, :] by the angle set of absolute position positions[t].

    Half-split pairing: component i is paired with component i + d/2, and the pair is
    turned by phi = position * base**(-2 i / d).  Positions count tokens of the whole
    context from 0, so row r of a chunk that starts at `prefix` has position prefix + r.
    """
    x = np.asarray(x, dtype=np.float64)
    T, _, d = x.shape
    half = d // 2
    inv_freq = np.float64(base) ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    phi = np.asarray(positions, dtype=np.float64).reshape(T, 1) * inv_freq.reshape(1, half)
    cos = np.cos(phi)[:, None, :]
    sin = np.sin(phi)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * cos - hi * sin, hi * cos + lo * sin], axis=-1)


# --------------------------------------------------------------------------- attention
def attention_weights(q: np.ndarray, k: np.ndarray, scale: float, first_pos: int = 0) -> np.ndarray:
    """softmax(scale * q k^T + mask) for ONE head.

    q: [n, d] queries at absolute positions first_pos .. first_pos+n-1;
    k: [m, d] keys at absolute positions 0 .. m-1.  Key j is visible to the query at
    position t iff j <= t; everything else carries -inf before the softmax (Fig. 1(b)).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    n, m = q.shape[0], k.shape[0]
    s = scale * (q @ k.T)
    t = first_pos + np.arange(n).reshape(n, 1)
    j = np.arange(m).reshape(1, m)
    s = np.where(j <= t, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    w = np.exp(s)
    return w / w.sum(axis=1, keepdims=True)


def _kv_head(h: int, n_q_heads: int, n_kv_heads: int) -> int:
    """Query head h reads key/value head floor(h / G), G = n_q_heads / n_kv_heads."""
    if n_q_heads % n_kv_heads:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    return h // (n_q_heads // n_kv_heads)


def causal_attention(q, k, v, scale, rope_base=None):
    """Full-context causal attention of one layer (Fig. 1(b)).

    q: [C, H, d]; k, v: [C, H_kv, d], un-rotated.  With rope_base set, Q and K are
    rotated by their absolute positions 0..C-1 first (V never is).  Returns [C, H, d].
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    C, H, d = q.shape
    Hkv = k.shape[1]
    if rope_base is not None:
        pos = np.arange(C)
        q = rope(q, pos, rope_base)
        k = rope(k, pos, rope_base)
    out = np.empty((C, H, d), dtype=np.float64)
    for h in range(H):
        g = _kv_head(h, H, Hkv)
        w = attention_weights(q[:, h, :], k[:, g, :], scale, first_pos=0)
        out[:, h, :] = w @ v[:, g, :]
    return out


def append_kv(k_cache, v_cache, k, v, prefix_len, rope_base=None, q=None):
    """Cache population of one chunk (App. C listing: cat(cache, local K/V)).

    k_cache, v_cache: [capacity, H_kv, d] fp64 arrays updated in place on rows
    [prefix_len, prefix_len + c); k, v: [c, H_kv, d] un-rotated.  K (and q, if given)
    are rotated by absolute positions prefix_len + r.  Returns the rotated q (or None).
    """
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    c = k.shape[0]
    if prefix_len < 0 or prefix_len + c > k_cache.shape[0]:
        raise ValueError("chunk does not fit the cache")
    pos = prefix_len + np.arange(c)
    if rope_base is not None:
        k = rope(k, pos, rope_base)
        if q is not None:
            q = rope(np.asarray(q, dtype=np.float64), pos, rope_base)
    k_cache[prefix_len:prefix_len + c] = k
    v_cache[prefix_len:prefix_len + c] = v
    return q


def chunk_attention(q, k_cache, v_cache, prefix_len, chunk_len, scale):
    """What one KV-Runahead process computes for its chunk (Sec. 4.1, Fig. 5(b)).

    q: [chunk_len, H, d] already rotated; caches hold rows [0, prefix_len+chunk_len).
    The query at chunk row r sits at absolute position prefix_len + r and sees cache
    rows 0 .. prefix_len + r.  Returns [chunk_len, H, d], the same shape as q.
    """
    q = np.asarray(q, dtype=np.float64)
    c, H, d = q.shape
    if c != chunk_len:
        raise ValueError("q does not match chunk_len")
    total = prefix_len + chunk_len
    Hkv = k_cache.shape[1]
    out = np.empty((c, H, d), dtype=np.float64)
    for h in range(H):
        g = _kv_head(h, H, Hkv)
        w = attention_weights(q[:, h, :], k_cache[:total, g, :], scale, first_pos=prefix_len)
        out[:, h, :] = w @ v_cache[:total, g, :]
    return out


def chunked_prefill(q, k, v, boundaries, scale, rope_base=None):
    """Run the chunks of a partition in order: append, then attend (chain p_0 -> p_1 -> ...).

    boundaries: [0 = b_0 < b_1 < ... < b_p = C].  Returns (out [C,H,d], k_cache, v_cache).
    """
    q = np.asarray(q, dtype=np.float64)
    C, H, d = q.shape
    Hkv = k.shape[1]
    b = [int(x) for x in boundaries]
    if b[0] != 0 or b[-1] != C or any(b[i + 1] <= b[i] for i in range(len(b) - 1)):
        raise ValueError("boundaries must rise strictly from 0 to C")
    k_cache = np.zeros((C, Hkv, d), dtype=np.float64)
    v_cache = np.zeros((C, Hkv, d), dtype=np.float64)
    out = np.empty((C, H, d), dtype=np.float64)
    for i in range(len(b) - 1):
        lo, hi = b[i], b[i + 1]
        qc = append_kv(k_cache, v_cache, k[lo:hi], v[lo:hi], lo, rope_base, q=q[lo:hi])
        if qc is None:
            qc = q[lo:hi]
        out[lo:hi] = chunk_attention(qc, k_cache, v_cache, lo, hi - lo, scale)
    return out, k_cache, v_cache


def attention_rows(q, k, v, rows, scale, rope_base=None):
    """Full-context causal attention for a list of absolute positions only.

    Same definition as causal_attention, evaluated row by row (each row is independent
    of the others), so that large contexts can be checked on a sample.
    q: [C,H,d], k,v: [C,H_kv,d] un-rotated.  Returns [len(rows), H, d].
    """
    q = np.asarray(q)
    k = np.asarray(k)
    v = np.asarray(v)
    C, H, d = q.shape
    Hkv = k.shape[1]
    rows = [int(r) for r in rows]
    tmax = max(rows) + 1
    kk = np.asarray(k[:tmax], dtype=np.float64)
    vv = np.asarray(v[:tmax], dtype=np.float64)
    if rope_base is not None:
        kk = rope(kk, np.arange(tmax), rope_base)
    out = np.empty((len(rows), H, d), dtype=np.float64)
    for n, t in enumerate(rows):
        qt = np.asarray(q[t:t + 1], dtype=np.float64)
        if rope_base is not None:
            qt = rope(qt, np.array([t]), rope_base)
        for h in range(H):
            g = _kv_head(h, H, Hkv)
            s = scale * (kk[:t + 1, g, :] @ qt[0, h, :])
            s = s - s.max()
            w = np.exp(s)
            w = w / w.sum()
            out[n, h, :] = w @ vv[:t + 1, g, :]
    return out


# --------------------------------------------------------------------------- work / traffic model
def chunk_lengths(boundaries):
    b = [int(x) for x in boundaries]
    return [b[i + 1] - b[i] for i in range(len(b) - 1)]


def rect_dot_products(boundaries):
    """Dot products of Q.K^T each process issues as a dense rectangle: c_i * (prefix_i + c_i)
    (Fig. 5 caption; Sec. 4.1)."""
    b = [int(x) for x in boundaries]
    return [(b[i + 1] - b[i]) * b[i + 1] for i in range(len(b) - 1)]


def tsp_dot_products(context_len, p):
    """Tensor/sequence-parallel baseline: every process multiplies its C/p queries by all
    C keys (Fig. 4 caption)."""
    if context_len % p:
        raise ValueError("even split needs p | C")
    return [(context_len // p) * context_len] * p


def useful_pairs(prefix_len, chunk_len):
    """(query, key) pairs under the causal mask for one chunk, diagonal included."""
    return chunk_len * prefix_len + chunk_len * (chunk_len + 1) // 2


def useful_flops(prefix_len, chunk_len, n_q_heads, head_dim):
    """2d multiply-adds for Q.K^T plus 2d for P.V per visible pair per head."""
    return 4 * head_dim * n_q_heads * useful_pairs(prefix_len, chunk_len)


def kvr_traffic_entries(boundaries):
    """(K,V) rows put on the network by the chain p_0 -> p_1 -> ...: process i forwards its
    whole cache, K rows and V rows counted separately (Fig. 5 caption; Eq. 5-6)."""
    b = [int(x) for x in boundaries]
    return 2 * sum(b[1:-1])


def tsp_traffic_entries(context_len, p):
    """all-gather: every process receives the K and V rows of all others (Fig. 4 caption; Eq. 3-4)."""
    return 2 * (p - 1) * context_len


def ttft_lower_bound_ratio(p):
    """TTFT*(p) / TTFT(1) of Eq. 2."""
    return 0.5 * (1.0 / p + 1.0 / (p * p))


# --------------------------------------------------------------------------- load balancing
def analytic_cost(prefix_len, chunk_len):
    """Twice the area under the diagonal of a chunk's rectangle: c * (2 prefix + c)."""
    return float(chunk_len * (2 * prefix_len + chunk_len))


def makespan(boundaries, cost=analytic_cost):
    """Largest per-chunk cost of a partition: with every chunk on its own worker and many
    layers, the slowest worker sets the pace (Sec. 4.2, second bullet)."""
    b = [int(x) for x in boundaries]
    return max(cost(b[i], b[i + 1] - b[i]) for i in range(len(b) - 1))


def chain_ttft(boundaries, n_layers, before_attn, attn, handoff=None):
    """Time to first token of the chain p_0 -> p_1 -> ... with one process per chunk (Sec. 4
    overview; Fig. 5(b), layer misalignment): in every layer a process first does its own work up
    to the cache append (`before_attn`), can attend only once the cache of its precedent has
    arrived as well (`handoff` after that cache was complete), attends (`attn`) and moves on to
    the next layer.  Written as the event times of every (process, layer), nothing folded."""
    b = [int(x) for x in boundaries]
    p = len(b) - 1
    cache = [[0.0] * n_layers for _ in range(p)]   # own K,V appended and all earlier rows present
    done = [[0.0] * n_layers for _ in range(p)]    # process leaves the layer
    for layer in range(n_layers):
        for i in range(p):
            start = done[i][layer - 1] if layer > 0 else 0.0
            own = start + before_attn(b[i], b[i + 1] - b[i])
            if i > 0:
                sent = handoff(b[i - 1], b[i] - b[i - 1]) if handoff is not None else 0.0
                own = max(own, cache[i - 1][layer] + sent)
            cache[i][layer] = own
            done[i][layer] = own + attn(b[i], b[i + 1] - b[i])
    return done[p - 1][n_layers - 1]


def equal_split(context_len, p, granularity):
    """Even partitioning (KVR-E), boundaries rounded to the granularity grid."""
    g = granularity
    return [g * int(math.floor(k * context_len / (p * g) + 0.5)) for k in range(p + 1)]


def sqrt_rule(context_len, p, granularity):
    """Continuous optimum of the analytic cost, b_k = C sqrt(k/p), rounded to the grid."""
    g = granularity
    return [g * int(math.floor(context_len * math.sqrt(k / p) / g + 0.5)) for k in range(p + 1)]


def brute_force_balance(context_len, p, granularity, cost=analytic_cost):
    """Exhaustive search over all strictly rising boundary tuples on the granularity grid.

    Returns (boundaries, makespan); among equal makespans the lexicographically smallest
    boundary vector is kept.
    """
    if context_len % granularity or context_len < p * granularity:
        raise ValueError("context does not fit the grid")
    n = context_len // granularity
    best, best_b = None, None
    for cut in itertools.combinations(range(1, n), p - 1):
        b = [0] + [granularity * x for x in cut] + [context_len]
        m = makespan(b, cost)
        if best is None or m < best:
            best, best_b = m, b
    return best_b, best


# --------------------------------------------------------------------------- partition search
# Sec. 4.2 describes three off-line tools on top of the makespan objective: a one-dimensional
# search for two processes, a hierarchical grid search for more, and a lookup table whose
# entries are linearly interpolated at inference time.  The paper drives them with measured
# TTFT; here the objective is the makespan of per-chunk costs.  Details the paper leaves open
# (stride schedule, what "zooming in" keeps, rounding of interpolated boundaries) are fixed
# as stated in each docstring.
def two_way_scan(context_len, granularity, cost=analytic_cost):
    """Best split of a context between two processes by trying every grid position of the
    single interior boundary (what the paper's one-dimensional search converges to,
    Sec. 4.2 / Fig. 6(a)).  Ties go to the smaller boundary.  Returns (boundaries, makespan)."""
    g = granularity
    best, best_b = None, None
    for b1 in range(g, context_len, g):
        m = makespan([0, b1, context_len], cost)
        if best is None or m < best:
            best, best_b = m, [0, b1, context_len]
    return best_b, best


def grid_search_strides(context_len, p, granularity):
    """Stride schedule of the hierarchical grid search: the first stride is the largest
    granularity * 2^k with 2 * stride < C / p, then it halves down to the granularity.
    For the paper's example (C = 96, granularity 2, three or four partitions) this gives
    8, 4, 2 as in Fig. 6(b-d)."""
    stride = granularity
    while 2 * (2 * stride) * p < context_len:
        stride *= 2
    out = []
    while stride >= granularity:
        out.append(stride)
        stride //= 2
    return out


def hierarchical_grid_search(context_len, p, granularity, cost=analytic_cost, start=None, objective=None):
    """Hierarchical grid search of Sec. 4.2 (Fig. 6(b-d); cost model in the appendix on lookup
    table generation: five values per interior boundary and level).

    Level by level, every interior boundary is tried at its current value plus
    {-2,-1,0,1,2} * stride, all 5^(p-1) combinations; combinations that are not strictly
    rising inside (0, C) are dropped; the combination with the smallest makespan (ties: the
    lexicographically smallest boundary vector) becomes the centre of the next level, whose
    stride is half as large, so the next level scans exactly +-1 old stride around it.
    Starts from the even split unless `start` is given.  Returns (boundaries, makespan, levels)
    where levels is the list of (stride, centre after the level).  With `objective` (a function
    of the boundary list) that value is minimised instead of the makespan of `cost`: the paper
    searches on the time to first token.
    """
    if objective is None:
        objective = lambda b: makespan(b, cost)
    cur = list(start) if start is not None else equal_split(context_len, p, granularity)
    assert cur[0] == 0 and cur[-1] == context_len and len(cur) == p + 1
    levels = []
    best_m = objective(cur)
    for stride in grid_search_strides(context_len, p, granularity):
        axes = [[cur[k] + o * stride for o in (-2, -1, 0, 1, 2)] for k in range(1, p)]
        best, best_b = None, None
        for inner in itertools.product(*axes):
            b = [0] + list(inner) + [context_len]
            if any(b[i + 1] <= b[i] for i in range(p)):
                continue
            m = objective(b)
            if best is None or m < best or (m == best and b < best_b):
                best, best_b = m, b
        cur, best_m = best_b, best
        levels.append((stride, list(cur)))
    return cur, best_m, levels


def interpolate_partition(context_len, granularity, len_lo, bounds_lo, len_hi, bounds_hi):
    """Predicted partitioning of a context from two lookup-table entries (KVR-P, Sec. 4.2 and
    the partitioning paragraph of Sec. 5): the cumulative boundary RATIOS b_k / C of the two
    entries are blended linearly in the context length, scaled by the new length and rounded
    to the nearest grid point (halves up).  A length outside [len_lo, len_hi] takes the ratios
    of the nearer entry.  Boundaries that collide after rounding are pushed apart by one
    granule, first upwards from the left, then downwards from the right.
    """
    p = len(bounds_lo) - 1
    assert len(bounds_hi) == p + 1
    g = granularity
    if len_hi == len_lo:
        w = 0.0
    else:
        w = (context_len - len_lo) / (len_hi - len_lo)
        w = min(1.0, max(0.0, w))
    b = [0] * (p + 1)
    for k in range(1, p):
        r = (1.0 - w) * (bounds_lo[k] / len_lo) + w * (bounds_hi[k] / len_hi)
        b[k] = g * int(math.floor(r * context_len / g + 0.5))
    b[p] = context_len
    for k in range(1, p):
        if b[k] < b[k - 1] + g:
            b[k] = b[k - 1] + g
    for k in range(p - 1, 0, -1):
        if b[k] > b[k + 1] - g:
            b[k] = b[k + 1] - g
    return b


def lookup_partition(context_len, granularity, table):
    """Prediction from a lookup table {context length: boundaries} (Fig. 3(b)): blend the two
    entries that bracket the length; below the smallest or above the largest entry the
    nearest entry's ratios are used."""
    lens = sorted(table)
    lo = max([x for x in lens if x <= context_len], default=lens[0])
    hi = min([x for x in lens if x >= context_len], default=lens[-1])
    return interpolate_partition(context_len, granularity, lo, table[lo], hi, table[hi])


# --------------------------------------------------------------------------- decoder layer
# What one KV-Runahead process runs per layer around the attention block (Sec. 4.1: every process
# runs each layer on its own chunk; App. C listing: q/k/v projections before, output projection
# after the attention).  The paper does not write out the normalisation and the MLP; they are
# taken from the LLaMA architecture of the models in Sec. 5: pre-norm RMSNorm, no biases,
# SwiGLU MLP, two residual connections.
def _no_rounding(t):
    return t


def round_to_bf16(t):
    """fp64 -> nearest bf16 (ties to even) -> fp64; the storage rounding of a bf16 tensor."""
    return bf16_bits_to_f64(f64_to_bf16_bits(t))


def rms_norm(x, gain, eps):
    """y[t, :] = x[t, :] / sqrt(mean_j x[t, j]^2 + eps) * gain."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def linear(x, w):
    """y = x w^T for a weight stored [out_features, in_features]; no bias."""
    return x @ w.T


def silu(x):
    return x / (1.0 + np.exp(-x))


def swiglu_mlp(x, w_gate, w_up, w_down, rnd=_no_rounding):
    act = rnd(silu(linear(x, w_gate)) * linear(x, w_up))
    return linear(act, w_down)


def decoder_layer(x, weights, n_q_heads, n_kv_heads, head_dim, scale, rope_base, eps,
                  boundaries=None, rnd=_no_rounding, trace=None):
    """One pre-norm decoder layer over a whole context x [C, hidden] (fp64).

    weights: dict with 'norm1', 'norm2' [hidden]; 'wq' [H d, hidden]; 'wk', 'wv' [H_kv d, hidden];
    'wo' [hidden, H d]; 'w_gate', 'w_up' [ffn, hidden]; 'w_down' [hidden, ffn].
    boundaries: None runs the context in one piece; a partition runs chunk after chunk through the
    KV-cache (the result is the same: rows of a chunk depend on earlier rows only through K and V).
    rnd: applied wherever a tensor is stored between two operations; the identity gives the exact
    layer, round_to_bf16 models bf16 storage of every intermediate.
    trace: an optional dict that receives the intermediate 'x2' [C, hidden] (input plus attention
    branch), which tests need to scale their error bounds.
    Returns (y [C, hidden], k_cache, v_cache).
    """
    C, hidden = x.shape
    H, Hkv, d = n_q_heads, n_kv_heads, head_dim
    bounds = [0, C] if boundaries is None else [int(b) for b in boundaries]
    k_cache = np.zeros((C, Hkv, d))
    v_cache = np.zeros((C, Hkv, d))
    y = np.zeros_like(x)
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        xc = x[lo:hi]
        h1 = rnd(rms_norm(xc, weights["norm1"], eps))
        q = rnd(linear(h1, weights["wq"])).reshape(hi - lo, H, d)
        k = rnd(linear(h1, weights["wk"])).reshape(hi - lo, Hkv, d)
        v = rnd(linear(h1, weights["wv"])).reshape(hi - lo, Hkv, d)
        pos = np.arange(lo, hi)
        if rope_base is not None:
            q = rnd(rope(q, pos, rope_base))
            k = rnd(rope(k, pos, rope_base))
        k_cache[lo:hi] = k
        v_cache[lo:hi] = v
        a = rnd(chunk_attention(q, k_cache, v_cache, lo, hi - lo, scale))
        x2 = rnd(xc + linear(a.reshape(hi - lo, H * d), weights["wo"]))
        if trace is not None:
            trace.setdefault("x2", np.zeros_like(x))[lo:hi] = x2
        h2 = rnd(rms_norm(x2, weights["norm2"], eps))
        y[lo:hi] = rnd(x2 + swiglu_mlp(h2, weights["w_gate"], weights["w_up"], weights["w_down"], rnd))
    return y, k_cache, v_cache


def layer_kv_cache(x, weights, n_kv_heads, head_dim, rope_base, eps, rnd=_no_rounding):
    """K (rotated) and V of every token of the context x [C, hidden]: what the rows of later chunks see of
    earlier ones (App. C listing: the cache each process hands on).  Returns (k [C, H_kv, d], v)."""
    C = x.shape[0]
    h1 = rnd(rms_norm(x, weights["norm1"], eps))
    k = rnd(linear(h1, weights["wk"])).reshape(C, n_kv_heads, head_dim)
    v = rnd(linear(h1, weights["wv"])).reshape(C, n_kv_heads, head_dim)
    if rope_base is not None:
        k = rnd(rope(k, np.arange(C), rope_base))
    return k, v


def decoder_layer_rows(x, weights, n_q_heads, n_kv_heads, head_dim, scale, rope_base, eps, rows,
                       rnd=_no_rounding, cache=None):
    """Rows `rows` (absolute positions) of decoder_layer's output, evaluated one row at a time so that a long
    context can be checked on a sample: a row depends on earlier rows only through their K and V.

    cache: (k, v) from layer_kv_cache, or None to compute it here (with the same rnd).  Everything after
    the cache - query projection, rotation, attention over keys 0..t, output projection, residual, norm,
    SwiGLU MLP, residual - is done for the requested rows only, same steps as decoder_layer.
    Returns (y [len(rows), hidden], x2 [len(rows), hidden])."""
    H, Hkv, d = n_q_heads, n_kv_heads, head_dim
    rows = [int(r) for r in rows]
    tmax = max(rows) + 1
    k, v = cache if cache is not None else layer_kv_cache(x[:tmax], weights, Hkv, d, rope_base, eps, rnd)
    y = np.empty((len(rows), x.shape[1]))
    x2s = np.empty_like(y)
    for n, t in enumerate(rows):
        xt = x[t:t + 1]
        h1 = rnd(rms_norm(xt, weights["norm1"], eps))
        q = rnd(linear(h1, weights["wq"])).reshape(1, H, d)
        if rope_base is not None:
            q = rnd(rope(q, np.array([t]), rope_base))
        a = np.empty((1, H, d))
        for h in range(H):
            g = _kv_head(h, H, Hkv)
            s = scale * (k[:t + 1, g, :] @ q[0, h, :])
            w = np.exp(s - s.max())
            a[0, h, :] = (w / w.sum()) @ v[:t + 1, g, :]
        a = rnd(a)
        x2 = rnd(xt + linear(a.reshape(1, H * d), weights["wo"]))
        h2 = rnd(rms_norm(x2, weights["norm2"], eps))
        y[n] = rnd(x2 + swiglu_mlp(h2, weights["w_gate"], weights["w_up"], weights["w_down"], rnd))[0]
        x2s[n] = x2[0]
    return y, x2s

