#!/usr/bin/env python3
"""Benchmark of the KV-Runahead per-chunk hot path on one MI355X.

One step = one pass of the whole path over the 16k-token Llama-7B-shape workload: for each of the
8 balanced chunks, kvra_append_kv (RoPE on K and Q, K/V into the cache) then kvra_chunk_attn, as
successive launches on one stream.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line: useful causal-attention TFLOP/s over the whole step, the roofline of the
dominant kernel (chunk attention, bf16 MFMA) from HIP-event timings taken inside the timed steps,
and the fp64 CPU oracle timed on a bounded sample as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBPS = 8000.0         # MI355X HBM3E, published
WORKLOAD = "llama7b_16k_balanced"

# HBM bytes per kvra_chunk_attn call (mean over the calls of a step) from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this file, scaled by what the same counters read for a plain copy of known size.
# A measured constant, not a live reading: `source` names the tracked summary it was copied from and the
# commit whose kernel that run profiled.
ATTN_TRAFFIC = {
    "llama7b_16k_balanced": {"bytes": 3.18e8,
                             "source": "profiles/chunk_attn_append_llama7b_16k_balanced.md: FETCH_SIZE 265.8 MiB + WRITE_SIZE "
                                       "37.4 MiB per call (persistent kernel, merge inside, tails of chunks 3-7 run in gangs, "
                                       "the merging piece of a cut unit stores no partial result of its own); above the "
                                       "algorithmic bytes because the pieces of the leftover units of chunks 0 and 1, and a "
                                       "fourth of the tails of chunks 3 and 4, read the K/V of their head at other times than "
                                       "its other row tiles (L2 hit rate 76 %); 1.3 TB/s at this launch time, a sixth of the "
                                       "HBM peak, so not what bounds the kernel"},
}


def useful_flops(prefix, c, H, d):
    return 4 * d * H * (c * prefix + c * (c + 1) // 2)


def cpu_baseline(cfg, sample_heads=8):
    """Times the oracle, as it stands, on a bounded sample: full 16k context, first `sample_heads`
    query heads (and their kv heads)."""
    from oracle import kvra_oracle as orc
    from paper_2405_05329_amd import synth
    C, H, Hkv, d = cfg["C"], cfg["H"], cfg["Hkv"], cfg["d"]
    q, k, v = synth.make_qkv(0, cfg["cfg_id"], C, H, Hkv, d)
    G = H // Hkv
    hs = sample_heads
    kv = max(1, hs // G)
    qf = orc.bf16_bits_to_f64(q[:, :hs])
    kf = orc.bf16_bits_to_f64(k[:, :kv])
    vf = orc.bf16_bits_to_f64(v[:, :kv])
    t0 = time.perf_counter()
    orc.causal_attention(qf, kf, vf, synth.default_scale(d), rope_base=synth.ROPE_BASE)
    dt = time.perf_counter() - t0
    flops = useful_flops(0, C, hs, d)
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle.causal_attention (fp64 numpy) on {hs} of {H} query heads over the full "
                      f"{C}-token context, {dt:.1f} s",
            "seconds": dt}


def layer_bench(args):
    """--layer: one step = the decoder layer (kvra_layer_chunk: RMSNorm, q/k/v projections, append,
    attention, output projection, RMSNorm, SwiGLU MLP) over the 8 balanced chunks of the 32k-token
    Llama-7B shape.  Not the headline metric; printed in the same one-line form."""
    import torch
    from paper_2405_05329_amd import kvra, synth

    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    shp = synth.LAYER_SHAPES["llama7b"]
    C, H, Hkv, d = cfg["C"], cfg["H"], cfg["Hkv"], cfg["d"]
    assert (H, Hkv, d) == (shp["H"], shp["Hkv"], shp["d"]), "layer bench needs a Llama-7B-shaped workload"
    hidden, ffn = shp["hidden"], shp["ffn"]
    bounds = cfg["boundaries"]
    p = len(bounds) - 1
    scale = synth.default_scale(d)

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    wt = {k: dev(v) for k, v in synth.make_layer_weights(0, cfg["cfg_id"], hidden, ffn, H, Hkv, d,
                                                         shp["weight_std"]).items()}
    layer = kvra.make_layer(hidden, ffn, H, Hkv, d, synth.RMS_EPS, synth.ROPE_BASE, scale, wt["norm1"], wt["wqkv"],
                            wt["wo"], wt["norm2"], wt["w_gate"], wt["w_up"], wt["w_down"])
    x = dev(synth.normal_bf16(0, cfg["cfg_id"], 0, (C, hidden)))
    y = torch.empty_like(x)
    k_cache = torch.zeros((C, Hkv, d), dtype=torch.bfloat16, device="cuda")
    v_cache = torch.zeros_like(k_cache)
    cmax = max(bounds[i + 1] - bounds[i] for i in range(p))
    nbytes = kvra.kvra_layer_workspace_bytes(layer, cmax)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    def run_step(events=None):
        for i in range(p):
            lo, hi = bounds[i], bounds[i + 1]
            if events is not None:
                events[i][0].record(stream)
            kvra.kvra_layer_chunk(layer, x[lo:hi], y[lo:hi], k_cache, v_cache, lo, hi - lo, C, ws, nbytes,
                                  stream=stream)
            if events is not None:
                events[i][1].record(stream)

    for _ in range(args.warmup):
        run_step()
    ev = [[[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(p)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        run_step(ev[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    chunk_ms = np.array([[e[0].elapsed_time(e[1]) for e in step] for step in ev]).mean(axis=0)
    qkv_rows = (H + 2 * Hkv) * d
    lin_per_token = 2 * (hidden * qkv_rows + hidden * H * d + 3 * hidden * ffn)
    attn_flops = [useful_flops(bounds[i], bounds[i + 1] - bounds[i], H, d) for i in range(p)]
    lin_flops = [lin_per_token * (bounds[i + 1] - bounds[i]) for i in range(p)]
    total = sum(attn_flops) + sum(lin_flops)

    # per-operator times of the first chunk, same launches issued one by one
    lo, hi = bounds[0], bounds[1]
    c = hi - lo
    h = torch.empty((c, hidden), dtype=torch.bfloat16, device="cuda")
    q = torch.empty((c, H, d), dtype=torch.bfloat16, device="cuda")
    kk = torch.empty((c, Hkv, d), dtype=torch.bfloat16, device="cuda")
    vv = torch.empty_like(kk)
    att = torch.empty_like(q)
    x2 = torch.empty_like(h)
    act = torch.empty((c, ffn), dtype=torch.bfloat16, device="cuda")
    ops = [
        ("rms_norm", lambda: kvra.kvra_rms_norm(x[lo:hi], wt["norm1"], h, c, hidden, synth.RMS_EPS), 0),
        ("qkv_proj", lambda: kvra.kvra_qkv_proj(h, wt["wqkv"], q, kk, vv, c, H, Hkv, d, hidden), 2 * c * hidden * qkv_rows),
        ("append_kv", lambda: kvra.kvra_append_kv(kk, vv, q, k_cache, v_cache, lo, c, C, H, Hkv, d, synth.ROPE_BASE), 0),
        ("chunk_attn", lambda: kvra.kvra_chunk_attn(q, k_cache, v_cache, lo, c, H, Hkv, d, scale, att), attn_flops[0]),
        ("out_proj+res", lambda: kvra.kvra_linear(att, wt["wo"], None, x[lo:hi], x2, c, hidden, H * d), 2 * c * hidden * H * d),
        ("gate_up+swiglu", lambda: kvra.kvra_linear(h, wt["w_gate"], wt["w_up"], None, act, c, ffn, hidden), 4 * c * hidden * ffn),
        ("down_proj+res", lambda: kvra.kvra_linear(act, wt["w_down"], None, x2, y[lo:hi], c, hidden, ffn), 2 * c * hidden * ffn),
    ]
    breakdown = {}
    lin_ms, lin_fl = 0.0, 0
    for name, fn, fl in ops:
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(5):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        breakdown[name] = {"ms": round(ms, 4), "tflops": round(fl / ms / 1e9, 1) if fl else None}
        if name in ("qkv_proj", "out_proj+res", "gate_up+swiglu", "down_proj+res"):
            lin_ms += ms
            lin_fl += fl
    achieved = lin_fl / lin_ms / 1e9

    # context-level load balancing with the whole layer as the cost (Sec. 4.2): fit
    # t = a + b c + e c (2 prefix + c) to measured layer times and let kvra_balance cut the context
    makespan = {"attention_balanced_ms": float(chunk_ms.max())}
    if not args.no_extras:
        def layer_ms(prefix, c, reps=3):
            # back to back, as in a step: a launch timed alone, with the chip idle before it, runs at other clocks
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for rep in range(reps + 1):
                if rep:
                    evs[rep - 1][0].record(stream)
                kvra.kvra_layer_chunk(layer, x[prefix:prefix + c], y[prefix:prefix + c], k_cache, v_cache, prefix, c, C,
                                      ws, nbytes, stream=stream)
                if rep:
                    evs[rep - 1][1].record(stream)
            torch.cuda.synchronize()
            return float(np.mean([e0.elapsed_time(e1) for e0, e1 in evs]))
        table = {}
        for pr in (0, 8192, 16384, 24576, 30720):
            for c in (512, 1024, 2048, 4096, 8192, cmax):
                if pr + c <= C:
                    table[(pr, c)] = layer_ms(pr, c)
        A = np.array([[1.0, c, c * (2 * pr + c)] for (pr, c) in table])
        coef, *_ = np.linalg.lstsq(A, np.array(list(table.values())), rcond=None)
        model = lambda prefix, c: float(coef[0] + coef[1] * c + coef[2] * c * (2 * prefix + c))

        def measured_chunks(bnds):
            """Mean per-chunk layer time (ms) of a partition: one untimed pass, then three timed ones, every pass
            the chunks back to back with events around each kvra_layer_chunk call."""
            n = len(bnds) - 1
            acc = np.zeros(n)
            for rep in range(4):
                evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
                for i in range(n):
                    lo_, hi_ = bnds[i], bnds[i + 1]
                    evs[i][0].record(stream)
                    kvra.kvra_layer_chunk(layer, x[lo_:hi_], y[lo_:hi_], k_cache, v_cache, lo_, hi_ - lo_, C, ws, nbytes,
                                          stream=stream)
                    evs[i][1].record(stream)
                torch.cuda.synchronize()
                if rep:
                    acc += np.array([e0.elapsed_time(e1) for e0, e1 in evs])
            return acc / 3

        # the search refined on measurements of its own candidates, as in the attention-only bench: the ratio
        # measured / model of every chunk that was run corrects the model around it
        seen = []
        w_prefix, w_chunk = C / 16.0, C / 64.0

        def cost(prefix, c):
            if c > cmax:
                return 1e9               # the workspace of this run holds chunks up to the workload's longest
            t = model(prefix, c)
            if seen:
                pts = np.array(seen)
                w = np.exp(-(((pts[:, 0] - prefix) / w_prefix) ** 2 + ((pts[:, 1] - c) / w_chunk) ** 2))
                sw = float(w.sum())
                if sw > 1e-6:
                    t *= 1.0 + float(np.dot(w, pts[:, 2] - 1.0)) / max(sw, 1.0)
            return t

        history, best = [], None
        for it in range(5):
            bal, pred = kvra.kvra_balance(C, p, 64, cost)
            tot = measured_chunks(bal)
            history.append({"boundaries": bal, "predicted_ms": round(pred, 4), "measured_ms": round(float(tot.max()), 4)})
            if best is None or tot.max() < best[1]:
                best = (bal, float(tot.max()))
            for i in range(p):
                seen.append((bal[i], bal[i + 1] - bal[i], float(tot[i]) / model(bal[i], bal[i + 1] - bal[i])))
            if it >= 1 and abs(pred - tot.max()) <= 0.03 * tot.max():
                break
        bal = best[0]
        pred = max(cost(bal[i], bal[i + 1] - bal[i]) for i in range(p))
        bal_ms = float(measured_chunks(bal).max())
        eq = kvra.kvra_equal_split(C, p, 64)
        makespan.update({
            "cost_fit_ms": {"const": float(coef[0]), "per_token": float(coef[1]), "per_causal_area": float(coef[2])},
            "search": history,
            "layer_balanced_boundaries": bal, "layer_balanced_predicted_ms": pred,
            "layer_balanced_measured_ms": bal_ms,
            "prediction_error": abs(pred - bal_ms) / bal_ms,
            "model_only_prediction_error": abs(history[0]["predicted_ms"] - history[0]["measured_ms"]) / history[0]["measured_ms"],
            "attention_balanced_measured_ms": float(measured_chunks(bounds).max()),
            "equal_split_measured_ms": float(measured_chunks(eq).max()),
            "layer_balanced_first_chunk_share": bal[1] / C, "attention_balanced_first_chunk_share": bounds[1] / C,
        })
    result = {
        "metric": "decoder-layer TFLOP/s (useful FLOPs: causal attention + linear layers), chunked prefill",
        "value": total / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload + "+layer", "context_len": C, "hidden": hidden, "ffn": ffn,
                   "n_q_heads": H, "n_kv_heads": Hkv, "head_dim": d, "chunks": p, "boundaries": bounds,
                   "useful_gflop_per_step": total / 1e9},
        "pct_of_bf16_peak": 100.0 * total / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "roofline": {"kernel": "linear_kernel", "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None,
                     "note": "the four linear launches of chunk 0, algorithmic FLOPs / summed launch time"},
        "per_chunk": {"layer_ms": [round(float(v), 4) for v in chunk_ms],
                      "layer_tflops": [round((attn_flops[i] + lin_flops[i]) / chunk_ms[i] / 1e9, 1) for i in range(p)]},
        "chunk0_breakdown": breakdown,
        "makespan": makespan,
        "cpu_baseline": None,
    }
    print(json.dumps(result))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--event-every", type=int, default=4,
                    help="every how many timed steps carry the HIP events that time the kernels (1 = every step)")
    ap.add_argument("--no-makespan", action="store_true",
                    help="skip the equal-split and kvra_balance makespan measurements and the matrix-pipe probe "
                         "(profiling runs: only the workload's own kernels are launched)")
    ap.add_argument("--no-extras", action="store_true", help="same as --no-makespan (kept for older command lines)")
    ap.add_argument("--extras", action="store_true",
                    help="also: HIP-graph replay of the step, the chain-of-processes TTFT, the paper's grid search "
                         "and lookup-table prediction on the measured cost model (tens of seconds of host time)")
    ap.add_argument("--workload", default=WORKLOAD,
                    help="a key of synth.CONFIGS; the default is the workload the metric is quoted on")
    ap.add_argument("--layer", action="store_true",
                    help="time the whole decoder layer per chunk (use with --workload llama7b_32k_balanced)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also issue one plain 256 MiB device-to-device copy (outside the timed region) so "
                         "that a rocprofv3 --pmc run holds a dispatch of known traffic to scale counters by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures the single-GPU hot path only; run with --gpus 1 "
              "(no multi-GPU figure exists for it)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2405_05329_amd import kvra, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    if args.layer:
        layer_bench(args)
        return
    torch.cuda.set_device(0)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    cfg = synth.CONFIGS[args.workload]
    C, H, Hkv, d = cfg["C"], cfg["H"], cfg["Hkv"], cfg["d"]
    bounds = cfg["boundaries"]
    p = len(bounds) - 1
    scale = synth.default_scale(d)

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    qb, kb, vb = synth.make_qkv(0, cfg["cfg_id"], C, H, Hkv, d)
    q_master, k_in, v_in = dev(qb), dev(kb), dev(vb)
    del qb, kb, vb
    n_buf = min(args.steps + args.warmup, 24)
    # Q is rotated in place, so steps take turns on n_buf copies; a copy that comes round again is
    # rotated once more (same work; a rotation keeps the magnitudes, so the softmax load is unchanged)
    q_work = [q_master.clone() for _ in range(n_buf)]
    k_cache = torch.zeros((C, Hkv, d), dtype=torch.bfloat16, device="cuda")
    v_cache = torch.zeros((C, Hkv, d), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((C, H, d), dtype=torch.bfloat16, device="cuda")
    stream = torch.cuda.current_stream()

    # Two events per chunk, around the attention call (every event costs about 3.5 us of stream time, so none
    # is spent on the append: its time is the stretch from the previous chunk's end event to this chunk's
    # start event, and a chunk's time - append + attention - runs from end event to end event).
    def run_step(bnds, qw, events=None, stream=stream):
        for i in range(len(bnds) - 1):
            lo, hi = bnds[i], bnds[i + 1]
            kvra.kvra_append_kv(k_in[lo:hi], v_in[lo:hi], qw[lo:hi], k_cache, v_cache, lo, hi - lo, C,
                                H, Hkv, d, synth.ROPE_BASE, stream=stream)
            if events is not None:
                events[i][0].record(stream)
            kvra.kvra_chunk_attn(qw[lo:hi], k_cache, v_cache, lo, hi - lo, H, Hkv, d, scale, out[lo:hi],
                                 stream=stream)
            if events is not None:
                events[i][1].record(stream)

    def new_events(n):
        return [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n)]

    def chunk_times(first, passes):
        """(append ms, attention ms) per pass and chunk from the events of consecutive passes; `first` is the
        event recorded just before the first pass."""
        app, att = [], []
        prev = first
        for e in passes:
            a_row, t_row = [], []
            for pair in e:
                a_row.append(prev.elapsed_time(pair[0]))
                t_row.append(pair[0].elapsed_time(pair[1]))
                prev = pair[1]
            app.append(a_row)
            att.append(t_row)
        return np.array(app), np.array(att)

    if args.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.fill_(1)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for s in range(args.warmup):
        run_step(bounds, q_work[s % n_buf])
    torch.cuda.synchronize()
    for s in range(args.warmup, args.warmup + args.steps):   # restore un-rotated Q where a buffer is reused
        if s >= n_buf:
            q_work[s % n_buf].copy_(q_master)
    # Every event costs stream time that is no part of the workload (2 p + 1 events per step would be 2-3 % of it),
    # so only every args.event_every-th timed step carries them: one before its first append, two per chunk.
    every = max(1, args.event_every)
    ev = {s: (torch.cuda.Event(enable_timing=True), new_events(p))     # counted from the last step backwards
          for s in range(args.steps) if (args.steps - 1 - s) % every == 0}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        if s in ev:
            ev[s][0].record(stream)
            run_step(bounds, q_work[(args.warmup + s) % n_buf], ev[s][1])
        else:
            run_step(bounds, q_work[(args.warmup + s) % n_buf])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_per_step = wall * 1e3 / args.steps
    flops_chunk = [useful_flops(bounds[i], bounds[i + 1] - bounds[i], H, d) for i in range(p)]
    flops_step = sum(flops_chunk)
    per_step = [chunk_times(first, [pairs]) for first, pairs in ev.values()]
    append_ms = np.concatenate([a for a, _ in per_step])   # [steps with events, p]
    attn_ms = np.concatenate([t for _, t in per_step])
    attn_mean = attn_ms.mean(axis=0)
    append_mean = append_ms.mean(axis=0)
    attn_avg_launch_ms = float(attn_ms.mean())
    achieved = (flops_step / p) / (attn_avg_launch_ms * 1e-3) / 1e12
    append_bytes = [8 * (bounds[i + 1] - bounds[i]) * Hkv * d + 4 * (bounds[i + 1] - bounds[i]) * H * d for i in range(p)]
    append_gbps = float(sum(append_bytes) / (append_mean.sum() * 1e-3) / 1e9)
    algorithmic_bytes = float(np.mean([4 * (bounds[i + 1] - bounds[i]) * H * d + 4 * bounds[i + 1] * Hkv * d for i in range(p)]))
    traffic = ATTN_TRAFFIC.get(args.workload)

    result = {
        "metric": "chunked causal-attn TFLOP/s (useful FLOPs, % bf16 MFMA peak); balanced makespan",
        "value": flops_step / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "context_len": C, "n_q_heads": H, "n_kv_heads": Hkv, "head_dim": d,
                   "chunks": p, "boundaries": bounds, "useful_gflop_per_step": flops_step / 1e9},
        "pct_of_bf16_peak": 100.0 * flops_step / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "roofline": {"kernel": "chunk_attn_kernel", "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "traffic": traffic["bytes"] if traffic else None,
                     "traffic_source": traffic["source"] if traffic else None,
                     "algorithmic_bytes": algorithmic_bytes,
                     "traffic_over_algorithmic": traffic["bytes"] / algorithmic_bytes if traffic else None,
                     "avg_launch_ms": attn_avg_launch_ms,
                     "timing": f"HIP events on the launch stream around every kvra_chunk_attn call of every "
                               f"{every}. timed step ({len(ev)} of {args.steps} steps, {len(ev) * p} launches); the append "
                               "is timed from the previous event to the call's start event"},
        "per_chunk": {"attn_ms": [round(float(x), 4) for x in attn_mean],
                      "attn_ms_median": [round(float(x), 4) for x in np.median(attn_ms, axis=0)],
                      "attn_ms_min": [round(float(x), 4) for x in attn_ms.min(axis=0)],
                      "append_ms": [round(float(x), 4) for x in append_mean],
                      "attn_tflops": [round(flops_chunk[i] / (attn_mean[i] * 1e-3) / 1e12, 1) for i in range(p)]},
        "append_kv": {"bound": "hbm", "achieved": append_gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                      "frac": append_gbps / PEAK_HBM_GBPS},
        "makespan": {"balanced_ms": float((attn_mean + append_mean).max())},
        "paper_context": "KV-Runahead reports 1.4x (Llama 7B) / 1.6x (Falcon 7B) TTFT speedup over tensor/sequence "
                         "parallelism on 8x A100, FP16, 300 GB/s (whole model; not comparable to this kernel metric)",
    }

    # What the matrix pipes of THIS GPU sustain with nothing else in the way (a loop of MFMAs on register operands
    # of the workload's value distribution, all compute units busy, right after the timed steps): GPUs of one model
    # differ by several per cent in the clock they hold under that load, and the attention kernel follows it.
    try:
        if args.no_makespan or args.no_extras:
            raise RuntimeError("left out of profiling runs (--no-makespan)")
        from paper_2405_05329_amd import probe
        alone = probe.matrix_pipes_alone(torch)
        alone["achieved_over_it"] = achieved / alone["tflops"]
        alone["what"] = ("v_mfma_f32_32x32x16_bf16 back to back on register operands, no memory or LDS access in the "
                         "loop, measured in this process after the timed steps; context for frac, which stays "
                         "against the published peak")
        result["roofline"]["matrix_pipes_alone"] = alone
    except (RuntimeError, OSError) as e:
        result["roofline"]["matrix_pipes_alone"] = None
        print(f"bench.py: matrix-pipe probe skipped: {e}", file=sys.stderr)

    reps = 5

    def measured_chunks(bnds):
        """Mean per-chunk (append ms, append + attention ms) of a partition over `reps` passes."""
        n = len(bnds) - 1
        # untimed passes first: after host-side work (the search) the GPU has been idle, and the first
        # milliseconds of work after an idle period run at lower clocks (15 % slower launches measured)
        for rep in range(8):
            run_step(bnds, q_work[rep % n_buf])
        for rep in range(reps):
            q_work[rep % n_buf].copy_(q_master)
        first = torch.cuda.Event(enable_timing=True)
        passes = [new_events(n) for _ in range(reps)]
        first.record(stream)
        for rep in range(reps):
            run_step(bnds, q_work[rep % n_buf], passes[rep])
        torch.cuda.synchronize()
        a_ms, t_ms = chunk_times(first, passes)
        app, tot = a_ms.sum(axis=0), (a_ms + t_ms).sum(axis=0)
        return app / reps, tot / reps

    if not (args.no_makespan or args.no_extras):
        # ---- equal-split comparator (KVR-E) ----------------------------------------------------------
        eq = kvra.kvra_equal_split(C, p, 64)
        eq_append, eq_total = measured_chunks(eq)
        result["makespan"]["equal_split_ms"] = float(eq_total.max())
        result["makespan"]["equal_split_boundaries"] = eq

        # ---- kvra_balance on a cost measured on this GPU (Sec. 4.2: the search runs on measured times) ----
        # Times of append + attention on a grid of (prefix, chunk) pairs; between grid points the cost follows
        # the launch plan, which knows what the grid cannot show: the row-tile count jumps with the chunk
        # length (a 1088-token chunk needs five row tiles per head, a 1024-token one four), and the schedule
        # gives every compute unit plan.steps_per_slot tile steps.  Model, fitted by least squares:
        #   t = a0 + steps_per_slot * (a1 + a2 * rows_per_tile / 256) + a3 * chunk
        qw = q_work[0]

        def measure(prefix, c):
            # back to back, as in a step: a launch timed alone, with the chip idle before and after it, runs
            # at higher clocks than the same launch in a stream of work (10 - 20 % on these boxes)
            # (and with the same two events per pair of launches as the makespan measurement has)
            n_rep = 6
            evs = new_events(n_rep + 1)
            for rep in range(n_rep + 2):
                kvra.kvra_append_kv(k_in[prefix:prefix + c], v_in[prefix:prefix + c], qw[prefix:prefix + c], k_cache,
                                    v_cache, prefix, c, C, H, Hkv, d, synth.ROPE_BASE, stream=stream)
                if rep >= 1:
                    evs[rep - 1][0].record(stream)
                kvra.kvra_chunk_attn(qw[prefix:prefix + c], k_cache, v_cache, prefix, c, H, Hkv, d, scale,
                                     out[prefix:prefix + c], stream=stream)
                if rep >= 1:
                    evs[rep - 1][1].record(stream)
            torch.cuda.synchronize()
            # end event to end event: one append + one attention, as a chunk of a step is timed
            return float(np.mean([evs[j][1].elapsed_time(evs[j + 1][1]) for j in range(n_rep)]))

        def features(prefix, c):
            pl = kvra.kvra_chunk_attn_plan(prefix, c, H, Hkv, d, cus)
            return [1.0, pl["steps_per_slot"], pl["steps_per_slot"] * pl["rows_per_tile"] / 256.0, float(c)]

        step_c = max(64, C // 256 * 8)
        cs = sorted({step_c * k for k in (1, 2, 3, 4, 6, 8, 12, 16, 24)} | {C // 16 + 64, C // 8 - 192, C // 4 + 256, C // 3})
        ps = [C * k // 8 for k in range(8)]
        table = {(pr, c): measure(pr, c) for pr in ps for c in cs if pr + c <= C and c >= 64}
        A = np.array([features(pr, c) for (pr, c) in table])
        y = np.array(list(table.values()))
        # the fit serves a search whose answer has every chunk near (step time / p): points near that time
        # weigh most, tiny and huge launches little
        t_star = ms_per_step / p
        wt = np.exp(-((y - t_star) / (0.5 * t_star)) ** 2) + 0.02
        coef, *_ = np.linalg.lstsq(A * wt[:, None], y * wt, rcond=None)
        resid = np.abs(A @ coef - y) / y
        near = np.abs(y - t_star) <= 0.5 * t_star

        feat_cache = {}

        def model(prefix, c):
            f = feat_cache.get((prefix, c))
            if f is None:
                f = feat_cache[(prefix, c)] = np.array(features(prefix, c))
            return float(np.dot(coef, f))

        # The fit is smooth where the kernel's time is not (the row-tile size and the cut of the schedule change
        # with the shape), so the search is refined on measurements of its own candidates, as the paper's
        # search is: every candidate partition is run, the ratio measured / model of each of its chunks is kept,
        # and the cost near a measured point is the model times that ratio (Gaussian weights, widths C/16 in
        # the prefix and C/64 in the chunk length; far from every measured point the model stands alone).
        seen = []            # (prefix, chunk, measured / model)
        w_prefix, w_chunk = C / 16.0, C / 64.0

        def cost(prefix, c):
            t = model(prefix, c)
            if seen:
                pts = np.array(seen)
                w = np.exp(-(((pts[:, 0] - prefix) / w_prefix) ** 2 + ((pts[:, 1] - c) / w_chunk) ** 2))
                s = float(w.sum())
                if s > 1e-6:
                    t *= 1.0 + float(np.dot(w, pts[:, 2] - 1.0)) / max(s, 1.0)
            return t

        history, best = [], None
        host_ms = 0.0
        for it in range(6):
            t0 = time.perf_counter()
            bal, mk = kvra.kvra_balance(C, p, 64, cost)
            host_ms += (time.perf_counter() - t0) * 1e3
            _, tot = measured_chunks(bal)
            history.append({"boundaries": bal, "predicted_ms": round(mk, 4), "measured_ms": round(float(tot.max()), 4)})
            if best is None or tot.max() < best[1]:
                best = (bal, float(tot.max()))
            for i in range(p):
                seen.append((bal[i], bal[i + 1] - bal[i], float(tot[i]) / model(bal[i], bal[i + 1] - bal[i])))
            if it >= 1 and abs(mk - tot.max()) <= 0.03 * tot.max():
                break
        bal = best[0]
        # fresh measurements of the kept candidate and of the workload's own boundaries, after the search ended
        _, bal_total = measured_chunks(bal)
        _, ref_total = measured_chunks(bounds)
        mk = max(cost(bal[i], bal[i + 1] - bal[i]) for i in range(p))
        result["makespan"]["kvra_balance"] = {
            "cost_model": "t = a0 + steps_per_slot * (a1 + a2 * rows_per_tile / 256) + a3 * chunk, fitted to "
                          f"{len(table)} measured (prefix, chunk) points (steps_per_slot and rows_per_tile from "
                          "kvra_chunk_attn_plan), times the measured / model ratio of the candidates the search has "
                          "already run (Gaussian weights around each measured chunk)",
            "coefficients_ms": [float(x) for x in coef],
            "fit_error_mean": float(resid.mean()), "fit_error_max": float(resid.max()),
            "fit_error_max_near_step_time": float(resid[near].max()) if near.any() else None,
            "search": history,
            "boundaries": bal, "predicted_ms": mk, "measured_ms": float(bal_total.max()),
            "prediction_error": float(abs(mk - bal_total.max()) / bal_total.max()),
            "model_only_prediction_error": float(abs(history[0]["predicted_ms"] - history[0]["measured_ms"]) / history[0]["measured_ms"]),
            "host_ms": host_ms,
            "workload_boundaries_measured_ms": float(ref_total.max()),
            "workload_chunks_measured_ms": [round(float(x), 4) for x in ref_total],
            "searched_chunks_predicted_ms": [round(cost(bal[i], bal[i + 1] - bal[i]), 4) for i in range(p)],
            "searched_chunks_measured_ms": [round(float(x), 4) for x in bal_total],
            "kept": "searched" if bal_total.max() <= ref_total.max() else "workload boundaries (the searched split measured slower)"}

    if args.extras:
        extras(args, result, kvra, synth, torch, locals())

    if not args.no_cpu_baseline:
        del q_work
        torch.cuda.empty_cache()
        result["cpu_baseline"] = cpu_baseline(cfg)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))


def extras(args, result, kvra, synth, torch, env):
    """--extras: what the default run leaves out because it costs host time and is not part of the metric."""
    C, H, Hkv, d, p = env["C"], env["H"], env["Hkv"], env["d"], env["p"]
    bounds, q_master, stream = env["bounds"], env["q_master"], env["stream"]
    run_step, measured_chunks = env["run_step"], env["measured_chunks"]
    flops_step = env["flops_step"]
    # the same step recorded once into a HIP graph and replayed: what the host-side launch path and the
    # timing events of the eager loop cost (Q is rotated in place again on every replay, which changes its
    # values but not the work)
    qg = q_master.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run_step(bounds, qg, None, torch.cuda.current_stream())
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_rep = max(10, args.steps // 4)
    g0.record(stream)
    for _ in range(n_rep):
        graph.replay()
    g1.record(stream)
    torch.cuda.synchronize()
    graph_ms = g0.elapsed_time(g1) / n_rep
    result["hip_graph_replay"] = {"ms_per_step": graph_ms, "tflops": flops_step / (graph_ms * 1e-3) / 1e12, "replays": n_rep}
    del graph, qg
    if "cost" not in env:
        return
    cost = env["cost"]
    eq = kvra.kvra_equal_split(C, p, 64)

    def makespan_ms(bnds):
        return float(measured_chunks(bnds)[1].max())

    # per-chunk times in the chain of processes (one per chunk, 32 layers, every layer waiting for the
    # precedent's cache; no transfer time: one GPU measures none), through the library's own evaluator
    def chain_ms(bnds):
        app, tot = measured_chunks(bnds)
        a = {bnds[i]: float(app[i]) for i in range(len(bnds) - 1)}
        t = {bnds[i]: float(tot[i] - app[i]) for i in range(len(bnds) - 1)}
        return kvra.kvra_chain_ttft(bnds, 32, lambda pre, c: a[pre], lambda pre, c: t[pre])
    result["makespan"]["chain_ttft_32_layers_ms"] = {"balanced": chain_ms(bounds), "equal_split": chain_ms(eq)}
    # the paper's own search (hierarchical grid search, KVR-S) on the same cost, from the even split as in the
    # paper and seeded with the exact optimum of the analytic model
    gs_b, gs_m, gs_ev = kvra.kvra_search_grid(C, p, 64, cost)
    seed_b, _ = kvra.kvra_balance(C, p, 64)
    gs2_b, gs2_m, gs2_ev = kvra.kvra_search_grid(C, p, 64, cost, start=seed_b)
    result["makespan"]["grid_search"] = {
        "from_even_split": {"boundaries": gs_b, "predicted_ms": gs_m, "cost_evaluations": gs_ev, "measured_ms": makespan_ms(gs_b)},
        "seeded": {"boundaries": gs2_b, "predicted_ms": gs2_m, "cost_evaluations": gs2_ev, "measured_ms": makespan_ms(gs2_b)}}
    # lookup table at 4k spacing and predicted partitionings (KVR-P) for lengths between entries, against the
    # partitioning searched at that length (KVR-S) and the even split (KVR-E)
    if C >= 16384:
        lut = {L: kvra.kvra_balance(L, p, 64, cost)[0] for L in (4096, 8192, 12288, 16384)}
        pred = {}
        for L in (10240, 14336):
            kvr_p = kvra.kvra_table_predict(L, 64, lut)
            kvr_s = kvra.kvra_balance(L, p, 64, cost)[0]
            kvr_e = kvra.kvra_equal_split(L, p, 64)
            pred[str(L)] = {"kvr_p_boundaries": kvr_p, "kvr_p_ms": makespan_ms(kvr_p), "kvr_s_boundaries": kvr_s,
                            "kvr_s_ms": makespan_ms(kvr_s), "kvr_e_ms": makespan_ms(kvr_e)}
        result["makespan"]["lookup_table_4k_spacing"] = pred


if __name__ == "__main__":
    main()
