"""Where the time of each kvra_chunk_attn launch of a workload goes, from per-workgroup time stamps.

Needs the timeline build of the library (python -m paper_2405_05329_amd.build --trace), whose attention
kernel stamps the constant 100 MHz clock at the start of every piece of work, its first tile step, its last
tile step done and its end, together with the compute unit it ran on.  For every chunk of the workload this prints one table row:

  launch     HIP-event time of the call (median of --reps, product library, no stamps)
  span       first workgroup entry to last workgroup exit (timeline build)
  ideal      tile steps of the launch / CUs x the steady step time (the median time per tile step of the
             workgroups of the chunk that fills the chip best, printed below the table)
  steps      time the CUs spent inside tile loops, averaged over CUs; beyond `ideal` this is partly filled
             row tiles and the slower or faster clock of that launch
  pro/epi    time between a piece's start and its first step, and between its last step and its end (the
             merge of a cut unit is part of the last piece's epi), per CU
  gap        time a CU sat between two pieces, per CU
  ramp       first entry on a CU after the first entry anywhere, averaged over CUs
  tail       last exit anywhere minus the last exit on a CU, averaged over CUs (idle CUs at the end:
             partly filled last round, uneven units)
  launch - span   dispatch of the kernel

Per CU, span = ramp + pro + steps + epi + gap + tail; the columns are these terms averaged over the CUs
(a CU that never got a workgroup counts as ramp = span).

Usage: python -m paper_2405_05329_amd.timeline [--workload llama7b_16k_balanced] [--reps 20]
"""
from __future__ import annotations

import argparse
import ctypes
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

TRACE_WORDS = 8
TRACE_PIECES = 8   # pieces per workgroup that leave stamps
TICK_US = 0.01   # 100 MHz


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="llama7b_16k_balanced")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--dump", default=None, help="write the raw stamps of every chunk to this .npz")
    ap.add_argument("--trace-lib", default=None, help="timeline build to load (default: libkvra_trace.so beside this file)")
    args = ap.parse_args()

    import torch
    from paper_2405_05329_amd import kvra, synth

    pkg = os.path.dirname(os.path.abspath(__file__))
    tlib = ctypes.CDLL(args.trace_lib or os.path.join(pkg, "libkvra_trace.so"))
    i64, i32, f32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_void_p
    tlib.kvra_chunk_attn.restype = i32
    tlib.kvra_chunk_attn.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, f32, vp, vp]
    tlib.kvra_trace_attach.restype = i32
    tlib.kvra_trace_attach.argtypes = [vp, ctypes.c_longlong]

    torch.cuda.set_device(0)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    cfg = synth.CONFIGS[args.workload]
    C, H, Hkv, d, bounds = cfg["C"], cfg["H"], cfg["Hkv"], cfg["d"], cfg["boundaries"]
    scale = synth.default_scale(d)

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    qb, kb, vb = synth.make_qkv(0, cfg["cfg_id"], C, H, Hkv, d)
    q, k_in, v_in = dev(qb), dev(kb), dev(vb)
    k_cache = torch.zeros((C, Hkv, d), dtype=torch.bfloat16, device="cuda")
    v_cache = torch.zeros_like(k_cache)
    out = torch.empty((C, H, d), dtype=torch.bfloat16, device="cuda")
    kvra.kvra_append_kv(k_in, v_in, q, k_cache, v_cache, 0, C, C, H, Hkv, d, synth.ROPE_BASE)
    max_groups = 1 << 12
    trace = torch.zeros((max_groups * TRACE_PIECES, TRACE_WORDS), dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()

    rows, dumps = [], {}
    for i in range(len(bounds) - 1):
        lo, c = bounds[i], bounds[i + 1] - bounds[i]
        plan = kvra.kvra_chunk_attn_plan(lo, c, H, Hkv, d, cus)
        # launch time: product library, HIP events, median
        times = []
        for rep in range(args.reps + 3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            kvra.kvra_chunk_attn(q[lo:lo + c], k_cache, v_cache, lo, c, H, Hkv, d, scale, out[lo:lo + c])
            e1.record()
            torch.cuda.synchronize()
            if rep >= 3:
                times.append(e0.elapsed_time(e1) * 1e3)
        launch_us = float(np.median(times))
        # stamps: timeline build, a few launches, keep the one with the median span
        tlib.kvra_trace_attach(trace.data_ptr(), max_groups)
        spans = []
        for rep in range(5):
            trace.zero_()
            torch.cuda.synchronize()
            rc = tlib.kvra_chunk_attn(q[lo:lo + c].data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), lo, c, H, Hkv, d,
                                      scale, out[lo:lo + c].data_ptr(), None)
            assert rc == 0, rc
            torch.cuda.synchronize()
            n_groups = plan["groups"] * plan["slots"]
            t = trace[:n_groups * TRACE_PIECES].cpu().numpy().astype(np.uint64)
            t = t[t[:, 3] != 0]                       # one record per piece a workgroup ran
            spans.append((int(t[:, 3].max() - t[:, 0].min()), t))
        tlib.kvra_trace_attach(None, 0)
        spans.sort(key=lambda x: x[0])
        t = spans[len(spans) // 2][1]
        dumps[f"chunk{i}"] = t
        t0 = t[:, 0].min()
        enter, loop0, loop1, exit_ = [(t[:, j] - t0).astype(np.float64) * TICK_US for j in range(4)]
        cu_key = ((t[:, 4] >> np.uint64(32)) << np.uint64(8)) | ((t[:, 4] >> np.uint64(8)) & np.uint64(0xFF))
        steps = t[:, 5].astype(np.float64)
        span = float(exit_.max())
        keys = np.unique(cu_key)
        ramp = tail = gap = 0.0
        for key in keys:
            sel = np.where(cu_key == key)[0]
            order = sel[np.argsort(enter[sel])]
            ramp += enter[order[0]]
            tail += span - exit_[order].max()
            gap += float(np.sum(np.maximum(enter[order[1:]] - exit_[order[:-1]], 0.0)))
        n_cu = cus
        idle_cus = n_cu - len(keys)          # CUs that never got a workgroup
        in_steps = float(np.sum(loop1 - loop0)) / n_cu
        pro = float(np.sum(loop0 - enter)) / n_cu
        epi = float(np.sum(exit_ - loop1)) / n_cu
        per_step = (loop1 - loop0) / np.maximum(steps, 1.0)
        rows.append(dict(chunk=i, prefix=lo, c=c, groups=len(steps), plan=plan, launch=launch_us, span=span,
                         total_steps=float(steps.sum()), in_steps=in_steps, pro=pro, epi=epi, gap=gap / n_cu,
                         ramp=(ramp + idle_cus * span) / n_cu, tail=tail / n_cu, idle_cus=idle_cus,
                         step_med=float(np.median(per_step)), cus_used=len(keys)))
    # steady step time: the chunk whose workgroups fill whole rounds of the chip best
    def fill(r):
        g = r["groups"]
        return g / (cus * np.ceil(g / cus))
    best = max(rows, key=lambda r: (fill(r), r["total_steps"]))
    t_step = best["step_med"]
    flops = lambda lo, c: 4 * d * H * (c * lo + c * (c + 1) // 2)
    print(f"workload {args.workload}: {H}/{Hkv} heads x {d}, context {C}; device with {cus} CUs; times in us")
    print(f"steady step time {t_step:.3f} us = median time per tile step ({best['plan']['key_tile']} keys x "
          f"{best['plan']['rows_per_tile']} rows) of the workgroups of chunk {best['chunk']} ({best['groups']} workgroups)")
    print()
    print("| chunk | prefix | c | units, pieces | row tile | launch | TFLOP/s | span | ideal | steps | pro | epi | gap | ramp | tail | launch - span | step med |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    for r in rows:
        p = r["plan"]
        shape = f"{p['units'] * p['groups']} u, {r['groups']} p" + (f", {p['partial_pieces']} merged" if p["partial_pieces"] else "")
        ideal = r["total_steps"] / cus * t_step
        print(f"| {r['chunk']} | {r['prefix']} | {r['c']} | {shape} | {p['rows_per_tile']} | {r['launch']:.1f} | "
              f"{flops(r['prefix'], r['c']) / r['launch'] / 1e6:.0f} | {r['span']:.1f} | {ideal:.1f} | {r['in_steps']:.1f} | "
              f"{r['pro']:.1f} | {r['epi']:.1f} | {r['gap']:.1f} | {r['ramp']:.1f} | {r['tail']:.1f} | "
              f"{r['launch'] - r['span']:.1f} | {r['step_med']:.3f} |")
    tot_launch = sum(r["launch"] for r in rows)
    tot_ideal = sum(r["total_steps"] / cus * t_step for r in rows)
    print()
    print(f"sum of launches {tot_launch:.1f} us, sum of ideal {tot_ideal:.1f} us ({100 * tot_ideal / tot_launch:.1f} %); "
          f"useful {sum(flops(r['prefix'], r['c']) for r in rows) / 1e9:.1f} GFLOP -> "
          f"{sum(flops(r['prefix'], r['c']) for r in rows) / tot_launch / 1e6:.0f} TFLOP/s over the attention calls")
    if args.dump:
        np.savez_compressed(args.dump, **dumps)


if __name__ == "__main__":
    main()
