"""Where the time of each kvra_chunk_attn launch of a workload goes, from per-workgroup time stamps.

Needs the timeline build of the library (python -m paper_2405_05329_amd.build --trace), whose attention
kernel stamps the constant 100 MHz clock at the start of every piece of work, its first tile step, its last
tile step done and its end, together with the compute unit it ran on.  For every chunk of the workload this prints one table row:

  launch     HIP-event time of the call inside whole steps of the workload (append + attention per chunk,
             back to back; mean of --reps steps, product library, no stamps)
  span       first workgroup entry to last workgroup exit (timeline build)
  ideal      tile steps of the launch / CUs x step med: the launch's tile steps spread evenly over the CUs at
             the steady step time of that launch (the clock is power-managed and differs from launch to
             launch, so every launch is measured against its own step time)
  steps      time the CUs spent inside tile loops, averaged over CUs (differs from `ideal` where pieces run
             partly filled row tiles, or slower than the median: first and last steps of a piece)
  step med   median over the pieces of (time in the tile loop / tile steps)
  GHz        median over the pieces of (shader-clock cycles in the tile loop / time in it): the clock the loop ran
             at; cycles per step = step med x GHz, against the 2048 matrix-pipe cycles of a step
  pro/epi    time between a piece's start and its first step, and between its last step and its end (the
             merge of a cut unit is part of the last piece's epi), per CU
  gap        time a CU sat between two pieces, per CU
  ramp       first entry on a CU after the first entry anywhere, averaged over CUs
  tail       last exit anywhere minus the last exit on a CU, averaged over CUs (idle CUs at the end:
             partly filled last round, uneven units)
  entry      kernel entry (before the arguments are read) to the start of the workgroup's first piece, mean
             over the workgroups; it lies before `span` begins, so it is part of launch - span
  launch - span   what the event pair sees beyond the workgroups' own time (dispatch, completion); the stamps
             come from the timeline build, which runs a little slower, so this can come out negative
  before, after   the same launch's dispatch and completion measured directly: a one-wave kernel that reads the
             same clock sits before and after the stamped attention launch on the stream (probe library);
             before = its stamp to the first workgroup's first stamp, after = last workgroup exit to the
             second kernel's stamp; `empty` = stamp to stamp of two such kernels with nothing in between
             (what any kernel boundary on the stream costs).  Blank without the probe library.

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

TRACE_WORDS = 10
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
    tlib.kvra_append_kv.restype = i32
    tlib.kvra_append_kv.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, i32, f32, vp]
    tlib.kvra_trace_attach.restype = i32
    tlib.kvra_trace_attach.argtypes = [vp, ctypes.c_longlong]

    probe_path = os.path.join(pkg, "libkvra_probe.so")
    plib = ctypes.CDLL(probe_path) if os.path.exists(probe_path) else None
    if plib is not None:
        plib.kvra_probe_stamp.restype = i32
        plib.kvra_probe_stamp.argtypes = [vp, vp]

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
    marks = torch.zeros(3, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()

    # launch time: product library, HIP events around every attention call inside whole steps of the workload
    # (append + attention per chunk, back to back on one stream, as bench.py runs them: a launch timed
    # alone, with the chip idle before it, pays its dispatch and a clock ramp that a stream of work hides)
    n_chunks = len(bounds) - 1
    acc = np.zeros((args.reps, n_chunks))
    for rep in range(args.reps + 3):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_chunks)]
        for i in range(n_chunks):
            lo, c = bounds[i], bounds[i + 1] - bounds[i]
            kvra.kvra_append_kv(k_in[lo:lo + c], v_in[lo:lo + c], q[lo:lo + c], k_cache, v_cache, lo, c, C, H, Hkv, d,
                                synth.ROPE_BASE)
            evs[i][0].record()
            kvra.kvra_chunk_attn(q[lo:lo + c], k_cache, v_cache, lo, c, H, Hkv, d, scale, out[lo:lo + c])
            evs[i][1].record()
        torch.cuda.synchronize()
        if rep >= 3:
            acc[rep - 3] = [e0.elapsed_time(e1) * 1e3 for e0, e1 in evs]
    launch_times = acc.mean(axis=0)

    rows, dumps = [], {}
    for i in range(len(bounds) - 1):
        lo, c = bounds[i], bounds[i + 1] - bounds[i]
        plan = kvra.kvra_chunk_attn_plan(lo, c, H, Hkv, d, cus)
        launch_us = launch_times[i]
        # stamps: two whole steps of the workload through the timeline build (append + attention per chunk, back
        # to back, like the steps timed above), the stamp buffer attached only around this chunk's attention
        # call of the second one; five times, the launch with the median span is kept
        spans = []
        for rep in range(5):
            trace.zero_()
            for step in range(2):
                for w in range(n_chunks):
                    wlo, wc = bounds[w], bounds[w + 1] - bounds[w]
                    sl = slice(wlo, wlo + wc)
                    rc = tlib.kvra_append_kv(k_in[sl].data_ptr(), v_in[sl].data_ptr(), q[sl].data_ptr(), k_cache.data_ptr(),
                                             v_cache.data_ptr(), wlo, wc, C, H, Hkv, d, synth.ROPE_BASE, None)
                    assert rc == 0, rc
                    stamped = step == 1 and w == i
                    if stamped:
                        if plib is not None:
                            plib.kvra_probe_stamp(marks.data_ptr(), None)
                        tlib.kvra_trace_attach(trace.data_ptr(), max_groups)
                    rc = tlib.kvra_chunk_attn(q[sl].data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), wlo, wc, H, Hkv, d,
                                              scale, out[sl].data_ptr(), None)
                    assert rc == 0, rc
                    if stamped:
                        tlib.kvra_trace_attach(None, 0)
                        if plib is not None:
                            plib.kvra_probe_stamp(marks[1:].data_ptr(), None)
                            plib.kvra_probe_stamp(marks[2:].data_ptr(), None)
            torch.cuda.synchronize()
            n_groups = plan["groups"] * plan["slots"]
            t = trace[:n_groups * TRACE_PIECES].cpu().numpy().astype(np.uint64)
            t = t[t[:, 3] != 0]                       # one record per piece a workgroup ran
            mk = marks.cpu().numpy().astype(np.int64)
            around = ((int(t[:, 0].min()) - int(mk[0])) * TICK_US, (int(mk[1]) - int(t[:, 3].max())) * TICK_US,
                      (int(mk[2]) - int(mk[1])) * TICK_US) if plib is not None else None
            spans.append((int(t[:, 3].max() - t[:, 0].min()), t, around))
        spans.sort(key=lambda x: x[0])
        t = spans[len(spans) // 2][1]
        around = tuple(float(np.median([s[2][j] for s in spans])) for j in range(3)) if plib is not None else None
        dumps[f"chunk{i}"] = t
        t0 = t[:, 0].min()
        enter, loop0, loop1, exit_ = [(t[:, j] - t0).astype(np.float64) * TICK_US for j in range(4)]
        cu_key = ((t[:, 4] >> np.uint64(32)) << np.uint64(8)) | ((t[:, 4] >> np.uint64(8)) & np.uint64(0xFF))
        steps = (t[:, 5] & np.uint64(0xFFFFFFFF)).astype(np.float64)
        entry_to_start = (t[:, 5] >> np.uint64(32)).astype(np.float64) * TICK_US   # first pieces only, else 0
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
        loop_cycles = (t[:, 9] - t[:, 8]).astype(np.float64)
        ok = (loop1 - loop0) > 5.0                 # pieces long enough for the two clocks to be compared
        ghz = float(np.median(loop_cycles[ok] / (loop1 - loop0)[ok]) / 1e3) if ok.any() else 0.0
        rows.append(dict(chunk=i, prefix=lo, c=c, groups=len(steps), plan=plan, launch=launch_us, span=span,
                         total_steps=float(steps.sum()), in_steps=in_steps, pro=pro, epi=epi, gap=gap / n_cu,
                         ramp=(ramp + idle_cus * span) / n_cu, tail=tail / n_cu, idle_cus=idle_cus,
                         step_med=float(np.median(per_step)), cus_used=len(keys), ghz=ghz, around=around,
                         entry=float(entry_to_start[entry_to_start > 0].mean()) if (entry_to_start > 0).any() else 0.0))
    flops = lambda lo, c: 4 * d * H * (c * lo + c * (c + 1) // 2)
    print(f"workload {args.workload}: {H}/{Hkv} heads x {d}, context {C}; device with {cus} CUs; times in us")
    print("step med = median over the launch's pieces of (time in the tile loop / tile steps); one tile step = "
          f"{rows[0]['plan']['key_tile']} keys x {rows[0]['plan']['rows_per_tile']} rows; "
          "2048 matrix-pipe cycles per SIMD at head_dim 128 and 64 alike")
    print()
    print("| chunk | prefix | c | units, pieces | row tile | launch | TFLOP/s | span | ideal | steps | pro | epi | gap | ramp | tail | launch - span | before | after | empty | entry | step med | GHz | cycles per step |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    around_txt = lambda a: " | ".join(f"{x:.1f}" for x in a) if a is not None else " | | "
    for r in rows:
        p = r["plan"]
        shape = f"{p['units'] * p['groups']} u, {r['groups']} p" + (f", {p['partial_pieces']} merged" if p["partial_pieces"] else "")
        ideal = r["total_steps"] / cus * r["step_med"]
        print(f"| {r['chunk']} | {r['prefix']} | {r['c']} | {shape} | {p['rows_per_tile']} | {r['launch']:.1f} | "
              f"{flops(r['prefix'], r['c']) / r['launch'] / 1e6:.0f} | {r['span']:.1f} | {ideal:.1f} | {r['in_steps']:.1f} | "
              f"{r['pro']:.1f} | {r['epi']:.1f} | {r['gap']:.1f} | {r['ramp']:.1f} | {r['tail']:.1f} | "
              f"{r['launch'] - r['span']:.1f} | {around_txt(r['around'])} | {r['entry']:.1f} | {r['step_med']:.3f} | {r['ghz']:.2f} | {r['step_med'] * r['ghz'] * 1e3:.0f} |")
    tot_launch = sum(r["launch"] for r in rows)
    tot_ideal = sum(r["total_steps"] / cus * r["step_med"] for r in rows)
    print()
    print(f"sum of launches {tot_launch:.1f} us, sum of ideal {tot_ideal:.1f} us ({100 * tot_ideal / tot_launch:.1f} %); "
          f"useful {sum(flops(r['prefix'], r['c']) for r in rows) / 1e9:.1f} GFLOP -> "
          f"{sum(flops(r['prefix'], r['c']) for r in rows) / tot_launch / 1e6:.0f} TFLOP/s over the attention calls")
    if args.dump:
        np.savez_compressed(args.dump, **dumps)


if __name__ == "__main__":
    main()
