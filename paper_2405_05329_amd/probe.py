"""What the matrix pipes deliver on this GPU with nothing else in the way: a loop of v_mfma_f32_32x32x16_bf16 on
register operands, timed for several numbers of busy compute units, one or two waves per SIMD, and operand
data of three kinds (zeros, ones, N(0,1) values).  A yardstick for the roofline fractions of the product
kernels: 32768 FLOP per MFMA and 8 passes of 4 cycles give 4096 FLOP per cycle and compute unit, which is the
published 2.5 PFLOP/s at 2.4 GHz on 256 compute units; the "clock" column is rate / (busy CUs x 4096 FLOP),
i.e. the clock at which pipes that never idle would deliver the measured rate.

Needs the probe library: python -m paper_2405_05329_amd.build --probe
Usage: python -m paper_2405_05329_amd.probe [--iters 20000]
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


def matrix_pipes_alone(torch, iters=20000, reps=3):
    """TFLOP/s of the MFMA-only loop on this GPU right now: all compute units busy, two waves per SIMD, N(0,1)
    bf16 operands (the value distribution of the synthetic workloads).  Median of `reps` launches after one
    untimed launch.  Raises if the probe library has not been built."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkvra_probe.so")
    if not os.path.exists(path):
        raise RuntimeError("libkvra_probe.so is not built: python -m paper_2405_05329_amd.build --probe")
    lib = ctypes.CDLL(path)
    vp, i32 = ctypes.c_void_p, ctypes.c_int
    lib.kvra_probe_mfma.restype = i32
    lib.kvra_probe_mfma.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    cus = torch.cuda.get_device_properties(torch.cuda.current_device()).multi_processor_count
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    ops = torch.randn((8, 64, 8), device="cuda", generator=g).to(torch.bfloat16)
    sink = torch.empty(cus * 512, dtype=torch.float32, device="cuda")
    times = []
    for rep in range(reps + 1):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        rc = lib.kvra_probe_mfma(ops.data_ptr(), sink.data_ptr(), cus, 8, iters, None, None)
        if rc != 0:
            raise RuntimeError(f"kvra_probe_mfma returned {rc}")
        e1.record()
        torch.cuda.synchronize()
        if rep:
            times.append(e0.elapsed_time(e1))
    ms = float(np.median(times))
    return {"tflops": cus * 8 * iters * 16 * 32768.0 / (ms * 1e-3) / 1e12, "ms": ms, "busy_cus": cus,
            "waves_per_simd": 2, "operands": "N(0,1) bf16"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=20000)
    args = ap.parse_args()
    import torch

    lib = ctypes.CDLL(os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkvra_probe.so"))
    vp, i32 = ctypes.c_void_p, ctypes.c_int
    lib.kvra_probe_mfma.restype = i32
    lib.kvra_probe_mfma.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    torch.cuda.set_device(0)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    data = {
        "zeros": torch.zeros((8, 64, 8), dtype=torch.bfloat16, device="cuda"),
        "ones": torch.ones((8, 64, 8), dtype=torch.bfloat16, device="cuda"),
        "N(0,1)": torch.randn((8, 64, 8), device="cuda", generator=g).to(torch.bfloat16),
    }
    sink = torch.empty(cus * 512, dtype=torch.float32, device="cuda")
    print(f"device with {cus} CUs; {args.iters} x 16 MFMAs per wave; one workgroup per CU")
    print()
    print("| busy CUs | waves per SIMD | operands | ms | TFLOP/s | % of 2.5 PFLOP/s x busy/256 | clock GHz |")
    print("|---|---|---|---|---|---|---|")
    for wgs in (cus, cus * 3 // 4, cus // 2, cus // 4):
        for waves in (4, 8):
            for name, ops in data.items():
                times = []
                for rep in range(4):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    rc = lib.kvra_probe_mfma(ops.data_ptr(), sink.data_ptr(), wgs, waves, args.iters, None, None)
                    assert rc == 0, rc
                    e1.record()
                    torch.cuda.synchronize()
                    if rep:
                        times.append(e0.elapsed_time(e1))
                ms = float(np.median(times))
                flop = wgs * waves * args.iters * 16 * 32768.0
                rate = flop / (ms * 1e-3)
                print(f"| {wgs} | {waves // 4} | {name} | {ms:.2f} | {rate / 1e12:.0f} | "
                      f"{100 * rate / (2.5e15 * wgs / 256):.0f} | {rate / (wgs * 4096.0) / 1e9:.2f} |")

    # the same loop on all CUs, N(0,1) operands, two waves per SIMD, with per-workgroup stamps: do the XCDs differ,
    # and does the shader-clock cycle counter (which timeline.py uses) agree with the clock the MFMA count implies?
    stamps = torch.zeros((cus, 8, 4), dtype=torch.int64, device="cuda")
    for rep in range(2):
        rc = lib.kvra_probe_mfma(data["N(0,1)"].data_ptr(), sink.data_ptr(), cus, 8, args.iters, stamps.data_ptr(), None)
        assert rc == 0, rc
        torch.cuda.synchronize()
    st = stamps.cpu().numpy()
    xcd = st[:, 0, 0]
    dur = (st[:, :, 2].max(axis=1) - st[:, :, 1].min(axis=1)) * 0.01          # us, first wave in to last wave out
    cycles = st[:, :, 3].max(axis=1)
    print()
    print(f"per XCD, {cus} busy CUs, N(0,1) operands, two waves per SIMD: mean workgroup time in us, relative to the fastest XCD")
    print()
    print("| XCD | workgroups | mean us | relative | GHz by the cycle counter | GHz by the MFMA count |")
    print("|---|---|---|---|---|---|")
    means = {int(x): float(dur[xcd == x].mean()) for x in np.unique(xcd)}
    fastest = min(means.values())
    for x, m in sorted(means.items()):
        sel = xcd == x
        by_counter = float((cycles[sel] / dur[sel]).mean()) / 1e3
        by_count = 2 * args.iters * 16 * 32 / m / 1e3      # two waves per SIMD, 32 cycles per MFMA
        print(f"| {x} | {int(sel.sum())} | {m:.1f} | {m / fastest:.3f} | {by_counter:.2f} | {by_count:.2f} |")


    # what a VALU instruction costs a wave while its SIMD partner is idle or issues MFMAs back to back
    lib.kvra_probe_valu.restype = i32
    lib.kvra_probe_valu.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp]
    cyc = torch.zeros((cus, 4), dtype=torch.int64, device="cuda")
    rounds = 500
    print()
    print(f"VALU issue: cycles per wave64 instruction of a stream of independent instructions ({rounds * 64} per wave), "
          "one timed wave per SIMD, all CUs")
    print()
    print("| stream | SIMD partner | cycles per instruction |")
    print("|---|---|---|")
    res = {}
    for with_exp in (0, 1):
        for with_mfma in (0, 1):
            for rep in range(2):
                rc = lib.kvra_probe_valu(data["N(0,1)"].data_ptr(), sink.data_ptr(), cyc.data_ptr(), cus, rounds, with_mfma,
                                         with_exp, None)
                assert rc == 0, rc
                torch.cuda.synchronize()
            res[(with_exp, with_mfma)] = float(cyc.cpu().numpy().mean()) / (rounds * 64)
    for with_mfma in (0, 1):
        partner = "MFMAs back to back" if with_mfma else "idle"
        fma = res[(0, with_mfma)]
        mixed = res[(1, with_mfma)]
        print(f"| v_fma_f32 | {partner} | {fma:.1f} |")
        print(f"| v_exp_f32 (from a 1:1 mix with v_fma_f32: 2 x {mixed:.1f} - {fma:.1f}) | {partner} | {2 * mixed - fma:.1f} |")


if __name__ == "__main__":
    main()
