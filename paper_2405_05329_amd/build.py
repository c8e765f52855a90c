"""Builds libkvra.so (HIP, gfx950 only) in-tree with hipcc.  Run: python -m paper_2405_05329_amd.build"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libkvra.so")

SOURCES = ["kvra_api.hip", "kvra_append.hip", "kvra_attn.hip", "kvra_gemm.hip", "kvra_balance.cpp", "kvra_search.cpp"]

# packed fp32 VALU ops are switched off for every device translation unit
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


TRACE_LIB = os.path.join(PKG, "libkvra_trace.so")


def build(verbose: bool = False, extra_flags=(), trace: bool = False) -> str:
    """trace=True builds libkvra_trace.so instead: the same library with per-workgroup time stamps in the
    attention kernel (-DKVRA_TRACE) and the kvra_trace_attach entry point, for timeline.py."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    objs = []
    if trace:
        extra_flags = tuple(extra_flags) + ("-DKVRA_TRACE",)
    bdir = os.path.join(PKG, "_build_trace" if trace else "_build")
    os.makedirs(bdir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(bdir, src.rsplit(".", 1)[0] + ".o")
        # -Wno-inline-asm: the LDS-direct loads name m0 in their clobber list (they have to set it), which
        # clang reports once per instantiation as "reserved register"; nothing else in these kernels uses m0
        cmd = [hipcc, "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument", "-Wno-inline-asm",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC, *DEVICE_FLAGS, *extra_flags,
               "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l or "error" in l)
        if p.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    lib = TRACE_LIB if trace else LIB
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib, *objs]
    subprocess.run(cmd, check=True)
    return lib


PROBE_LIB = os.path.join(PKG, "libkvra_probe.so")


def build_probe() -> str:
    """libkvra_probe.so: the matrix-pipe yardstick probe.py runs (one kernel, not part of the product library)."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cmd = [hipcc, "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wno-unused-command-line-argument", *DEVICE_FLAGS,
           "-x", "hip", os.path.join(CSRC, "kvra_probe.hip"), "-o", PROBE_LIB]
    subprocess.run(cmd, check=True)
    return PROBE_LIB


if __name__ == "__main__":
    if "--probe" in sys.argv:
        print(build_probe())
    else:
        print(build(verbose="-v" in sys.argv, trace="--trace" in sys.argv))
