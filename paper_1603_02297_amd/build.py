"""Build libttc.so in-tree with hipcc for gfx950.  Run as `python -m paper_1603_02297_amd.build`.

Every source is compiled to an object file (in parallel) and the objects are linked.  A plain call
recompiles everything; `--incremental` keeps objects that are newer than their source and every header.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libttc.so")
SOURCES = ["ttc_launch_f32.hip", "ttc_launch_mixed_real.hip", "ttc_launch_f64.hip", "ttc_launch_c64.hip",
           "ttc_launch_mixed_complex.hip", "ttc_launch_c128.hip", "ttc_plan.cpp", "ttc_cache.cpp", "ttc_device.hip"]


def _flags(verbose: bool):
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
             # packed fp32 instructions are kept out of every kernel of this library
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    if verbose:
        flags += ["-Rpass-analysis=kernel-resource-usage"]
    return flags


def build(verbose: bool = False, incremental: bool = False) -> str:
    """Compile every source of the library for gfx950 and link libttc.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    jobs, objects = [], []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJ, s + ".o")
        objects.append(obj)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            continue
        lang = ["-x", "hip"] if s.endswith(".hip") else ["-x", "c++"]
        cmd = [hipcc] + _flags(verbose) + ["-c"] + lang + [src, "-o", obj]
        jobs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for name, proc in jobs:
        out, _ = proc.communicate()
        if proc.returncode != 0:
            failed = True
            sys.stderr.write(out)
        elif verbose:
            sys.stderr.write(out)
    if failed:
        raise RuntimeError("hipcc failed compiling libttc.so")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objects + ["-o", LIB],
                         capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed linking libttc.so")
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, incremental="--incremental" in sys.argv))
