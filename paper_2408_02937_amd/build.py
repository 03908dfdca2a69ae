"""Builds librtams.so (HIP, gfx950 only) next to the sources."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librtams.so")
SOURCES = ["rtams.hip", "coarse.hip", "coarse_mfma.hip", "insert.hip", "pq.hip", "probe.hip", "group.hip", "scan.hip", "scan_mm.hip",
           "pq_scan.hip", "select.hip", "rearrange.hip", "maint.hip"]
HEADERS = ["rtams_dev.h", "rtams_launch.h", "search_common.h", os.path.join("..", "..", "include", "rtams.h"),
           os.path.join("..", "..", "include", "rtams_measure.h")]

# packed-fp32 instructions are switched off for every device compilation
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
OBJ = os.path.join(HERE, "_build")


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    # one compiler process per source file, all at once (the files share no device code), then the link
    jobs = []
    for s in SOURCES:
        obj = os.path.join(OBJ, s.replace(".hip", ".o"))
        cmd = [hipcc] + FLAGS + ["-c", os.path.join(CSRC, s), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        jobs.append((s, obj, subprocess.Popen(cmd)))
    failed = [s for s, _, p in jobs if p.wait() != 0]
    if failed:
        raise RuntimeError("hipcc failed for " + ", ".join(failed))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [obj for _, obj, _ in jobs] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
