"""Builds the HIP library (kernels + C boundary) for gfx950, in-tree: libamp.so, and libamp_strict.so, the same
sources compiled with -DAMP_STRICT_JOIN (joins completed with explicit acquire / release ordering instead of the
fence-free shortcut; the parity suite runs both so that a mismatch can be attributed)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libamp.so")
LIB_STRICT = os.path.join(HERE, "libamp_strict.so")
SOURCES = ["amp_kernels.hip", "amp_lib.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-shared", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False, strict: bool = True) -> str:
    src = [os.path.join(HERE, "csrc", s) for s in SOURCES]
    jobs = [(LIB, [])]
    if strict:
        jobs.append((LIB_STRICT, ["-DAMP_STRICT_JOIN"]))
    procs = [(out, subprocess.Popen(["hipcc"] + FLAGS + extra + src + ["-o", out], stdout=subprocess.PIPE,
                                    stderr=subprocess.STDOUT, text=True)) for out, extra in jobs]
    for out, p in procs:
        log, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (os.path.basename(out), log))
        if verbose:
            print(log)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
