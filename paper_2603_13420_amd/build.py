"""In-tree build of libpskv.so for gfx950 with hipcc (no JIT cache, no torch extension)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpskv.so")
SOURCES = ["pskv_api.cpp", "pskv_simple.hip", "pskv_stream.hip", "pskv_resident.hip", "pskv_bwd_simple.hip", "pskv_bwd_mfma.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# Packed-fp32 VALU forms are switched off for all device code (the host pass does not know
# the feature and says so; that warning is harmless).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wall", "-ffp-contract=fast"]


# bench.py's measurement helper (an MFMA-only kernel): a library of its own, outside the attention ABI
PROBE_LIB = os.path.join(HERE, "libpskv_probe.so")
PROBE_SOURCES = ["bench_probe.hip"]


def _compile(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l or "error" in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose and out.strip():
        print(out)


def build_library(verbose: bool = False, extra=()) -> str:
    _compile([HIPCC, *FLAGS, *extra, "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES], verbose)
    _compile([HIPCC, *FLAGS, *extra, "-o", PROBE_LIB] + [os.path.join(CSRC, s) for s in PROBE_SOURCES], verbose)
    return LIB


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "pskv.h"))
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    print(build_library(verbose=True, extra=sys.argv[1:]))
