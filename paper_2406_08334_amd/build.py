"""Build libptchunk.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libptchunk.so")
PROBE = os.path.join(HERE, "ptchunk_probe")
SOURCES = ["pt_ctx.hip", "pt_norm.hip", "pt_pack.hip", "pt_accum.hip", "pt_adamw.hip", "pt_stream.hip", "pt_host.hip", "pt_model.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                     # the fp32 sequence of the update is written out FMA by FMA
    "-fno-fast-math",
    "-fno-math-errno",                       # lets the host-side update loop vectorise its sqrt
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False) -> str:
    """Compiles every HIP source into one shared library, every time it is called."""
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = [hipcc()] + FLAGS + ["-o", LIB] + srcs
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # hipcc's host pass warns that it does not know the packed-fp32 feature: harmless
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed")
    if verbose and err.strip():
        print(err)
    # the Python-free driver of the C ABI (used under rocprofv3 for hardware counters)
    cmd = [hipcc(), "--offload-arch=gfx950", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "include"), os.path.join(CSRC, "pt_probe.cpp"),
           "-o", PROBE, "-L", HERE, "-lptchunk", "-Wl,-rpath,$ORIGIN"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed on pt_probe.cpp")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
