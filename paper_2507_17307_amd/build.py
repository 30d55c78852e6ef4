"""Compile the HIP library for gfx950 in-tree (paper_2507_17307_amd/librstitch.so)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "rstitch.hip")
LIB = os.path.join(HERE, "librstitch.so")
PROBE_SRC = os.path.join(HERE, "csrc", "traffic_probe.hip")
PROBE = os.path.join(HERE, "traffic_probe")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _run(cmd, verbose: bool) -> None:
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 feature name and says so; that is harmless
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if err.strip() and verbose:
        print(err, file=sys.stderr)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)


def build(verbose: bool = True) -> str:
    """The library, then the counter-run driver that links against it (found through $ORIGIN)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    _run([hipcc] + FLAGS + [SRC, "-o", LIB], verbose)
    probe_flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")]
    _run([hipcc] + probe_flags + [PROBE_SRC, "-o", PROBE, "-L" + HERE, "-lrstitch", "-Wl,-rpath,$ORIGIN"], verbose)
    return LIB


if __name__ == "__main__":
    build()
