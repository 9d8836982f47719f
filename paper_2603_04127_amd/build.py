"""Build the C-ABI shared library (libdark.so) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdark.so")
SOURCES = ["api.hip", "generic.hip", "fused.hip", "fused_feat.hip", "fused_causal.hip", "fused_scan.hip", "fused_bwd.hip", "ceilings.hip", "whiten.hip", "decode.hip"]
# per-file extra flags: the fused kernels never produce NaNs from finite inputs and want v_max3_f32
EXTRA = {"fused.hip": ["-fno-honor-nans"], "fused_feat.hip": ["-fno-honor-nans"],
         "fused_causal.hip": ["-fno-honor-nans"], "fused_scan.hip": ["-fno-honor-nans"], "fused_bwd.hip": ["-fno-honor-nans"], "whiten.hip": ["-fno-honor-nans"]}
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=default",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


LIB_TIMELINE = os.path.join(HERE, "libdark_timeline.so")


def build(verbose: bool = True, timeline: bool = False) -> str:
    """Compile every source and link the library.  timeline=True builds a second library beside it,
    libdark_timeline.so, whose two large forward kernels record wall-clock stamps (-DDARK_TIMELINE)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    suffix = ".tl.o" if timeline else ".o"
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", suffix))
        extra = EXTRA.get(src, []) + (["-DDARK_TIMELINE"] if timeline else [])
        cmd = [hipcc, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd)))
        objs.append(obj)
    for src, pr in procs:
        if pr.wait() != 0:
            raise RuntimeError(f"hipcc failed on {src}")
    lib = LIB_TIMELINE if timeline else LIB
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return lib


if __name__ == "__main__":
    build()
    sys.exit(0)
