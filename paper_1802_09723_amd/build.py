"""Build the HIP library (gfx950) in-tree: paper_1802_09723_amd/lib/librrm_hip.so."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIBDIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIBDIR, "librrm_hip.so")
SOURCES = ["rrm_api.hip", "scan.hip", "conv_gather.hip", "conv_pos.hip", "conv_scatter.hip", "fc.hip", "fc_batched.hip", "bin_conv.hip", "aux.hip", "probe.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-shared", "-fvisibility=hidden",
    "-munsafe-fp-atomics",
    # no wave-level aggregation of atomics: it reads the result back at once (a wait for the memory round
    # trip), while the kernels issue their few atomics from one lane and need the result late or never
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build_lib(verbose: bool = False) -> str:
    os.makedirs(LIBDIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv))
