"""Build libloki_alloc.so and the instruction-rate probe libloki_probe.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libloki_alloc.so")
SOURCES = ["loki_kernels.hip", "loki_static.hip", "loki_api.cpp"]
PROBE_LIB = os.path.join(HERE, "libloki_probe.so")
PROBE_SOURCES = ["loki_valu_rate.hip"]
HEADERS = ["loki_device.h", "loki_launch.h", "loki_host.h"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                                        # every fp64 op rounded on its own
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-fp32 instructions
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def build_library(force: bool = True, verbose: bool = False) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(CSRC, s) for s in PROBE_SOURCES] + [os.path.join(CSRC, h) for h in HEADERS] + \
        [os.path.join(os.path.dirname(HERE), "include", h) for h in ("loki_alloc.h", "loki_probe.h")]
    if not force and os.path.exists(LIB) and os.path.exists(PROBE_LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(d) for d in deps):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    for lib, sources in ((PROBE_LIB, [os.path.join(CSRC, s) for s in PROBE_SOURCES]), (LIB, srcs)):
        cmd = [hipcc] + HIPCC_FLAGS + ["-o", lib] + sources
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True, cwd=CSRC)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
