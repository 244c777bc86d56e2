"""Compile the HIP library for gfx950 in-tree: ``python -m paper_2108_02191_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librobe.so")
SOURCES = ["robe_api.hip"]
HEADERS = ["robe_device.h", "robe_kernels.h", "robe_backward_dedup.h", "robe_backward_regions.h", "robe_radix_sort.h", os.path.join("..", "..", "include", "robe.h")]


def hipcc_command(out: str = LIB) -> list:
    return [
        "hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        # hardware float atomics (global_atomic_add_f32) instead of a compare-and-swap loop
        "-munsafe-fp-atomics",
        # keep the device compiler from forming packed fp32 instructions (v_pk_*_f32).  The flag reaches
        # the host pass too, which has no such feature and says so once per inclusion: build() drops
        # exactly those lines from the log.
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unknown-warning-option",
        "-o", out,
    ] + [os.path.join(CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = False) -> str:
    cmd = hipcc_command()
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    for line in r.stderr.splitlines():
        if "'-packed-fp32-ops' is not a recognized feature for this target" in line:
            continue            # the host pass declining a device-only feature
        print(line, file=sys.stderr)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print("built", LIB)
    sys.exit(0)
