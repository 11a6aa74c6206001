"""Build the HIP library (csrc/*.hip -> libarith_sampling.so) for gfx950 with hipcc.

hipcc cross-compiles without a GPU.  The .so stays in-tree next to this file.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libarith_sampling.so")
SOURCES = ["as_api.hip", "as_step.hip", "as_threshold.hip", "as_model.hip", "as_interval.hip", "as_fused.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def stale():
    if not os.path.exists(OUT):
        return True
    t = os.path.getmtime(OUT)
    deps = sources() + [os.path.join(CSRC, "as_common.hpp"), os.path.join(CSRC, "as_row.hpp"),
                        os.path.join(HERE, "..", "include", "arith_sampling.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True, extra=()):
    if not force and not stale():
        return OUT
    cmd = ["hipcc"] + FLAGS + list(extra) + sources() + ["-o", OUT]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(force=True, extra=sys.argv[1:]))
