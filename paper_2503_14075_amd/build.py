"""Build libtwigpath.so (HIP, gfx950 only) next to this file.

    python -m paper_2503_14075_amd.build [--force]
    python -m paper_2503_14075_amd.build --trace    # diagnostic build libtwigpath_trace.so (-DTW_TRACE)
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtwigpath.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fvisibility=hidden",     # only the tw_* entry points of the header are exported
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(ROOT, "include", "twigpath.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, extra=(), out: str = LIB) -> str:
    if force or out != LIB or is_stale():
        cmd = ["hipcc"] + [f for f in FLAGS if f] + list(extra) + ["-o", out] + sources()
        subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    args = [a for a in sys.argv[1:] if a != "--force"]
    if "--trace" in args:
        args.remove("--trace")
        print(build(extra=["-DTW_TRACE"] + args, out=os.path.join(HERE, "libtwigpath_trace.so")))
    else:
        print(build(force=True, extra=args))
