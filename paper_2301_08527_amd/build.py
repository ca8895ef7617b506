"""Builds librocket_mi355x.so (the C-ABI library) in-tree with hipcc for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librocket_mi355x.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

COMMON = ["-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall"]
# device code: gfx950 only; packed-FP32 instruction selection is switched off
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return [os.path.join(CSRC, f) for f in ("sampler.cpp", "rocket.hip", "rocket_internal.hpp")] + \
           [os.path.join(ROOT, "include", "rocket.h")]


def build(force=True, verbose=False):
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in sources()):
        return LIB
    objs = []
    # the sampler must be bit-reproducible: no contraction into FMAs, no fast-math
    jobs = [
        (os.path.join(CSRC, "sampler.cpp"), [HIPCC, "-x", "c++", "-ffp-contract=off", "-fno-fast-math"] + COMMON),
        (os.path.join(CSRC, "rocket.hip"), [HIPCC] + DEVICE + COMMON),
    ]
    for src, cmd in jobs:
        obj = os.path.splitext(src)[0] + ".o"
        full = cmd + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(full))
        subprocess.check_call(full)
        objs.append(obj)
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(link))
    subprocess.check_call(link)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv, verbose=True))
