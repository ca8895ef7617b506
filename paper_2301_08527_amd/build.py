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
COMMON += os.environ.get("ROCKET_EXTRA_FLAGS", "").split()      # e.g. -DRK_TILE_POSITIONS=32768 for tuning runs
LIB = os.environ.get("ROCKET_LIB_OUT", LIB)
# device code: gfx950 only; packed-FP32 instruction selection is switched off
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


KERNEL_TUS = ("rocket_forward.hip", "rocket_forward_short.hip", "rocket_backward.hip", "rocket_ridge.hip",
              "rocket_prologue.hip", "rocket_train.hip", "rocket_calibrate.hip", "rocket_minirocket.hip",
              "rocket_minirocket_forward.hip")   # translation units that hold device code
HOST_TUS = ("rocket_api.hip",)


def sources():
    names = ("sampler.cpp", "rocket_internal.hpp", "rocket_device.hpp", "rocket_forward_impl.hpp") + KERNEL_TUS + HOST_TUS
    return [os.path.join(CSRC, f) for f in names] + [os.path.join(ROOT, "include", "rocket.h")]


# Instructions that must not appear in the kernels: indirect register-file indexing
# (an accumulator array indexed at run time) and scratch (spilled) memory traffic.
FORBIDDEN = ("s_set_gpr_idx_on", "v_movrel", "scratch_load", "scratch_store")


def check_device_code(asm, verbose=False):
    """Fails if the gfx950 assembly of the kernels holds a forbidden instruction."""
    text = open(asm).read()
    bad = [w for w in FORBIDDEN if w in text]
    if bad:
        raise RuntimeError("device code contains %s: a register array is indexed at run time or spilled" % bad)
    for line in text.splitlines():
        if ".private_segment_fixed_size:" in line and line.split(":")[1].strip() != "0":
            raise RuntimeError("a kernel uses scratch memory: " + line.strip())


def build(force=True, verbose=False):
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in sources()):
        return LIB
    tmp = os.path.join(CSRC, "_build")
    os.makedirs(tmp, exist_ok=True)
    for f in os.listdir(tmp):
        if f.endswith(".s") or f.endswith(".o"):
            os.remove(os.path.join(tmp, f))
    # the sampler must be bit-reproducible: no contraction into FMAs, no fast-math
    jobs = [(os.path.join(CSRC, "sampler.cpp"), [HIPCC, "-x", "c++", "-ffp-contract=off", "-fno-fast-math"] + COMMON)]
    # -save-temps keeps the gfx950 assembly of the same compilation for the check below
    jobs += [(os.path.join(CSRC, f), [HIPCC, "-save-temps=obj"] + DEVICE + COMMON) for f in KERNEL_TUS]
    jobs += [(os.path.join(CSRC, f), [HIPCC] + DEVICE + COMMON) for f in HOST_TUS]
    objs, procs = [], []
    for src, cmd in jobs:           # the translation units compile side by side
        obj = os.path.join(tmp, os.path.splitext(os.path.basename(src))[0] + ".o")
        full = cmd + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(full))
        procs.append((full, subprocess.Popen(full, stderr=None if verbose else subprocess.DEVNULL)))
        objs.append(obj)
    for full, p in procs:
        if p.wait() != 0:
            raise subprocess.CalledProcessError(p.returncode, full)
    asm = [os.path.join(tmp, f) for f in os.listdir(tmp) if f.endswith(".s") and "gfx950" in f]
    if len(asm) < len(KERNEL_TUS):
        raise RuntimeError("no gfx950 assembly was produced")
    for a in asm:
        check_device_code(a, verbose)
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(link))
    subprocess.check_call(link)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv, verbose=True))
