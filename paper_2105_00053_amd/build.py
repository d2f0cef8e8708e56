"""Builds the HIP library (gfx950) and the host-only check library, in-tree.

    python -m paper_2105_00053_amd.build

Each .hip translation unit is compiled to an object in parallel, then linked
into libpositnn_hip.so next to this file.  Packed-FP32 instruction selection is
switched off for all device code.
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpositnn_hip.so")
HOSTCHECK = os.path.join(HERE, "libpositnn_hostcheck.so")
RATES = os.path.join(HERE, "libpositnn_rates.so")  # instruction-issue microbenchmarks for bench.py --issue-rates
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ARCH = "gfx950"

UNITS = ["api_elementwise.hip", "api_gemm.hip", "api_conv.hip", "api_glue.hip", "api_noquire.hip", "api_loss.hip"]
# Floating-point model, stated rather than left to the compiler's default: the fp64 "buckets" that carry exact
# sums rely on every operation being the IEEE one that is written -- (r + C) - C must round r, not fold to r, and a
# multiply-add is fused only where the source says fma().  So: no fast-math, no contraction across operations.
FP_FLAGS = ["-fno-fast-math", "-ffp-contract=off"]
DEVICE_FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=" + ARCH,
                "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + FP_FLAGS + [
                "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + "\n")
        raise RuntimeError("build step failed: " + cmd[-1])
    return r.stdout


def _compile(unit):
    src = os.path.join(CSRC, unit)
    obj = os.path.join(OBJ, unit.replace(".hip", ".o"))
    _run([HIPCC] + DEVICE_FLAGS + ["-c", src, "-o", obj])
    return obj


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(UNITS))) as ex:
        objs = list(ex.map(_compile, UNITS))
    _run([HIPCC, "-shared", "-fPIC", "--offload-arch=" + ARCH, "-o", LIB] + objs)
    # host-only build of the scalar functions, for CPU unit tests
    _run([HIPCC, "-O2", "-std=c++17", "-fPIC", "-shared", "--cuda-host-only", "-x", "hip"] + FP_FLAGS + [
          "-Wno-unused-command-line-argument", os.path.join(CSRC, "host_check.hip"), "-o", HOSTCHECK])
    _run([HIPCC] + DEVICE_FLAGS + ["-shared", os.path.join(CSRC, "issue_rates.hip"), "-o", RATES])
    if verbose:
        print("built", LIB, ",", HOSTCHECK, "and", RATES)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
