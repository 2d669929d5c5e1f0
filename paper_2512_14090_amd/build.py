"""Builds libaiq.so (HIP kernels + C boundary) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libaiq.so")
SOURCES = ["aiq_host.cpp", "aiq_kernels.hip", "aiq_fused.hip", "aiq_mbconv.hip", "aiq_deploy.hip", "aiq_int8.hip",
           "aiq_mbconv_codes.hip"]
HEADERS = ["aiq_internal.h", os.path.join("..", "..", "include", "aiq.h")]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
    # packed-FP32 instruction selection off; IEEE-exact fp32 division for the quantizer
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math",
    # the LDS-resident kernels are straight-line code: loops marked for unrolling are unrolled whatever their size
    "-mllvm", "-pragma-unroll-threshold=1000000",
    "-Wall", "-Wno-unused-function",
]


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True, verbose=False):
    """Compiles every HIP source; returns the library path."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def build_copy_probe():
    """Optional, not part of build(): the stand-alone copy kernel of known size against which the HBM traffic
    counters (FETCH_SIZE, WRITE_SIZE) are calibrated.  Returns the path of the executable."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(HERE, "copy_probe")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Wno-unused-value",
                    os.path.join(CSRC, "copy_probe.hip"), "-o", out], check=True)
    return out


def build_mfma_mix_probe():
    """Optional, not part of build(): the stand-alone microbenchmark of what instructions issued between MFMAs
    cost (profiles/mfma_valu_issue_microbenchmark.md).  Returns the path of the executable."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(HERE, "mfma_mix_probe")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                    "-packed-fp32-ops", os.path.join(CSRC, "mfma_mix_probe.hip"), "-o", out], check=True)
    return out


if __name__ == "__main__":
    if "--mfma-mix-probe" in sys.argv:
        print(build_mfma_mix_probe())
    elif "--copy-probe" in sys.argv:
        print(build_copy_probe())
    else:
        print(build(force=True, verbose="-v" in sys.argv))
