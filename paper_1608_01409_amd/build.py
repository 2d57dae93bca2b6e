"""Build libsconv.so (hipcc, gfx950) in-tree, next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsconv.so")
SOURCES = ["sconv_api.cpp", "sconv_host.cpp", "sconv_kernels.hip"]
# -packed-fp32-ops is switched off: the packed FP32 forms are not to be generated for this machine.
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False) -> str:
    subprocess.check_call([sys.executable, os.path.join(CSRC, "gen_lds_loops.py")])
    subprocess.check_call([sys.executable, os.path.join(CSRC, "gen_lds2.py")])
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip", *DEVICE_FLAGS,
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


def build_ceilings(hipcc: str | None = None) -> str:
    """The ceilings microbenchmark (stand-alone program, see csrc/sconv_ceilings.hip); only the profiling
    runs use it, so it is built on request: python -m paper_1608_01409_amd.build --ceilings"""
    hipcc = hipcc or os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([sys.executable, os.path.join(CSRC, "gen_ceilings.py")])
    exe = os.path.join(HERE, "sconv_ceilings")
    cmd = [hipcc, "-O3", "-std=c++17", *DEVICE_FLAGS, "-I", CSRC, os.path.join(CSRC, "sconv_ceilings.hip"), "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    return exe


if __name__ == "__main__":
    print(build(verbose=True))
    if "--ceilings" in sys.argv[1:]:
        print(build_ceilings())
