"""Builds librtn.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librtn.so")
SOURCES = ["rtn_api.hip", "ternarize_pack.hip", "tmm_mfma.hip", "tgemm_popc.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra",
         "-Wno-unused-parameter",
         # keep hipcc from forming packed-fp32 instructions out of scalar float code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_lib(verbose=False, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + FLAGS + list(extra) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build_lib(verbose=True, extra=sys.argv[1:])
