"""Builds librtn.so (HIP, gfx950 only) in-tree with hipcc: every source is compiled to
an object of its own, in parallel, and the objects are linked into the shared library."""
import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librtn.so")
PEAKS_LIB = os.path.join(HERE, "librtn_peaks.so")     # measurement aids for bench.py, not the product
SOURCES = ["rtn_api.hip", "ternarize_pack.hip", "tgemm_popc.hip", "quaternary.hip", "dwconv.hip", "tmm_mfma.hip", "tmm_inst_gemm.hip",
           "tmm_inst_conv.hip", "tmm_inst_tern1.hip", "tmm_inst_tern2.hip", "tmm_inst_bf16.hip",
           "tmm_inst_gemm_fp4.hip", "tmm_inst_conv_fp4.hip", "tmm_inst_tern1_fp4.hip", "tmm_inst_tern2_fp4.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         "-Wno-unused-parameter",
         # keep hipcc from forming packed-fp32 instructions out of scalar float code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# the host pass does not know the target feature above and says so once per kernel
NOISE = "is not a recognized feature for this target"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if NOISE not in l)
    if out.strip():
        print(out, flush=True)
    if p.returncode != 0:
        raise subprocess.CalledProcessError(p.returncode, cmd)


def build_lib(verbose=False, extra=(), jobs=None):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or min(len(SOURCES), int(os.environ.get("MAX_JOBS", "0")) or os.cpu_count() or 4)
    with tempfile.TemporaryDirectory(prefix="rtn_build_") as tmpdir:
        objs = [os.path.join(tmpdir, s.replace(".hip", ".o")) for s in SOURCES]
        cmds = [[hipcc] + FLAGS + list(extra) + ["-c", os.path.join(CSRC, s), "-o", o]
                for s, o in zip(SOURCES, objs)]
        with ThreadPoolExecutor(max_workers=jobs) as ex:
            list(ex.map(lambda c: _run(c, verbose), cmds))
        tmp = LIB + ".tmp.%d" % os.getpid()
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp], verbose)
    os.replace(tmp, LIB)
    tmp = PEAKS_LIB + ".tmp.%d" % os.getpid()
    _run([hipcc] + FLAGS + ["-shared", os.path.join(CSRC, "peaks.hip"), "-o", tmp], verbose)
    os.replace(tmp, PEAKS_LIB)
    return LIB


if __name__ == "__main__":
    build_lib(verbose=True, extra=sys.argv[1:])
