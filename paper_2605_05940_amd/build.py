"""Compile the HIP sources under ``csrc/`` into ``libnpd.so`` for gfx950 (cross-compiles without a GPU)."""
import concurrent.futures
import glob
import os
import shutil
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libnpd.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # no implicit fusing of a*b+c: every fused multiply-add in the kernels is written out, so that two
    # streams fed the same data round the same way wherever the expression is inlined
    "-ffp-contract=off",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False, extra=(), out: str = LIB, jobs: int = 6) -> str:
    """Every source becomes an object of its own (in parallel), then one shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = tempfile.mkdtemp(prefix="npd_build_")
    try:
        def compile_one(src):
            obj = os.path.join(tmp, os.path.basename(src)[:-4] + ".o")
            cmd = [hipcc, *HIPCC_FLAGS, *extra, "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.check_call(cmd)
            return obj
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
            objs = list(pool.map(compile_one, sources()))
        cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", out, *objs]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return out


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
