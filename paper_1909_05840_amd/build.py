"""Build libqbert.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqbert.so")
SOURCES = ("api.hip", "quantize.hip", "qgemm_i8.hip", "bwd_bf16.hip", "hessian.hip")
# packed-fp32 instructions are switched off for every device translation unit
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wno-inline-asm",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# the quantizers (also the one in the GEMM's 8-bit-output epilogue) need one rounding per operation: no fused
# multiply-add contraction there.  (__fmul_rn/__fadd_rn are plain operators to the compiler and would be fused.)
PER_FILE = {"quantize.hip": ["-ffp-contract=off"], "qgemm_i8.hip": ["-ffp-contract=off"]}


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    def compile_one(src):
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc] + COMMON + PER_FILE.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True, stderr=None if verbose else subprocess.DEVNULL)
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), 8)) as pool:   # one translation unit per worker
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]
    subprocess.run(cmd, check=True)
    for o in objs:
        os.remove(o)
    return LIB


if __name__ == "__main__":
    print("built", build(verbose=True))
