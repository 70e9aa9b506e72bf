"""Compile the CPU oracles (plain C, gcc) into oracle/liboracle_gemm.so.

Test infrastructure only.  The flags matter for what the oracle means:
-ffp-contract=off keeps the product and the sum as two separately rounded
operations (the multiply-then-add of the paper's Section 2.1 loop body), and
no fast-math option is ever given, so the compiler may not reassociate.  No
-march flag: the object must run on whatever host the GPU machine has.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = [os.path.join(HERE, "gemm_ref.c"), os.path.join(HERE, "gemm_ref_f32.c"),
           os.path.join(HERE, "gemm_general_ref.c"), os.path.join(HERE, "gemm_strided_ref.c")]
LIB = os.path.join(HERE, "liboracle_gemm.so")

FLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
         "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(p) for p in SOURCES):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc", *FLAGS, *SOURCES, "-o", tmp, "-lm"])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
