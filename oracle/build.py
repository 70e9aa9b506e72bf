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


def source_digest() -> str:
    """SHA-256 over the compiler flags and the contents of the sources."""
    import hashlib
    h = hashlib.sha256(" ".join(FLAGS).encode())
    for p in SOURCES:
        with open(p, "rb") as f:
            h.update(os.path.basename(p).encode() + b"\0" + f.read())
    return h.hexdigest()[:32]


def built_digest():
    """The digest stored in the built library (the text "oracle-build-id:<digest>" in its bytes), or None."""
    import re
    if not os.path.exists(LIB):
        return None
    with open(LIB, "rb") as f:
        m = re.search(rb"oracle-build-id:([0-9a-f]{32})", f.read())
    return m.group(1).decode() if m else None


def is_stale() -> bool:
    """True when the library is missing or was built from other sources or flags than the ones on disk."""
    return built_digest() != source_digest()


def build(force: bool = True) -> str:
    if not force and not is_stale():
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc", *FLAGS, '-DORACLE_BUILD_ID="%s"' % source_digest(), *SOURCES, "-o", tmp, "-lm"])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
