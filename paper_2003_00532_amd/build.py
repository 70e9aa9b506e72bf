"""Compile libgemm_f64.so for gfx950 with hipcc (in-tree, next to this file)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgemm_f64.so")
SOURCES = [os.path.join(CSRC, "gemm_f64.hip"), os.path.join(CSRC, "gemm_f32.hip"), os.path.join(CSRC, "mfma_probe.hip")]
DEPENDS = SOURCES + [os.path.join(CSRC, "gemm_mfma.hpp"), os.path.join(CSRC, "gemm_host.hpp"),
                     os.path.join(os.path.dirname(HERE), "include", "gemm_f64.h"),
                     os.path.join(os.path.dirname(HERE), "include", "gemm_f32.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         # keep hipcc from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument",
         # the global->LDS copies name M0, a register the compiler reserves, in their clobber lists on purpose
         "-Wno-inline-asm"]


def source_digest() -> str:
    """SHA-256 over the compiler flags and the contents of every file the library is built from."""
    import hashlib
    h = hashlib.sha256(" ".join(FLAGS).encode())
    for p in DEPENDS:
        with open(p, "rb") as f:
            h.update(os.path.basename(p).encode() + b"\0" + f.read())
    return h.hexdigest()[:32]


def build(verbose: bool = False) -> str:
    """Compile every source to an object (in parallel: one hipcc per file) and link them into the library."""
    from concurrent.futures import ThreadPoolExecutor
    noise = "is not a recognized feature for this target"
    compile_flags = [f for f in FLAGS if f != "-shared"] + ['-DGEMM_BUILD_ID="%s"' % source_digest()]

    def compile_one(src):
        obj = os.path.join(HERE, os.path.basename(src) + ".%d.o" % os.getpid())
        res = subprocess.run([HIPCC, *compile_flags, "-c", src, "-o", obj], capture_output=True, text=True)
        err = "\n".join(ln for ln in res.stderr.splitlines() if noise not in ln)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
        return obj, err

    objs = []
    try:
        with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
            for obj, err in pool.map(compile_one, SOURCES):
                objs.append(obj)
                if verbose and err.strip():
                    print(err)
        tmp = LIB + ".tmp.%d" % os.getpid()
        res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stderr)
        os.replace(tmp, LIB)
    finally:
        for obj in objs:
            if os.path.exists(obj):
                os.remove(obj)
    return LIB


def built_digest():
    """The digest stored in the built library, or None when there is no library or it carries none.  Read from the
    file's bytes (the library holds the text "gemm-build-id:<digest>"), not by loading it: loading would pull in the
    system HIP runtime before PyTorch has loaded its own."""
    import re
    if not os.path.exists(LIB):
        return None
    with open(LIB, "rb") as f:
        m = re.search(rb"gemm-build-id:([0-9a-f]{32})", f.read())
    return m.group(1).decode() if m else None


def is_stale() -> bool:
    """True when there is no library or it was built from other sources or flags than the ones on disk (file times
    play no part: they do not survive every way a tree is copied)."""
    return built_digest() != source_digest()


if __name__ == "__main__":
    print(build(verbose=True))
