"""Compile libgemm_f64.so for gfx950 with hipcc (in-tree, next to this file)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgemm_f64.so")
SOURCES = [os.path.join(CSRC, "gemm_f64.hip"), os.path.join(CSRC, "gemm_f32.hip")]
DEPENDS = SOURCES + [os.path.join(CSRC, "gemm_mfma.hpp"), os.path.join(CSRC, "gemm_host.hpp"),
                     os.path.join(os.path.dirname(HERE), "include", "gemm_f64.h"),
                     os.path.join(os.path.dirname(HERE), "include", "gemm_f32.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         # keep hipcc from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def build(verbose: bool = False, save_temps_dir: str = None) -> str:
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, *FLAGS, *SOURCES, "-o", tmp]
    if save_temps_dir:
        os.makedirs(save_temps_dir, exist_ok=True)
        cmd += ["-save-temps=obj"]
    res = subprocess.run(cmd, capture_output=True, text=True, cwd=save_temps_dir or None)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in res.stderr.splitlines() if noise not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    os.replace(tmp, LIB)
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in DEPENDS)


if __name__ == "__main__":
    print(build(verbose=True))
