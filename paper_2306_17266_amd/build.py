"""Compile the HIP library (csrc/) for gfx950 into paper_2306_17266_amd/libsushi.so with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsushi.so")
SOURCES = ["kernels.hip", "stream_kernel.hip", "model.cpp", "sched.cpp", "sushi_api.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def build(verbose=False):
    cmd = ["hipcc"] + FLAGS + ["-DSUSHI_BUILD"] + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


def build_tools():
    """The stand-alone measurement programs (not part of the library)."""
    out = os.path.join(HERE, "vmem_patterns")
    cmd = ["hipcc"] + [f for f in FLAGS if f not in ("-fPIC", "-shared")] + [os.path.join(CSRC, "vmem_patterns.hip"), "-o", out]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    return out


if __name__ == "__main__":
    import sys
    print(build(verbose=True))
    if "--tools" in sys.argv:
        print(build_tools())
