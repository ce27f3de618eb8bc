"""Compile the HIP library (csrc/) for gfx950 into paper_2306_17266_amd/libsushi.so with hipcc.

Every source becomes an object file under csrc/_build/ (compiled side by side), then one link.
build(force=False) recompiles only sources that are newer than their object (or whose headers are)."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libsushi.so")
SOURCES = ["kernels.hip", "dwconv.hip", "conv_patch.hip", "int8.hip", "stream_kernel.hip", "team_kernel_mobile.hip", "model.cpp", "sched.cpp", "sushi_api.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose=False, force=True):
    os.makedirs(OBJ, exist_ok=True)
    sources = list(SOURCES)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(HERE, "..", "include", "sushi.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    jobs = []
    for s in sources:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s + ".o")
        stale = force or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), newest_header)
        if stale:
            jobs.append(["hipcc"] + FLAGS + ["-DSUSHI_BUILD", "-x", "hip", "-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        outs = list(pool.map(_run, jobs))
    outs.append(_run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] +
                     [os.path.join(OBJ, s + ".o") for s in sources] + ["-o", LIB]))
    if verbose:
        text = "\n".join(o for o in outs if o.strip())
        if text:
            print(text)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, force="--force" in sys.argv))
