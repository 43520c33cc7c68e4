"""Builds libedl.so (HIP kernels + C boundary) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libedl.so")
SOURCES = ["edl_api.cpp", "host_logic.cpp", "pipeline.cpp", "profiler.cpp", "tune.cpp", "k_update.hip", "k_norm.hip", "k_misc.hip", "k_conv.hip"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-result",
         # packed-fp32 arithmetic is switched off for device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False, extra=(), lib=LIB) -> str:
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(HERE, "_build", s + ".o")
        objs.append(obj)
        cmd = ["hipcc", "-x", "hip", "-c", src, "-o", obj] + FLAGS + list(extra)
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for s, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            failed = True
            print("== %s failed ==\n%s" % (s, out), file=sys.stderr)
        elif verbose and out.strip():
            print("== %s ==\n%s" % (s, out))
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.run(["hipcc", "-shared", "-o", lib] + objs + ["--offload-arch=gfx950", "-lpthread"], check=True)
    return lib


if __name__ == "__main__":
    print(build(verbose=True))
