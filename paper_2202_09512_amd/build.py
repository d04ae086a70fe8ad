"""Build libnnrescal.so (HIP, gfx950) next to this file.  Usage: python -m paper_2202_09512_amd.build"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = ["kernels_small.hip", "kernels_tiny.hip", "kernels_update.hip", "kernels_dense.hip", "kernels_sparse.hip", "api.hip", "select.hip", "start.hip", "transpose.hip", "validate.hip"]
LIB = os.path.join(HERE, "libnnrescal.so")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         # packed-fp32 instructions are switched off for all device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def build(verbose=True):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    objs, procs = [], []
    for f in SRC:
        o = os.path.join(bdir, f.replace(".hip", ".o"))
        objs.append(o)
        cmd = [hipcc, *FLAGS, "-I", os.path.join(HERE, "..", "include"), "-c", os.path.join(HERE, "csrc", f), "-o", o]
        procs.append((f, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for f, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {f}:\n{out}")
        if verbose and out.strip():
            print(out)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
