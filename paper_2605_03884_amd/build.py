"""Compile the HIP kernels and the C ABI into paper_2605_03884_amd/libqkvcard.so for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqkvcard.so")
CLIENT_SRC = os.path.join(CSRC, "handoff_client.cpp")
CLIENT = os.path.join(HERE, "handoff_client")          # a plain HIP host program that links the library
SOURCES = ["api.hip", "classify.hip", "pack.hip", "unpack.hip", "assign.hip", "attend.hip", "controller.hip", "requant.hip"]

# -ffp-contract=off: every fused multiply-add in the kernels is written out, none is invented;
# packed fp32 instructions are switched off on this target.
FLAGS = ["-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950", "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument"]


def build(verbose=False):
    """Always recompiles (one object per source, in parallel, then one link); returns the library path."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]

    def compile_one(src):
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + compile_flags + ["-I", os.path.join(HERE, "..", "include"), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    build_client(verbose)
    return LIB


def build_client(verbose=False):
    """The example host program (no device code of its own), linked against the library beside it."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O2", "-std=c++17", "-Wall", "--offload-arch=gfx950", "-I", os.path.join(HERE, "..", "include"), CLIENT_SRC,
           "-o", CLIENT, "-L", HERE, "-lqkvcard", "-Wl,-rpath,$ORIGIN"]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return CLIENT


if __name__ == "__main__":
    print(build(verbose=True))
