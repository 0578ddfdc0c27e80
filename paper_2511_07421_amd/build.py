"""Compile the library (paper_2511_07421_amd/liba3gnn.so) with hipcc: the HIP kernels for gfx950 and
the host-side CPU sampler."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "liba3gnn.so")
BUILD_DIR = os.path.join(HERE, "_build")
SOURCES = [os.path.join(HERE, "csrc", "a3gnn.hip"), os.path.join(HERE, "csrc", "a3cpu.cpp")]
HEADERS = [os.path.join(HERE, "csrc", name) for name in sorted(os.listdir(os.path.join(HERE, "csrc")))
           if name.endswith(".hpp")] + [os.path.join(ROOT, "include", "a3gnn.h"),
                                        os.path.join(ROOT, "include", "a3gnn_cpu.h")]


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cxx = os.environ.get("CXX", "g++")
    os.makedirs(BUILD_DIR, exist_ok=True)
    cpu_obj = os.path.join(BUILD_DIR, "a3cpu.o")
    # the host sampler is plain C++ (it picks its vector code at run time): the host compiler
    host = [cxx, "-O3", "-std=c++17", "-fPIC", "-pthread", "-Wall", "-I", os.path.join(ROOT, "include"),
            "-c", SOURCES[1], "-o", cpu_obj]
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument", "-pthread",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
           "-o", LIB, cpu_obj, SOURCES[0]]  # the object first: what follows a .hip source is read as HIP
    for name, c in (("host compiler", host), ("hipcc", cmd)):
        if verbose:
            print(" ".join(c))
        res = subprocess.run(c, cwd=HERE, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        # hipcc's host pass does not know the packed-fp32 target feature and says so once per use: noise
        lines = [ln for ln in res.stdout.splitlines() if "packed-fp32-ops" not in ln]
        if res.returncode != 0:
            raise RuntimeError(name + " failed:\n" + "\n".join(lines))
        if verbose and lines:
            print("\n".join(lines))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
