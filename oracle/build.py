"""Compile the CPU oracle (test infrastructure) into oracle/liba3oracle.so with g++."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liba3oracle.so")


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "a3_oracle.cpp")
    hdr = os.path.join(HERE, "a3_oracle.h")
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(src), os.path.getmtime(hdr)):
        return LIB
    cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", LIB, src]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build())
