"""Compile the CPU oracle (test infrastructure) into oracle/libee_oracle.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libee_oracle.so")


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "ee_oracle.cpp")
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(src):
        return LIB
    cmd = ["g++", "-std=c++17", "-O3", "-mavx2", "-fopenmp", "-ffp-contract=off", "-fPIC",
           "-shared", "-Wall", "-Wextra", "-o", LIB, src]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build())
