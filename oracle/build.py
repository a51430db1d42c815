"""Builds the CPU oracle (test infrastructure) into oracle/libams_oracle.so with g++."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libams_oracle.so")


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "ams_oracle.cpp")
    hdr = os.path.join(HERE, "ams_oracle.h")
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(src), os.path.getmtime(hdr)):
        return LIB
    cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-pthread",
           "-Wall", "-Wextra", "-o", LIB, src]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
