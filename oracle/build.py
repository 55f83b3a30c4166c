"""Compile the CPU oracle into oracle/liboracle.so (plain g++, generic x86-64, no GPU code)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ma_oracle.cpp")
OUT = os.path.join(HERE, "liboracle.so")

# -ffp-contract=off: no fused multiply-add unless the source asks for one with fmaf.
FLAGS = ["-O2", "-ffp-contract=off", "-std=c++17", "-shared", "-fPIC", "-pthread",
         "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    tmp = OUT + ".tmp.%d" % os.getpid()
    subprocess.run(["g++", *FLAGS, SRC, "-o", tmp], check=True)
    os.replace(tmp, OUT)
    return OUT


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
