"""Compile the CPU oracle into oracle/libchoco_oracle.so (host only, g++).

Test infrastructure: nothing in the product package imports this module.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "choco_oracle.cpp")
LIB = os.path.join(HERE, "libchoco_oracle.so")

# No fused multiply-add and no value-changing optimisation: every product and
# sum in the oracle is rounded exactly where the source says.
FLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
         "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["g++"] + FLAGS + [SRC, "-o", tmp])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
