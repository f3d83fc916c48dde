"""Compile the CPU oracle (test infrastructure) into oracle/libq4kv_oracle.so with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "q4kv_oracle.c")
LIB = os.path.join(HERE, "libq4kv_oracle.so")

# -ffp-contract=off and no -ffast-math: the quantizer's binary32 divisions and
# roundings must stay IEEE so that its output is defined bit for bit.
CMD = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
       "-o", LIB, SRC, "-lm"]


def build(force=True):
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(CMD)
    return LIB


if __name__ == "__main__":
    print(build())
