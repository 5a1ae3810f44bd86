"""Compile the C oracle into oracle/librtlynx_oracle.so with gcc (no GPU toolchain involved)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "rtlynx_oracle.c")
LIB = os.path.join(HERE, "librtlynx_oracle.so")


def build(force: bool = False) -> str:
    stale = (not os.path.exists(LIB)) or os.path.getmtime(LIB) < os.path.getmtime(SRC)
    if force or stale:
        # -ffp-contract=off: the fp32 operation order of the oracle is part of its definition.
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC",
               SRC, "-o", LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
