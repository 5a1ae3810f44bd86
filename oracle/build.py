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


def build_sanitized() -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU
    involved): oracle/librtlynx_oracle_san.so. Load it in a process that preloads the ASan runtime."""
    lib = os.path.join(HERE, "librtlynx_oracle_san.so")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-shared", "-fPIC", SRC, "-o", lib, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


def sanitizer_runtime() -> str:
    """Path of gcc's libasan.so (to be put first in LD_PRELOAD of the process that loads the build above)."""
    out = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True)
    return os.path.realpath(out.stdout.strip())


if __name__ == "__main__":
    print(build(force=True))
