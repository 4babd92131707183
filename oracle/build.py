"""Compile the C oracle into oracle/liboea_oracle.so with gcc (no HIP, no GPU)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oea_oracle.c")
LIB = os.path.join(HERE, "liboea_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    # -O2 without -ffast-math: the compiler may not reorder the fp64 sums.
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.check_call(cmd)
    return LIB


SAN_EXE = os.path.join(HERE, "oracle_sanitize")


def build_sanitized() -> str:
    """The oracle and its driver (sanitize_main.c) as one executable under AddressSanitizer and
    UndefinedBehaviorSanitizer; a report aborts the run (-fno-sanitize-recover)."""
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", SAN_EXE, SRC, os.path.join(HERE, "sanitize_main.c"),
           "-lm"]
    subprocess.check_call(cmd)
    return SAN_EXE


if __name__ == "__main__":
    print(build(force=True))
    if sys.argv[1:2] == ["--sanitize"]:
        print(build_sanitized())
    sys.exit(0)
