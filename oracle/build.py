"""Compiles the CPU oracle (plain C, gcc) into oracle/libfastpoint_ref.so.

Test infrastructure: only tests/, the smoke check and the benchmark's
cpu_baseline leg use the result.  -ffp-contract=off and no -ffast-math keep
every binary32 operation separately rounded."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fastpoint_ref.c")
LIB = os.path.join(HERE, "libfastpoint_ref.so")
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
          "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    subprocess.run(["gcc", *CFLAGS, "-o", LIB, SRC, "-lm"], check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
