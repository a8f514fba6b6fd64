"""Compiles the CPU oracle (plain C, gcc) into oracle/libfastpoint_ref.so.

Test infrastructure: only tests/, the smoke check and the benchmark's
cpu_baseline leg use the result.  -ffp-contract=off and no -ffast-math keep
every binary32 operation separately rounded.

build(sanitize=True) (or FASTPOINT_ORACLE_SANITIZE=1 in the environment of a process that
loads the oracle) builds and returns oracle/libfastpoint_ref_san.so instead: the same source
with -fsanitize=address,undefined and no recovery, so that an access out of bounds, a signed
overflow or a misaligned access inside the oracle aborts the process.  Python itself is not
built with the sanitizer, so such a process has to be started with the AddressSanitizer
runtime preloaded (asan_runtime() names it) and leak detection off."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fastpoint_ref.c")
LIB = os.path.join(HERE, "libfastpoint_ref.so")
LIB_SAN = os.path.join(HERE, "libfastpoint_ref_san.so")
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
          "-Wall", "-Wextra"]
SANFLAGS = ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]


def asan_runtime() -> str:
    """Path of the AddressSanitizer runtime that gcc links sanitized code against."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True,
                          stdout=subprocess.PIPE).stdout.decode().strip()


def build(force: bool = False, sanitize: bool = None) -> str:
    if sanitize is None:
        sanitize = os.environ.get("FASTPOINT_ORACLE_SANITIZE", "") == "1"
    lib = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    flags = CFLAGS + (SANFLAGS if sanitize else [])
    subprocess.run(["gcc", *flags, "-o", lib, SRC, "-lm"], check=True)
    return lib


if __name__ == "__main__":
    import sys
    print(build(force=True, sanitize="--sanitize" in sys.argv[1:]))
