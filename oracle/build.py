"""Compile the C oracle into oracle/libwgkv_oracle.so with gcc.

Test infrastructure only: the library built here is loaded by tests, by the
smoke check and by the benchmark's cpu_baseline leg, never by the product path.

`build(sanitize=True)` (or `python -m oracle.build --sanitize`) writes a second
library, oracle/libwgkv_oracle_san.so, compiled with AddressSanitizer and
UndefinedBehaviorSanitizer; the environment variable WGKV_ORACLE_LIB makes the
Python wrapper load it instead.  The CPU test suite under the sanitizers, from
the repository root (the sanitizer's runtime has to be loaded before Python's
own allocations, hence the preload, which is added to whatever is preloaded
already; Python itself never frees everything, so leak reports are off):

    python -m oracle.build --sanitize && \
    LD_PRELOAD="$(gcc -print-file-name=libasan.so)${LD_PRELOAD:+:$LD_PRELOAD}" \
    ASAN_OPTIONS=detect_leaks=0 UBSAN_OPTIONS=halt_on_error=1 \
    WGKV_ORACLE_LIB=oracle/libwgkv_oracle_san.so \
    python -m pytest tests -q -m "not gpu"
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "wgkv_oracle.c")
LIB = os.path.join(HERE, "libwgkv_oracle.so")
LIB_SANITIZED = os.path.join(HERE, "libwgkv_oracle_san.so")


def build(force: bool = True, sanitize: bool = False) -> str:
    lib = LIB_SANITIZED if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined"] if sanitize else ["-O2"]
    cmd = ["gcc", *opt, "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra", "-o", lib, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True, sanitize="--sanitize" in sys.argv[1:]))
    sys.exit(0)
