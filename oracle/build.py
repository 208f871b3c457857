"""Compile the CPU oracle (plain C, gcc) into oracle/libsocket_oracle.so.

Test infrastructure: the shared object built here is loaded only by the tests,
the smoke check and the benchmark's CPU-baseline leg.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "socket_oracle.c")
LIB = os.path.join(HERE, "libsocket_oracle.so")


LIB_SANITIZED = os.path.join(HERE, "libsocket_oracle_asan.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.check_call(cmd)
    return LIB


def build_sanitized() -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer (host code only;
    single-threaded, so that every report names one plain loop).  To load it the process must
    have the sanitizer runtime preloaded: see sanitizer_runtime()."""
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-Wno-unknown-pragmas",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-o", LIB_SANITIZED, SRC, "-lm"]
    subprocess.check_call(cmd)
    return LIB_SANITIZED


def sanitizer_runtime() -> str:
    """Path of gcc's libasan.so, to be put first in LD_PRELOAD of a process that loads the sanitized build."""
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
