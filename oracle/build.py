"""Builds the C oracle (gcc, OpenMP) into oracle/libeinsum_ref.so.  Test infrastructure only."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "einsum_ref.c")
LIB = os.path.join(HERE, "libeinsum_ref.so")
# x86-64-v2 rather than the build machine's own instruction set: the library is built in one container and timed on
# another machine's host cores
FLAGS = ["-O3", "-march=x86-64-v2", "-fopenmp", "-std=c11", "-fno-fast-math"]
SAN_LIB = os.path.join(HERE, "_build", "libeinsum_ref_san.so")
SAN_FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-fopenmp", "-std=c11", "-fno-fast-math"]


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc"] + FLAGS + ["-fPIC", "-shared", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized() -> str:
    """The same source under the address and undefined-behaviour sanitizers (gcc's), for tests/test_host_sanitizers.py.
    A process that loads it must have gcc's libasan loaded first (LD_PRELOAD)."""
    os.makedirs(os.path.dirname(SAN_LIB), exist_ok=True)
    subprocess.run(["gcc"] + SAN_FLAGS + ["-fPIC", "-shared", "-o", SAN_LIB, SRC, "-lm"], check=True)
    return SAN_LIB


def sanitizer_runtime() -> str:
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()


if __name__ == "__main__":
    print(build(force=True))
