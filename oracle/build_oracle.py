"""Compiles the CPU oracle (test infrastructure) into oracle/libdynoracle.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "dyn_oracle.cpp")
LIB = os.path.join(HERE, "libdynoracle.so")


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
           "-shared", "-fPIC", SRC, "-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


SAN_LIB = os.path.join(HERE, "libdynoracle_san.so")


def build_sanitized(force: bool = False) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (host code only).  A process that loads it
    needs the sanitizer runtime preloaded: see asan_runtime()."""
    if not force and os.path.exists(SAN_LIB) and os.path.getmtime(SAN_LIB) >= os.path.getmtime(SRC):
        return SAN_LIB
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-Wall", "-Wextra", "-shared", "-fPIC", SRC,
           "-o", SAN_LIB]
    subprocess.run(cmd, check=True)
    return SAN_LIB


def asan_runtime() -> str:
    """Path of the compiler's AddressSanitizer runtime (to be preloaded ahead of everything else)."""
    return subprocess.run(["g++", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
