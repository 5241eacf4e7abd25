"""Compile the CPU oracle (test infrastructure) into oracle/libfadeo.so with the host compiler."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
# FADE_HOST_SANITIZE=1: a separate build with AddressSanitizer + UndefinedBehaviorSanitizer (host code only), for running
# the CPU tests once under the sanitizers: LD_PRELOAD=$(gcc -print-file-name=libasan.so) FADE_HOST_SANITIZE=1 pytest -m "not gpu"
SANITIZE = os.environ.get("FADE_HOST_SANITIZE") == "1"
LIB = os.path.join(HERE, "libfadeo_san.so" if SANITIZE else "libfadeo.so")


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "fadeo.cpp")
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(src), os.path.getmtime(os.path.join(HERE, "fadeo.h"))):
        return LIB
    cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB, src]
    if SANITIZE:
        cmd[3:3] = ["-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build())
