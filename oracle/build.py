"""Compile the CPU oracle into oracle/liblx_oracle.so with the host compiler."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "lx_oracle.cpp")
LIB = os.path.join(HERE, "liblx_oracle.so")
LIB_SAN = os.path.join(HERE, "liblx_oracle_san.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and \
            os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-fno-fast-math", "-ffp-contract=off", SRC, "-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized(force: bool = False) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (host code, CPU only):
    any finding aborts the process.  Loading it into Python needs the ASan runtime first in the
    library list (LD_PRELOAD=asan_runtime()); lx_oracle.py loads this library instead of the plain
    one when LX_ORACLE_SANITIZED=1."""
    if not force and os.path.exists(LIB_SAN) and \
            os.path.getmtime(LIB_SAN) >= os.path.getmtime(SRC):
        return LIB_SAN
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-fno-fast-math", "-ffp-contract=off", SRC, "-o", LIB_SAN]
    subprocess.run(cmd, check=True)
    return LIB_SAN


def asan_runtime() -> str:
    return subprocess.run(["g++", "-print-file-name=libasan.so"], check=True, capture_output=True,
                          text=True).stdout.strip()


if __name__ == "__main__":
    print(build())
