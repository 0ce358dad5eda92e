"""Compile oracle/moe_oracle.c into oracle/libmoe_oracle.so with gcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "moe_oracle.c")
LIB = os.path.join(HERE, "libmoe_oracle.so")


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", tmp, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


CHECK_SRC = os.path.join(HERE, "sanitize_check.c")
CHECK_EXE = os.path.join(HERE, "sanitize_check")


def build_sanitize_check(sanitize: bool = True) -> str:
    """The oracle and its small driver (sanitize_check.c) as one executable under
    -fsanitize=address,undefined (static runtimes: another preloaded library must not come
    before them).  sanitize=False builds the same program plainly."""
    exe = CHECK_EXE + ("" if sanitize else "_plain")
    tmp = exe + f".tmp{os.getpid()}"
    flags = (["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
              "-static-libubsan", "-fno-omit-frame-pointer", "-g"] if sanitize else [])
    cmd = ["gcc", "-O1", "-std=c11", "-Wall", "-Wextra", "-Wno-unknown-pragmas", *flags, "-o", tmp, CHECK_SRC, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, exe)
    return exe


if __name__ == "__main__":
    print(build(force=True))
    print(build_sanitize_check())
