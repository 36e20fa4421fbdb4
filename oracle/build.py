"""Compile the CPU oracle (plain C + OpenMP) into oracle/liboracle.so.  Test infrastructure only."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "knn_softmax_oracle.c")
SRCS = [SRC, os.path.join(HERE, "topk_oracle.c")]
LIB = os.path.join(HERE, "liboracle.so")
LIB_SANITIZED = os.path.join(HERE, "liboracle_sanitized.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(p) for p in SRCS):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-ffp-contract=off", "-o", LIB] + SRCS + ["-lm"]
    subprocess.check_call(cmd)
    return LIB


def build_sanitized() -> str:
    """The same sources under AddressSanitizer and UndefinedBehaviorSanitizer (-O1, host code only), for the test that
    runs a small case of every exported function through it.  A process that loads it must have the sanitizer
    runtime loaded first (LD_PRELOAD of `gcc -print-file-name=libasan.so`)."""
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-o", LIB_SANITIZED] + SRCS + ["-lm"]
    subprocess.check_call(cmd)
    return LIB_SANITIZED


def sanitizer_runtime() -> str:
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
