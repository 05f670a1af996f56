"""Compile oracle/oracle.c into oracle/liboracle.so (gcc, OpenMP, no FP contraction)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oracle.c")
LIB = os.path.join(HERE, "liboracle.so")

# x86-64-v3 (AVX2 + FMA) rather than -march=native: the library is built on one
# machine and carried to another.  fmaf() still compiles to a hardware fma;
# -ffp-contract=off keeps every other mul/add separately rounded.
FLAGS = ["-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall"]


# Checker build (CPU only): AddressSanitizer + UndefinedBehaviorSanitizer, no OpenMP (its runtime's
# own allocations drown the report), frame pointers for readable stacks.  Used as
#   LD_PRELOAD=$(gcc -print-file-name=libasan.so) ORACLE_SANITIZE=1 python -m pytest tests/test_oracle_pins.py
SAN_LIB = os.path.join(HERE, "liboracle_san.so")
SAN_FLAGS = ["-O1", "-g", "-march=x86-64-v3", "-ffp-contract=off", "-fsanitize=address,undefined",
             "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-shared", "-fPIC", "-Wall"]


def build_sanitized() -> str:
    tmp = SAN_LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc", *SAN_FLAGS, SRC, "-o", tmp, "-lm"])
    os.replace(tmp, SAN_LIB)
    return SAN_LIB


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc", *FLAGS, SRC, "-o", tmp, "-lm"])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    import sys
    print(build_sanitized() if "--sanitize" in sys.argv[1:] else build())
