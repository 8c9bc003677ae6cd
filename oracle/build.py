"""Compile the C oracle with gcc into oracle/liboracle.so (test infrastructure only).

-ffp-contract=off keeps every fp32 operation of the pinned recipes a separate, individually rounded
IEEE operation (the fused steps are written as explicit fmaf calls); -mfma only makes fmaf fast.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "h1bkv_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")


def build(force: bool = False) -> str:
    # H1BKV_ORACLE_LIB names another build of the same source (the sanitizer build of the CPU test tier): used as it is
    other = os.environ.get("H1BKV_ORACLE_LIB")
    if other:
        return other
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-mfma", "-mpopcnt", "-Wall", "-Wextra", "-o", LIB + ".tmp", SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


def build_sanitized(out_path: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (any report aborts the process)."""
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-mfma", "-mpopcnt", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-Wall", "-Wextra", "-o", out_path, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return out_path


if __name__ == "__main__":
    print(build(force=True))
