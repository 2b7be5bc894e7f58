"""Compile the C oracle into oracle/liboracle_attn.so with gcc (host code only).

`build(sanitize=True)` makes a second library, oracle/liboracle_attn_san.so, instrumented with the host compiler's
address and undefined-behaviour sanitizers (no GPU code is involved); tests/test_oracle_sanitized.py runs the oracle's
pins against it.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oracle_attn.c")
LIB = os.path.join(HERE, "liboracle_attn.so")
LIB_SAN = os.path.join(HERE, "liboracle_attn_san.so")

COMMON = ["-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = True, sanitize: bool = False) -> str:
    lib = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"] if sanitize else ["-O2"]
    subprocess.run(["gcc"] + opt + COMMON + ["-o", lib, SRC, "-lm"], check=True)
    return lib


def sanitizer_runtime() -> str:
    """Path of the address sanitizer's runtime, which a process that loads the instrumented library must preload."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()


if __name__ == "__main__":
    print(build())
