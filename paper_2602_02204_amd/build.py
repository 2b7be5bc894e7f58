"""Compile the HIP library for gfx950 into paper_2602_02204_amd/libomni_attn.so (in-tree, so it travels with the repo)."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "omni_attn.hip")
LIB = os.path.join(HERE, "libomni_attn.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # hipcc must not form packed-fp32 instructions for these kernels
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return [SRC] + sorted(glob.glob(os.path.join(HERE, "csrc", "*.hpp"))) + [os.path.join(ROOT, "include", "omni_attn.h")]


def up_to_date() -> bool:
    return os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in sources())


def build(force: bool = True, extra=()) -> str:
    if not force and up_to_date():
        return LIB
    cmd = ["hipcc"] + FLAGS + list(extra) + ["-I", os.path.join(ROOT, "include"), "-o", LIB, SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build())
