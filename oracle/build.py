"""Compile the C oracle into ``oracle/liboracle_attn.so`` with gcc (host only)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(HERE, "attn_oracle.c")
LIBRARY = os.path.join(HERE, "liboracle_attn.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIBRARY) and os.path.getmtime(LIBRARY) >= os.path.getmtime(SOURCE):
        return LIBRARY
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIBRARY, SOURCE, "-lm"]
    subprocess.run(cmd, check=True)
    return LIBRARY


if __name__ == "__main__":
    print(build())
