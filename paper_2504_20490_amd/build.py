"""Compile libhspmd_attn.so for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIBRARY = os.path.join(HERE, "libhspmd_attn.so")
SOURCES = ["hspmd_attn_api.hip", "schedule.cpp", "fwd_kernel.hip", "bwd_kernels.hip", "bwd_dkv_kernel.hip", "merge_kernel.hip", "probe.hip", "rope_kernel.hip"]
HEADERS = ["attn_device.hpp", "kernels.hpp", "schedule.hpp", os.path.join("..", "..", "include", "hspmd_attn.h")]

# Packed fp32 VALU forms are switched off for all device code of this library.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _stale() -> bool:
    if not os.path.exists(LIBRARY):
        return True
    built = os.path.getmtime(LIBRARY)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return any(os.path.getmtime(d) > built for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not _stale():
        return LIBRARY
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-shared", "-o", LIBRARY]
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        cmd += (["-x", "hip", path] if s.endswith(".cpp") else [path])
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIBRARY


if __name__ == "__main__":
    print(build(verbose=True))
