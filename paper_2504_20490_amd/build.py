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


# what decides a kernel's HBM traffic: the attention kernels, their shared device code and the launch order
KERNEL_SOURCES = ["fwd_kernel.hip", "bwd_kernels.hip", "bwd_dkv_kernel.hip", "attn_device.hpp", "kernels.hpp",
                  "schedule.hpp", "schedule.cpp"]


def sources_digest() -> str:
    """sha256 (first 16 hex digits) over the attention kernels' sources: names the kernels a measurement was
    taken with, so that a stored figure can be told from one of an older build."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(KERNEL_SOURCES):
        with open(os.path.join(CSRC, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def _stale() -> bool:
    if not os.path.exists(LIBRARY):
        return True
    built = os.path.getmtime(LIBRARY)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return any(os.path.getmtime(d) > built for d in deps)


# Per-source flags (none at present; every source is compiled on its own, in parallel, and the objects are linked).
EXTRA_FLAGS: dict = {}
BUILD_DIR = os.path.join(HERE, "_build")


def _compile(hipcc: str, source: str) -> tuple:
    path = os.path.join(CSRC, source)
    obj = os.path.join(BUILD_DIR, os.path.splitext(source)[0] + ".o")
    cmd = [hipcc, *HIPCC_FLAGS, *EXTRA_FLAGS.get(source, []), "-c", "-o", obj]
    cmd += (["-x", "hip", path] if source.endswith(".cpp") else [path])
    proc = subprocess.run(cmd, capture_output=True, text=True)
    return obj, proc.returncode, proc.stderr


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not _stale():
        return LIBRARY
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(BUILD_DIR, exist_ok=True)
    noise = "is not a recognized feature for this target"
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        results = list(pool.map(lambda s: _compile(hipcc, s), SOURCES))
    errors = []
    for (obj, rc, stderr), source in zip(results, SOURCES):
        err = "\n".join(l for l in stderr.splitlines() if noise not in l)
        if rc != 0:
            raise RuntimeError(f"hipcc failed on {source}:\n" + err)
        if err.strip():
            errors.append(err)
    proc = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIBRARY, *[r[0] for r in results]],
                          capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("link failed:\n" + proc.stderr)
    if verbose and errors:
        print("\n".join(errors))
    return LIBRARY


if __name__ == "__main__":
    print(build(verbose=True))
