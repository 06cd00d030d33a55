"""Invariants of the compiled attention kernels that the source code relies on and the compiler does not check.

The global -> LDS copies are inline assembly that writes the M0 register (the copy's LDS base) without being able to
declare it (M0 is a reserved register): this is sound only while the compiler itself keeps nothing in M0 in these
kernels.  And the kernels order their copies by hand with `s_waitcnt vmcnt(N)` counts that assume no other vector
memory instruction of the wave is in flight inside the tile loops: a register spill (scratch traffic) would break
that count, besides costing time.  Both properties are read off the device assembly that hipcc emits for the
kernels' sources (no GPU needed)."""
import os
import re
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2504_20490_amd import build as lib_build

KERNEL_FILES = ["fwd_kernel.hip", "bwd_kernels.hip", "bwd_dkv_kernel.hip"]


def _device_asm(source: str) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = [hipcc, *lib_build.HIPCC_FLAGS, "-S", "--cuda-device-only", "-o", out, os.path.join(lib_build.CSRC, source)]
        proc = subprocess.run(cmd, capture_output=True, text=True)
        assert proc.returncode == 0, proc.stderr[-2000:]
        with open(out) as f:
            return f.read()


@pytest.fixture(scope="module")
def asm():
    with ThreadPoolExecutor(max_workers=3) as pool:
        return dict(zip(KERNEL_FILES, pool.map(_device_asm, KERNEL_FILES)))


@pytest.mark.parametrize("source", KERNEL_FILES)
def test_compiler_keeps_nothing_in_m0(asm, source):
    inside, uses, ours = False, [], 0
    for line in asm[source].splitlines():
        code = line.split(";")[0]
        if "#ASMSTART" in line:
            inside = True
        elif "#ASMEND" in line:
            inside = False
        elif re.search(r"\bm0\b", code):
            if inside:
                ours += 1
            else:
                uses.append(line.strip())
    assert ours > 0, "the copies' own M0 writes were not found: the check looks at the wrong text"
    assert not uses, f"compiler-generated uses of M0 next to the hand-written copies: {uses[:5]}"


@pytest.mark.parametrize("source", KERNEL_FILES)
def test_no_register_spills_in_the_attention_kernels(asm, source):
    text = asm[source]
    kernels = re.findall(r"^\s*\.amdhsa_kernel\s+(\S+)", text, flags=re.M)
    assert kernels
    spilled = re.findall(r"^\s*(scratch_(?:load|store)\S*)", text, flags=re.M)
    assert not spilled, f"{len(spilled)} scratch accesses (vector register spills) in {source}"
    for name, count in re.findall(r"^\s*\.amdhsa_kernel\s+(\S+).*?\.amdhsa_private_segment_fixed_size\s+(\d+)", text, flags=re.M | re.S):
        assert int(count) == 0, f"{name} uses {count} bytes of scratch memory per lane"
