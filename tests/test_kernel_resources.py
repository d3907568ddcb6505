"""Compile-only checks of the gfx950 code objects (no GPU needed): two mistakes that do not show up as
compile errors and that cost this code base dearly when they happened.

* A register array that the compiler cannot keep in registers (an array of HIP's uint4 struct behind a
  generic lambda, a dynamically indexed array) lands in scratch memory: the kernel still computes the
  right values, several times slower.  Every kernel must have a private segment of 0 bytes.
* Inline assembly next to MFMAs is not covered by the compiler's hazard handling (the wait states an MFMA
  needs after a VALU write of its operands): no kernel may contain an inline-assembly block.
"""
import glob
import os
import re
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCES = sorted(glob.glob(os.path.join(ROOT, "paper_2602_02711_amd", "csrc", "*.hip")))
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "--cuda-device-only", "-S"]
SCRATCH_ALLOWED = {}        # file name -> bytes per lane (none accepted at present)


def device_asm(src):
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        proc = subprocess.run(["hipcc", *FLAGS, src, "-o", out], capture_output=True, text=True)
        assert proc.returncode == 0, proc.stderr[-2000:]
        return open(out).read()


@pytest.fixture(scope="module")
def listings():
    with ThreadPoolExecutor(max_workers=4) as pool:
        return dict(zip(SOURCES, pool.map(device_asm, SOURCES)))


def test_no_kernel_uses_scratch_memory(listings):
    for src, text in listings.items():
        sizes = [int(v) for v in re.findall(r"\.private_segment_fixed_size:\s*(\d+)", text)]
        limit = SCRATCH_ALLOWED.get(os.path.basename(src), 0)
        assert all(v <= limit for v in sizes), (os.path.basename(src), max(sizes))


def test_no_inline_assembly_in_kernels(listings):
    for src, text in listings.items():
        assert "#ASMSTART" not in text, os.path.basename(src)
