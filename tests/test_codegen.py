"""A property of the generated gfx950 code that the decode tile kernel relies on and that the
compiler does not guarantee by itself; checked on the assembly hipcc emits (no GPU needed)."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2402_14808_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def tile_kernel_asm():
    src = os.path.join(ROOT, "paper_2402_14808_amd", "csrc", "relay_tiles.hip")
    flags = [f for f in build.FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "relay_tiles.s")
        cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + flags + ["--cuda-device-only", "-S", src, "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return open(out).read()


def test_tile_kernels_use_no_scratch_memory(tile_kernel_asm):
    """A kernel that spills vector registers needs scratch memory set up at every wavefront
    launch; that alone cost 3 us of a 30 us decode step when it happened."""
    sizes = re.findall(r"\.private_segment_fixed_size:\s*(\d+)", tile_kernel_asm)
    spills = re.findall(r"\.vgpr_spill_count:\s*(\d+)", tile_kernel_asm)
    assert len(sizes) >= 10 and all(int(x) == 0 for x in sizes), sizes
    assert all(int(x) == 0 for x in spills), spills
