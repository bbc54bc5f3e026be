"""A property of the generated gfx950 code that the decode tile kernel relies on and that the
compiler does not guarantee by itself; checked on the assembly hipcc emits (no GPU needed)."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2402_14808_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _device_asm(name):
    src = os.path.join(ROOT, "paper_2402_14808_amd", "csrc", name + ".hip")
    flags = [f for f in build.FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, name + ".s")
        cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + flags + ["--cuda-device-only", "-S", src, "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return open(out).read()


@pytest.fixture(scope="module")
def tile_kernel_asm():
    return _device_asm("relay_tiles")


@pytest.fixture(scope="module")
def rows_kernel_asm():
    return _device_asm("relay_rows")


def test_tile_kernels_use_no_scratch_memory(tile_kernel_asm):
    """A kernel that spills vector registers needs scratch memory set up at every wavefront
    launch; that alone cost 3 us of a 30 us decode step when it happened."""
    sizes = re.findall(r"\.private_segment_fixed_size:\s*(\d+)", tile_kernel_asm)
    spills = re.findall(r"\.vgpr_spill_count:\s*(\d+)", tile_kernel_asm)
    assert len(sizes) >= 10 and all(int(x) == 0 for x in sizes), sizes
    assert all(int(x) == 0 for x in spills), spills


def test_many_rows_kernels_use_no_scratch_memory(rows_kernel_asm):
    sizes = re.findall(r"\.private_segment_fixed_size:\s*(\d+)", rows_kernel_asm)
    spills = re.findall(r"\.vgpr_spill_count:\s*(\d+)", rows_kernel_asm)
    assert len(sizes) >= 2 and all(int(x) == 0 for x in sizes), sizes
    assert all(int(x) == 0 for x in spills), spills


@pytest.mark.parametrize("which", ["tiles", "rows"])
def test_m0_belongs_to_the_lds_loads_alone(which, tile_kernel_asm, rows_kernel_asm):
    """The many-rows item loads K/V into LDS with a hand-written global_load_lds_dwordx4 that sets
    M0 (the LDS base) itself, without telling the compiler: every other use of M0 in these
    kernels would be a conflict.  Every write of M0 must be the statement's own, directly in front
    of its load, and nothing else may read or write it."""
    text = tile_kernel_asm if which == "tiles" else rows_kernel_asm
    lines = [l.strip() for l in text.splitlines() if l.strip() and not l.strip().startswith(";")]
    loads = 0
    for i, l in enumerate(lines):
        if not re.search(r"\bm0\b", l):
            continue
        assert re.fullmatch(r"s_mov_b32 m0, s\d+", l), l
        assert lines[i + 1].startswith("s_nop") and lines[i + 2].startswith("global_load_lds_dwordx4"), lines[i:i + 3]
        loads += 1
    assert loads == sum(1 for l in lines if l.startswith("global_load_lds_dwordx4")) and loads > 0
