"""Host-only tests of the library's index logic (no GPU): the tile geometry shared by the convolution
kernels is compiled for the host and checked by brute force against the definition of a 3x3 pad-1
neighbourhood."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not available")
def test_tile_geometry_bruteforce(tmp_path):
    exe = str(tmp_path / "tile_geom_check")
    src = os.path.join(ROOT, "tests", "host", "tile_geom_check.cpp")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wno-unused-value", "-o", exe, src],
                          stderr=subprocess.DEVNULL)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout
    assert out.stdout.startswith("ok ") and int(out.stdout.split()[1]) > 3_000_000
