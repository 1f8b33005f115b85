"""Host-only tests of the library's index logic (no GPU): the tile geometry shared by the convolution
kernels is compiled for the host and checked by brute force against the definition of a 3x3 pad-1
neighbourhood.  The same check, and a driver that calls every routine of the C oracle on exactly-sized
heap buffers, also run under AddressSanitizer and UndefinedBehaviorSanitizer (host code only)."""
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


def _has_sanitizer_report(text: str) -> bool:
    return "AddressSanitizer" in text or "runtime error" in text or "LeakSanitizer" in text


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not available")
def test_tile_geometry_under_host_sanitizers(tmp_path):
    exe = str(tmp_path / "tile_geom_check_san")
    src = os.path.join(ROOT, "tests", "host", "tile_geom_check.cpp")
    # (host pass only: each sanitizer option follows an -Xarch_host of its own)
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Wno-unused-value",
                           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                           "-Xarch_host", "-fno-sanitize-recover=all", "-o", exe, src], stderr=subprocess.DEVNULL)
    assert int(subprocess.run(["nm", exe], capture_output=True, text=True).stdout.count("__asan")) > 0
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.startswith("ok "), out.stdout + out.stderr
    assert not _has_sanitizer_report(out.stderr)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_routines_under_host_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize_check")
    src = os.path.join(ROOT, "tests", "host", "oracle_sanitize_check.c")
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", "-o", exe, src, "-lm"])
    env = dict(os.environ, OMP_NUM_THREADS="4")
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert out.returncode == 0 and out.stdout.strip() == "ok", out.stdout + out.stderr
    assert not _has_sanitizer_report(out.stderr)
