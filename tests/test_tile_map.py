"""The workgroup -> tile mapping of the tiled projection kernels is plain C++ shared by host and device
(csrc/tile_map.h); a host program checks it exhaustively over matrix widths, k lengths and 1..200 token
tiles: every tile exactly once, nothing outside the matrix, and the shares of the eight XCDs equal up to
the partly empty last window of each band."""
import os
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_tile_mapping_covers_every_tile_once_and_balances_the_xcds():
    src = os.path.join(ROOT, "tests", "tile_map_check.cpp")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "tile_map_check")
        subprocess.run(["g++", "-O2", "-std=c++17", "-o", exe, src], check=True)
        r = subprocess.run([exe], capture_output=True, text=True)
    sys.stdout.write(r.stdout)
    assert r.returncode == 0 and r.stdout.strip().startswith("ok"), r.stdout + r.stderr
