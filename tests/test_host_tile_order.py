"""Host logic shared with the kernels as plain C++ headers, compiled with g++ and run here: the
temporal convolution's workgroup-id -> tile order (every tile exactly once, balanced XCD shares)
and the attention kernels' token-tile walk (every tile of a range exactly once over all waves)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_tile_order_covers_every_tile_once(tmp_path):
    exe = tmp_path / "host_tconv_tiles"
    subprocess.run(["g++", "-O1", "-std=c++17", "-Wall", "-Wextra", os.path.join(ROOT, "tests", "host_tconv_tiles.cpp"),
                    "-o", str(exe)], check=True)
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, text=True)
    sys.stdout.write(res.stdout)
    assert res.returncode == 0 and res.stdout.startswith("OK")


def test_token_tile_walk_covers_every_tile_once(tmp_path):
    exe = tmp_path / "host_tile_walk"
    subprocess.run(["g++", "-O1", "-std=c++17", "-Wall", "-Wextra", os.path.join(ROOT, "tests", "host_tile_walk.cpp"),
                    "-o", str(exe)], check=True)
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, text=True)
    sys.stdout.write(res.stdout)
    assert res.returncode == 0 and res.stdout.startswith("OK")
