"""Host logic of the temporal-convolution launch: the workgroup-id -> tile order (plain C++
shared with the kernel) covers every tile exactly once and balances the XCD shares."""
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
