"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the C oracle, driven over
small shapes with exactly sized buffers, and the plain C++ headers that the kernels share with the host
(token-tile walk, state slices, convolution tile order).  GPU code cannot run under a sanitizer on this
hardware pool; these are the parts of the arithmetic and the index logic that can."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
       "-static-libasan"]


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env)
    sys.stdout.write(res.stdout)
    assert res.returncode == 0 and res.stdout.startswith("OK"), res.stdout[-2000:]


def test_oracle_under_sanitizers(tmp_path):
    exe = tmp_path / "oracle_san"
    subprocess.run(["gcc", "-std=c11", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra", *SAN,
                    os.path.join(ROOT, "tests", "host_oracle_sanitize.c"),
                    os.path.join(ROOT, "oracle", "linattn_oracle.c"), "-o", str(exe)], check=True)
    _run(exe)


def test_shared_host_headers_under_sanitizers(tmp_path):
    for src in ("host_tile_walk.cpp", "host_tconv_tiles.cpp"):
        exe = tmp_path / src.replace(".cpp", "_san")
        subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", *SAN, os.path.join(ROOT, "tests", src),
                        "-o", str(exe)], check=True)
        _run(exe)
