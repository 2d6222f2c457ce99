"""Builds libsvlinattn.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libsvlinattn.so")
SOURCES = [os.path.join(CSRC, f) for f in ("sv_linattn.hip", "sv_tconv.hip", "sv_measure.hip")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # packed-fp32 VALU forms stay off (device-side feature; the host pass ignores it)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # The epoch ticket (EpochSource::begin) is one lane's fetch-and-add whose result is needed much later.  The
    # compiler's atomic optimizer would turn it into a wave-wide reduction that needs the result at once, and
    # the wave would wait for the atomic's round trip before its first load.
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    # per-kernel register, scratch and LDS use as compiler remarks (parsed below)
    "-Rpass-analysis=kernel-resource-usage",
]
RESOURCES = os.path.join(PKG, "kernel_resources.txt")   # written by build(): one line per kernel


def source_fingerprint() -> str:
    """Short hash of the kernel sources with comments and white space taken out: measurements that were
    made on one build (rocprofv3 counter runs kept as text) carry it, so a reader can tell whether the
    kernels have changed since."""
    import hashlib
    import re
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if not name.endswith((".hip", ".hpp")):
            continue
        with open(os.path.join(CSRC, name)) as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"//[^\n]*", "", text)
        h.update(name.encode())
        h.update("".join(text.split()).encode())
    return h.hexdigest()[:16]


def kernel_resources(compiler_output: str) -> dict:
    """{kernel name: {"VGPRs": n, "AGPRs": n, "ScratchSize": bytes per lane, "VGPRs Spill": n, ...}} from the
    kernel-resource-usage remarks in hipcc's output."""
    res, cur = {}, None
    for line in compiler_output.splitlines():
        if "[-Rpass-analysis=kernel-resource-usage]" not in line or "remark:" not in line:
            continue
        body = line.split("remark:", 1)[1].replace("[-Rpass-analysis=kernel-resource-usage]", "").strip()
        key, _, val = body.partition(":")
        key, val = key.strip(), val.strip()
        if key == "Function Name":
            cur = res.setdefault(val, {})
        elif cur is not None:
            cur[key.split(" [")[0]] = val
    return res


def check_resources(res: dict) -> None:
    """No kernel of the library may keep data in scratch memory: every one of them is written to fit its
    registers, and one that does not runs many times slower without failing any test."""
    bad = [f"{k}: scratch {v.get('ScratchSize')} B/lane, {v.get('VGPRs Spill')} VGPRs spilled"
           for k, v in res.items()
           if v.get("ScratchSize", "0") != "0" or v.get("VGPRs Spill", "0") != "0" or v.get("Dynamic Stack") == "True"]
    if bad:
        raise RuntimeError("kernels that use scratch memory:\n  " + "\n  ".join(bad))


def build(verbose: bool = False, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, *SOURCES, "-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    lines = [l for l in res.stdout.splitlines() if noise not in l]
    # the remarks come with three lines each (message, source line, caret): keep them out of the log
    out, skip = [], 0
    for l in lines:
        if "[-Rpass-analysis=kernel-resource-usage]" in l:
            skip = 2
        elif skip:
            skip -= 1
        else:
            out.append(l)
    out = "\n".join(out)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    usage = kernel_resources(res.stdout)
    if not usage:
        raise RuntimeError("hipcc printed no kernel resource remarks")
    check_resources(usage)
    with open(RESOURCES, "w") as f:
        for name in sorted(usage):
            u = usage[name]
            f.write(f"{name} VGPRs={u.get('VGPRs')} AGPRs={u.get('AGPRs')} scratch={u.get('ScratchSize')} "
                    f"lds={u.get('LDS Size')} waves_per_simd={u.get('Occupancy')}\n")
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
