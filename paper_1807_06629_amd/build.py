"""Builds libprsgd.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_1807_06629_amd.build

Each translation unit under csrc/ is compiled to an object in _build/ and the objects are
linked into paper_1807_06629_amd/libprsgd.so.  Packed-FP32 instruction selection is turned off
for all device code.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libprsgd.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "is not a recognized feature for this target" not in l)
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False) -> str:
    os.makedirs(BUILD, exist_ok=True)
    hipcc = _hipcc()
    sources = sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))
    objects = [os.path.join(BUILD, f[:-4] + ".o") for f in sources]

    def compile_one(pair):
        src, obj = pair
        return _run([hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=min(8, len(sources))) as pool:
        for log in pool.map(compile_one, zip(sources, objects)):
            if verbose and log.strip():
                print(log)
    log = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objects])
    if verbose and log.strip():
        print(log)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
