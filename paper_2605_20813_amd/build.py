"""Compile csrc/*.hip for gfx950 and link libpulsecol.so next to this file (plus the
stand-alone roofline probe that sits beside bench.py at the repository root).

Usage: ``python -m paper_2605_20813_amd.build`` (cross-compiles without a GPU).
"""

from __future__ import annotations

import concurrent.futures
import glob
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libpulsecol.so")
PROBE_SRC = os.path.join(os.path.dirname(HERE), "roofline_probe.hip")
PROBE_PATH = os.path.join(os.path.dirname(HERE), "roofline_probe.bin")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # let the register allocator put MFMA results that the VALU consumes straight into VGPRs
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wno-unused-command-line-argument",
]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False) -> str:
    """Compile every kernel translation unit and link the shared library; returns its path."""
    hipcc = _hipcc()
    os.makedirs(OBJ_DIR, exist_ok=True)
    sources = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    if not sources:
        raise RuntimeError("no sources under " + CSRC)
    objs = [os.path.join(OBJ_DIR, os.path.basename(s)[:-4] + ".o") for s in sources]

    def compile_one(pair):
        src, obj = pair
        return _run([hipcc, *HIPCC_FLAGS, "-c", src, "-o", obj])

    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(sources))) as ex:
        for out in ex.map(compile_one, zip(sources, objs)):
            if verbose and out.strip():
                print(out)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs])
    # the stand-alone roofline probe that bench.py starts as a child process (a measurement aid,
    # not part of the library: it lives beside bench.py)
    if os.path.exists(PROBE_SRC):
        _run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
              "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-o", PROBE_PATH, PROBE_SRC])
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
