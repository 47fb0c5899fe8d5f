"""Builds libqflash.so (gfx950 only) in-tree with hipcc.

    python -m paper_2604_25306_amd.build            # compile every source, link
    python -m paper_2604_25306_amd.build --changed  # recompile only sources older than their object
"""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libqflash.so")
SOURCES = ["qflash_api.cpp", "qflash_plan.cpp", "qflash_kernels.hip", "qflash_qmax.hip", "qflash_cu.hip", "qflash_win.hip", "qflash_ring.hip", "qflash_dynamic.hip", "qflash_peaks.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]
_NOISE = "is not a recognized feature for this target"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if _NOISE not in l)
    if verbose and out.strip():
        print(out, flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)


def build(verbose: bool = True, only_changed: bool = False) -> str:
    """Compile every source for gfx950 (in parallel, one object each) and link libqflash.so next to
    this file.  only_changed: skip sources whose object is newer than the source and every header."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    jobs = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s + ".o")
        if only_changed and os.path.exists(obj) and \
                os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            continue
        jobs.append([hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC,
                                             "-x", "hip", "-c", src, "-o", obj])
    with concurrent.futures.ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        for f in [pool.submit(_run, cmd, verbose) for cmd in jobs]:
            f.result()
    tmp = LIB + ".tmp%d" % os.getpid()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wno-unused-command-line-argument"]
         + [os.path.join(OBJ, s + ".o") for s in SOURCES] + ["-o", tmp], verbose)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build(only_changed="--changed" in sys.argv[1:])
    sys.exit(0)
