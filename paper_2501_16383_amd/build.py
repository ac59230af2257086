"""Compile the HIP sources into paper_2501_16383_amd/librkv.so for gfx950 (MI355X)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librkv.so")
SOURCES = ["rkv_api.hip", "rkv_kernels.hip", "rkv_append_mfma.hip", "rkv_select.hip", "rkv_decode_general.hip", "rkv_decode_mfma.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
    # packed-FP32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("packed-fp32-ops", "is not a recognized feature")
    err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in noise))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build_library(verbose: bool = False) -> str:
    """One object per source file, compiled side by side (the decode kernel's many variants take most
    of the time), then linked into the shared library."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    extra = os.environ.get("RKV_EXTRA_HIPCC_FLAGS", "").split()     # tuning experiments only
    cflags = [f for f in FLAGS if f != "-shared"]
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)        # objects live here for the duration of the build only
    with tempfile.TemporaryDirectory(prefix="obj_", dir=os.path.join(HERE, "_build")) as tmp:
        objs = [os.path.join(tmp, os.path.splitext(src)[0] + ".o") for src in SOURCES]
        jobs = [[hipcc(), *cflags, *extra, "-c", os.path.join(CSRC, src), "-o", obj] for src, obj in zip(SOURCES, objs)]
        with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 1, 6)) as ex:
            list(ex.map(lambda c: _run(c, verbose), jobs))
        _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden", *objs, "-o", LIB + ".tmp"], verbose)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
