"""Compile the HIP sources into paper_2501_16383_amd/librkv.so for gfx950 (MI355X)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librkv.so")
SOURCES = ["rkv_api.hip", "rkv_kernels.hip", "rkv_append_mfma.hip", "rkv_select.hip", "rkv_decode_general.hip", "rkv_decode_mfma.hip", "rkv_decode_row.hip"]
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


def _stamp(src: str, cflags) -> str:
    """What an object depends on: its source, every header of the library, the flags."""
    import hashlib
    h = hashlib.sha256(" ".join(cflags).encode())
    deps = [os.path.join(CSRC, src)] + sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h"))
    deps.append(os.path.join(HERE, "..", "include", "rkv.h"))
    for d in deps:
        with open(d, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def source_hash() -> str:
    """SHA-256 over the kernel sources and headers (names and contents, in name order): what a
    counter profile was taken on, so that a figure quoted from it can be tied to the code that runs."""
    import hashlib
    h = hashlib.sha256()
    files = sorted(f for f in os.listdir(CSRC) if f.endswith((".hip", ".h")))
    for name in files + ["../../include/rkv.h"]:
        h.update(os.path.basename(name).encode() + b"\0")
        with open(os.path.join(CSRC, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def build_library(verbose: bool = False, incremental: bool = False) -> str:
    """One object per source file, compiled side by side (the decode kernel's many variants take most
    of the time), then linked into the shared library.  incremental: keep the objects under _build/
    and recompile only the sources whose text, headers or flags changed (a developer's shortcut; the
    default compiles everything)."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    extra = os.environ.get("RKV_EXTRA_HIPCC_FLAGS", "").split()     # tuning experiments only
    cflags = [f for f in FLAGS if f != "-shared"] + extra
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    with tempfile.TemporaryDirectory(prefix="obj_", dir=bdir) as tmp:
        odir = os.path.join(bdir, "inc") if incremental else tmp
        os.makedirs(odir, exist_ok=True)
        objs = [os.path.join(odir, os.path.splitext(src)[0] + ".o") for src in SOURCES]
        jobs = []
        for src, obj in zip(SOURCES, objs):
            stamp = _stamp(src, cflags) if incremental else ""
            if incremental and os.path.exists(obj) and os.path.exists(obj + ".stamp") and open(obj + ".stamp").read() == stamp:
                continue
            jobs.append(([hipcc(), *cflags, "-c", os.path.join(CSRC, src), "-o", obj], obj, stamp))

        def one(job):
            cmd, obj, stamp = job
            _run(cmd, verbose)
            if incremental:
                with open(obj + ".stamp", "w") as f:
                    f.write(stamp)
        if jobs:
            with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 1, 6)) as ex:
                list(ex.map(one, jobs))
        _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden", *objs, "-o", LIB + ".tmp"], verbose)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    if "--source-hash" in sys.argv[1:]:
        print(source_hash())
    else:
        print(build_library(verbose=True, incremental="--incremental" in sys.argv[1:]))
