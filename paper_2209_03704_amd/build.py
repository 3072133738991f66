"""Build libkst.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2209_03704_amd.build [--incremental]

Every .hip file under csrc/ is compiled to an object (in parallel) and linked
into paper_2209_03704_amd/libkst.so.  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import concurrent.futures
import glob
import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libkst.so")

HIPCC = os.environ.get("HIPCC") or shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # Keep the compiler from forming packed-fp32 instructions.
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _up_to_date(src: str, obj: str) -> bool:
    """True when obj is newer than src, this script and every project header the compiler read
    for it last time (the .d file written beside the object)."""
    dep = obj + ".d"
    if not (os.path.exists(obj) and os.path.exists(dep)):
        return False
    t = os.path.getmtime(obj)
    names = open(dep).read().replace("\\\n", " ").split()
    deps = [n for n in names[1:] if n.endswith((".h", ".hip")) and not n.startswith("/opt/")] + [src, __file__]
    return all(os.path.exists(d) and os.path.getmtime(d) < t for d in deps)


def _compile(src: str, force: bool = True) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    if not force and _up_to_date(src, obj):
        return obj
    r = subprocess.run([HIPCC, *FLAGS, "-MD", "-MF", obj + ".d", "-c", src, "-o", obj], capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(jobs: int | None = None, force: bool = True) -> str:
    """Compile and link.  force=False recompiles only sources whose object is older than the source or one of
    the headers it includes: for iterating; the default compiles everything."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    if not srcs:
        raise RuntimeError("no sources under " + CSRC)
    jobs = jobs or min(len(srcs), int(os.environ.get("MAX_JOBS", "8")))
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda src: _compile(src, force), srcs))
    tmp = LIB + ".tmp.%d" % os.getpid()
    r = subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(force="--incremental" not in sys.argv))
