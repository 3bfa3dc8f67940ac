"""Compiles the HIP sources into paper_2510_02329_amd/libsj.so for gfx950 (in-tree, with hipcc).

Every source is compiled to an object of its own under _build/ (git-ignored) and the objects are linked;
`build_library(force=False)` reuses an object whose source and headers have not changed, which is what the
command line of this module does.  The driver's build check calls it with force=True: everything is compiled."""
from __future__ import annotations

import glob
import hashlib
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libsj.so")
OBJ_DIR = os.path.join(ROOT, "_build")
SOURCES = [os.path.join(HERE, "csrc", n) for n in ("sj_lib.hip", "sj_train.hip")]

FLAGS = [*os.environ.get("SJ_BUILD_DEFS", "").split(),
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        sys.stderr.write(out + "\n")
        raise RuntimeError("hipcc failed")
    if verbose and out.strip():
        print(out)


def _stamp(src: str) -> str:
    h = hashlib.sha256(" ".join(FLAGS).encode())
    for p in [src] + sorted(glob.glob(os.path.join(HERE, "csrc", "*.h"))) + sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        with open(p, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def build_library(verbose: bool = True, force: bool = True) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs, jobs = [], []
    for src in SOURCES:
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        stamp_file, stamp = obj + ".stamp", _stamp(src)
        objs.append(obj)
        fresh = (not force and os.path.exists(obj) and os.path.exists(stamp_file) and open(stamp_file).read() == stamp)
        if not fresh:
            jobs.append((src, obj, stamp_file, stamp))

    def compile_one(job):
        src, obj, stamp_file, stamp = job
        _run([hipcc, *FLAGS, "-c", "-o", obj, src], verbose)
        with open(stamp_file, "w") as f:
            f.write(stamp)

    with ThreadPoolExecutor(max_workers=4) as pool:
        list(pool.map(compile_one, jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH + ".tmp", *objs], verbose)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    build_library(force="--force" in sys.argv)
