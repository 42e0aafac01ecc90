"""Compile the HIP sources under ``csrc/`` into ``libsom.so`` (gfx950 only), in-tree.

``python -m paper_1305_1422_amd.build`` or ``build(force=True)``.  hipcc cross-compiles
without a GPU.  Packed-fp32 instruction selection is switched off for every kernel.

Environment hooks for timing experiments with variant builds: ``SOM_EXTRA_FLAGS`` (extra hipcc
flags), ``SOM_LIB_OUT`` / ``SOM_OBJ_DIR`` (where the variant library and its objects go), ``HIPCC``.
The binding loads ``SOM_LIB_PATH`` instead of the in-tree library when that variable is set.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.environ.get("SOM_OBJ_DIR", os.path.join(HERE, "_build"))
LIB = os.environ.get("SOM_LIB_OUT", os.path.join(HERE, "libsom.so"))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC] + os.environ.get("SOM_EXTRA_FLAGS", "").split()


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    headers = glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    jobs = []
    objs = []
    for src in sources():
        obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        if force or _stale(obj, [src] + headers):
            jobs.append([HIPCC] + FLAGS + ["-c", src, "-o", obj])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + r.stdout + r.stderr)
        return r.stderr

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        for warn in pool.map(run, jobs):
            # the host pass does not know the packed-fp32 feature and says so: harmless
            warn = "\n".join(l for l in warn.splitlines() if "packed-fp32-ops" not in l and l.strip())
            if verbose and warn:
                print(warn)
    if jobs or force or _stale(LIB, objs):
        run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
