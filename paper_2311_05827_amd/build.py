"""Build libaccept.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc.

Usage: ``python -m paper_2311_05827_amd.build`` or ``build()`` from Python.  The library
lands next to this file; it is git-ignored but travels with the working tree.
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
LIB_PATH = os.path.join(HERE, "libaccept.so")
SOURCES = ["api.hip", "uniform.hip", "mbq.hip"]

HIPCC_FLAGS = [
    "-O3",
    "--offload-arch=gfx950",
    "-std=c++17",
    "-fPIC",
    "-ffp-contract=off",           # the quantizer's multiply and add must stay two roundings
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # The encoder's work-queue atomic is issued by one lane and its answer is looked at an item
    # later; the atomic optimizer would rewrite it into a form that waits for the answer at once.
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"),
    "-I", CSRC,
]


def hipcc_path():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found (looked at $HIPCC, /opt/rocm/bin/hipcc, PATH)")


def _compile(hipcc, src, obj):
    cmd = [hipcc] + HIPCC_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    return src, r.returncode, (r.stdout + r.stderr), " ".join(cmd)


def build(verbose=True):
    """Compile every HIP source and link libaccept.so.  Always recompiles."""
    hipcc = hipcc_path()
    lib_path = LIB_PATH
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        results = list(ex.map(lambda so: _compile(hipcc, so[0], so[1]), zip(SOURCES, objs)))
    for src, rc, out, cmd in results:
        noise = "packed-fp32-ops' is not a recognized feature"
        shown = "\n".join(l for l in out.splitlines() if noise not in l)
        if rc != 0:
            raise RuntimeError("hipcc failed on %s\n%s\n%s" % (src, cmd, out))
        if verbose and shown.strip():
            print(shown, file=sys.stderr)
    tmp = lib_path + ".tmp"
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    r = subprocess.run(link, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed\n%s\n%s" % (" ".join(link), r.stdout + r.stderr))
    os.replace(tmp, lib_path)
    if verbose:
        print("built", lib_path, file=sys.stderr)
    return lib_path


if __name__ == "__main__":
    build()
