"""Build libchn.so (the C-ABI HIP library) in-tree for gfx950.

``python -m paper_1908_00213_amd.build`` compiles every translation unit under ``csrc/`` with hipcc
(objects in parallel, then one link) into ``paper_1908_00213_amd/libchn.so``.  hipcc cross-compiles
without a GPU.
"""
import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libchn.so")

SOURCES = ["host.cpp", "elementwise.hip", "reduce.hip", "gemm.hip", "lstm.hip", "softmax_ce.hip",
           "sgd.hip", "embed.hip"]

FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function",
         "-Wno-unknown-warning-option", "-Wno-unused-command-line-argument"]


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src, force, extra):
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    deps = [os.path.join(CSRC, src), os.path.join(CSRC, "common.h"),
            os.path.join(ROOT, "include", "chn.h")]
    if force or _stale(obj, deps):
        cmd = ["hipcc"] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        return src, r.stderr
    return src, ""


def build(force=False, verbose=False, extra=()):
    os.makedirs(OBJ, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        for src, err in ex.map(lambda s: _compile(s, force, list(extra)), SOURCES):
            if verbose and err.strip():
                print("[%s]\n%s" % (src, err))
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    if force or _stale(LIB, objs):
        cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
