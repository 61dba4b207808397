"""Build libprism.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2508_12851_amd.build [--define NAME=VALUE ...]

--define passes -DNAME=VALUE to every compilation: for measurements that vary a compile-time
constant of the kernels (a plain rebuild afterwards restores the library everything else uses).

Each .hip file under csrc/ is compiled to an object in _build/ (in parallel),
then linked into paper_2508_12851_amd/libprism.so.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
BUILD = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libprism.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "is not a recognized feature" not in l)
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def build_library(verbose: bool = True, jobs: int = 8, defines=()) -> str:
    os.makedirs(BUILD, exist_ok=True)
    srcs = sources()
    flags = FLAGS + ["-D" + d for d in defines]
    objs = [os.path.join(BUILD, os.path.basename(s)[:-4] + ".o") for s in srcs]

    def compile_one(pair):
        s, o = pair
        out = _run([HIPCC, *flags, "-c", s, "-o", o])
        return s, out

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for s, out in ex.map(compile_one, zip(srcs, objs)):
            if verbose:
                print("[build] compiled", os.path.relpath(s, ROOT), flush=True)
                if out.strip():
                    print(out)
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if verbose:
        print("[build] linked", os.path.relpath(LIB, ROOT), flush=True)
    return LIB


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--define", action="append", default=[], metavar="NAME=VALUE")
    build_library(defines=ap.parse_args().define)
    sys.exit(0)
