"""Builds the C-ABI library ``liblobra_mlora.so`` from ``csrc/`` with hipcc for gfx950.

The library is built in-tree (next to this file) so that it travels with the source tree.
``python -m paper_2509_01193_amd.build`` rebuilds it.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblobra_mlora.so")
CSRC_BENCH = os.path.join(HERE, "csrc_bench")                 # bench-only kernels (measured ceilings): their own library
LIB_CEILINGS = os.path.join(HERE, "liblobra_ceilings.so")
OBJ = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp")))


def headers():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(ROOT, "include", "lobra_mlora.h"))
    return hs


def build(force: bool = True, verbose: bool = False, defines=(), out: str = LIB, objdir: str = OBJ) -> str:
    """Compile every source (always, when force) and link the shared library.

    `defines` (e.g. ["LOBRA_GEMM_WM=2"]), `out` and `objdir` build a tuning variant next to the
    default library."""
    os.makedirs(objdir, exist_ok=True)
    newest_h = max(os.path.getmtime(h) for h in headers())

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        if (not force and os.path.exists(obj)
                and os.path.getmtime(obj) >= max(os.path.getmtime(src), newest_h)):
            return obj
        cmd = ([HIPCC] + FLAGS + ["-D" + d for d in defines]
               + (["-x", "hip"] if src.endswith(".hip") else []) + ["-c", src, "-o", obj])
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        if verbose and r.stderr.strip():
            print(r.stderr, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(4) as ex:
        objs = list(ex.map(compile_one, sources()))
    tmp = out + ".tmp%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    os.replace(tmp, out)
    return out


def build_ceilings(verbose: bool = False, out: str = LIB_CEILINGS) -> str:
    """The bench-only library of csrc_bench/ (never linked into, or loaded by, the product library)."""
    srcs = sorted(os.path.join(CSRC_BENCH, f) for f in os.listdir(CSRC_BENCH) if f.endswith(".hip"))
    tmp = out + ".tmp%d" % os.getpid()
    cmd = [HIPCC] + FLAGS + ["-shared", "-x", "hip"] + srcs + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (srcs, r.stdout, r.stderr))
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
    print(build_ceilings(verbose=True))
