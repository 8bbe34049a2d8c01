"""Build ``libbs.so`` and ``libbs_probe.so`` in-tree with hipcc for gfx950.

``python -m paper_1811_00206_amd.build`` compiles every ``csrc/*.hip`` into the
product library ``libbs.so`` and every ``probe/*.hip`` (measurement helpers for
the benchmark, not part of the method) into ``libbs_probe.so``, both next to
this file.  Cross-compilation needs no GPU.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
PROBE_SRC = os.path.join(HERE, "probe")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbs.so")
PROBE_LIB = os.path.join(HERE, "libbs_probe.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    # an unrolled loop with an early exit is unrolled by a later pass than the one that warns
    "-Wno-pass-failed",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def probe_sources():
    return sorted(glob.glob(os.path.join(PROBE_SRC, "*.hip")))


def _compile(src: str) -> str:
    obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
    subprocess.check_call([HIPCC, *FLAGS, "-c", src, "-o", obj])
    return obj


def _link(lib: str, objs) -> None:
    tmp = lib + f".tmp{os.getpid()}"
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, lib)


def build_library(verbose: bool = False) -> str:
    """Compile all sources (always; no staleness shortcut) and link libbs.so and
    libbs_probe.so."""
    os.makedirs(OBJDIR, exist_ok=True)
    srcs, psrcs = sources(), probe_sources()
    if not srcs:
        raise RuntimeError("no HIP sources found under " + CSRC)
    jobs = max(1, min(len(srcs) + len(psrcs), 8, os.cpu_count() or 1))
    with ThreadPoolExecutor(jobs) as ex:
        objs = list(ex.map(_compile, srcs + psrcs))
    _link(LIB, objs[:len(srcs)])
    if psrcs:
        _link(PROBE_LIB, objs[len(srcs):])
    if verbose:
        print("built", LIB, "and", PROBE_LIB)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)
    sys.exit(0)
