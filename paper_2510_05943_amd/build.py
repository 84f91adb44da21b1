"""Builds libearl_dispatch.so (gfx950) in-tree with hipcc.  `python -m paper_2510_05943_amd.build`."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libearl_dispatch.so")
SOURCES = ("earl_api.hip", "earl_plan.hip", "earl_copy.hip", "earl_selector.cpp")


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


YARDSTICK_SRC = os.path.join(ROOT, "tests", "yardstick", "copy_ceiling.hip")
YARDSTICK_LIB = os.path.join(ROOT, "tests", "yardstick", "libcopy_ceiling.so")


def _compile(sources, out, includes, verbose):
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument"]
    for inc in includes:
        cmd += ["-I", inc]
    cmd += list(sources) + ["-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out


def build(verbose: bool = True) -> str:
    """The library, and the plain-copy yardstick the benchmark compares it with (a shared object
    of its own under tests/, not part of the library)."""
    _compile([os.path.join(CSRC, s) for s in SOURCES], LIB_PATH,
             [os.path.join(ROOT, "include"), CSRC], verbose)
    _compile([YARDSTICK_SRC], YARDSTICK_LIB, [], verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build())
