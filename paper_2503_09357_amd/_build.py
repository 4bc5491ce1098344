"""Compile the native pieces of the package in-tree.

Two shared libraries live beside this file once built:

* ``libdagsched.so``          - HIP kernels for gfx950 plus the C-ABI (csrc/dagsched.hip)
* ``libdagsched_workload.so`` - seeded synthetic candidate generator (csrc/workload_gen.c)

Nothing here is executed on import; ``ensure_*`` build when the library is absent or older than
its sources, ``build_*`` always recompile.
"""
from __future__ import annotations

import os
import shutil
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG_DIR), "include")

HIP_LIB = os.path.join(PKG_DIR, "libdagsched.so")
GEN_LIB = os.path.join(PKG_DIR, "libdagsched_workload.so")

HIP_SOURCES = ["dagsched.hip"]


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), proc.stdout))
    return proc.stdout


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; the HIP library cannot be built")


def build_hip(verbose: bool = False) -> str:
    """hipcc -> libdagsched.so (gfx950 only)."""
    tmp = HIP_LIB + ".tmp"
    cmd = [
        _hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-function",
        "-I", INCLUDE,
        *[os.path.join(CSRC, s) for s in HIP_SOURCES],
        "-o", tmp,
    ]
    out = _run(cmd)
    os.replace(tmp, HIP_LIB)
    if verbose and out.strip():
        print(out)
    return HIP_LIB


def build_workload_gen() -> str:
    """gcc -> libdagsched_workload.so (host only)."""
    tmp = GEN_LIB + ".tmp"
    _run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall",
          os.path.join(CSRC, "workload_gen.c"), "-o", tmp])
    os.replace(tmp, GEN_LIB)
    return GEN_LIB


def _stale(lib: str, sources) -> bool:
    if not os.path.exists(lib):
        return True
    t = os.path.getmtime(lib)
    return any(os.path.exists(s) and os.path.getmtime(s) > t for s in sources)


def ensure_workload_gen() -> str:
    if _stale(GEN_LIB, [os.path.join(CSRC, "workload_gen.c")]):
        build_workload_gen()
    return GEN_LIB


def hip_sources():
    """Every file the HIP library is compiled from: the kernels, the host code and the public header."""
    import glob
    return sorted(glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(CSRC, "*.hip")) +
                  glob.glob(os.path.join(INCLUDE, "*.h")))


def ensure_hip() -> str:
    """Return the built HIP library; compile it when it is absent or older than one of its sources (where no
    compiler is at hand, as on a box that only runs what was built elsewhere, a stale library is an error)."""
    if _stale(HIP_LIB, hip_sources()):
        build_hip()
    return HIP_LIB
