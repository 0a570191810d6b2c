"""Builds libfa2.so (the HIP kernels and their C ABI) and libfa2_probe.so (the MFMA roof probe) in-tree with hipcc
for gfx950."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
SOURCES = [os.path.join(_PKG, "csrc", "fa2_fwd.hip")]
INCLUDE = os.path.join(_ROOT, "include")
LIBRARY = os.path.join(_PKG, "libfa2.so")
PROBE_SOURCES = [os.path.join(_PKG, "csrc", "mfma_probe.hip")]
PROBE_LIBRARY = os.path.join(_PKG, "libfa2_probe.so")

# Packed-fp32 VALU instructions are switched off for the device pass on purpose (the host pass
# prints a harmless "unknown feature" warning).
HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc(sources, library, verbose):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", INCLUDE, *sources, "-o", library]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose and res.stdout.strip():
        print(res.stdout)
    return library


def build_library(verbose: bool = False) -> str:
    """Compile the HIP sources into ``libfa2.so`` and ``libfa2_probe.so`` next to this file; returns the former's path."""
    _hipcc(PROBE_SOURCES, PROBE_LIBRARY, verbose)
    return _hipcc(SOURCES, LIBRARY, verbose)


if __name__ == "__main__":
    print(build_library(verbose=True))
