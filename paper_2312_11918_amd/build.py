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


def resource_usage():
    """Compile the attention kernels for the device only and return what the compiler reports per kernel: a list
    of dicts with the (demangled) kernel name, VGPRs, AGPRs, SGPRs, scratch bytes per lane, LDS bytes per workgroup
    and wavefronts per SIMD.  Nothing is written; used by the test that keeps every kernel free of scratch."""
    import re

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc, *flags, "-I", INCLUDE, "--cuda-device-only", "-c", "-o", os.devnull,
           "-Rpass-analysis=kernel-resource-usage", *SOURCES]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    keys = {"TotalSGPRs": "sgprs", "VGPRs": "vgprs", "AGPRs": "agprs", "ScratchSize [bytes/lane]": "scratch_bytes_per_lane",
            "Occupancy [waves/SIMD]": "waves_per_simd", "LDS Size [bytes/block]": "lds_bytes_per_workgroup"}
    kernels, cur = [], None
    for line in res.stdout.splitlines():
        m = re.search(r"remark:\s+(.*?)\s+\[-Rpass-analysis", line)
        if not m:
            continue
        text = m.group(1).strip()
        if text.startswith("Function Name:"):
            cur = {"mangled": text.split(":", 1)[1].strip()}
            kernels.append(cur)
        elif cur is not None and ":" in text:
            k, v = text.rsplit(":", 1)
            if k.strip() in keys:
                cur[keys[k.strip()]] = int(v)
    for k in kernels:
        m = re.search(r"fa2_fwd_kernelILi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELb(\d)ELb(\d)E", k["mangled"])
        if m:
            dt, d, wv, nbuf, causal, ragged = (int(x) for x in m.groups())
            k["name"] = (f"fa2_fwd_kernel<{'fp16' if dt == 0 else 'bf16'}, d={d}, {wv} wavefronts, {nbuf} LDS buffers"
                         f"{', causal' if causal else ''}{', partial tiles' if ragged else ''}>")
        else:
            k["name"] = k["mangled"]
    return kernels


if __name__ == "__main__":
    import sys

    if "--resource-usage" in sys.argv:
        rows = resource_usage()
        print("| kernel | VGPRs | AGPRs | SGPRs | scratch B/lane | LDS B/workgroup | wavefronts/SIMD |")
        print("|---|---|---|---|---|---|---|")
        for k in sorted(rows, key=lambda r: r["name"]):
            print(f"| {k['name']} | {k['vgprs']} | {k['agprs']} | {k['sgprs']} | {k['scratch_bytes_per_lane']} | "
                  f"{k['lds_bytes_per_workgroup']} | {k['waves_per_simd']} |")
    else:
        print(build_library(verbose=True))
