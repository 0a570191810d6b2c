"""fp64 CPU oracle for scaled dot-product attention -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``attention_oracle.c`` (the paper's Algorithm 1 "Standard Attention"
and the formula of Section 2, with S and P materialised, in fp64).  Only the tests, the smoke
check and the benchmark's ``cpu_baseline`` leg may import this package; it shares nothing with
the GPU library and the product path never routes through it.

Tensor layout is the paper's (batch, seqlen, heads, headdim) (Section 2): arrays are
``[B, N, H, d]``; LSE is ``[B, H, N]``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attention_oracle.c")
_LIB = os.path.join(_HERE, "libattention_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP).  Returns the path of the shared library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        ci, cd = ctypes.c_int, ctypes.c_double
        lib.fa_oracle_forward.argtypes = [dp, dp, dp, dp, dp, ci, ci, ci, ci, ci, cd, ci]
        lib.fa_oracle_forward.restype = ci
        lib.fa_oracle_rows.argtypes = [dp, dp, dp, ip, ci, dp, dp, ci, ci, ci, ci, ci, cd]
        lib.fa_oracle_rows.restype = ci
        lib.fa_oracle_forward_masked.argtypes = [dp, dp, dp, dp, dp, ci, ci, ci, ci, ci, cd, ci, ci]
        lib.fa_oracle_forward_masked.restype = ci
        lib.fa_oracle_rows_masked.argtypes = [dp, dp, dp, ip, ci, dp, dp, ci, ci, ci, ci, ci, cd, ci]
        lib.fa_oracle_rows_masked.restype = ci
        lib.fa_oracle_head_probs.argtypes = [dp, dp, dp, dp, dp, ci, ci, ci, ci, ci, cd, ci, ci]
        lib.fa_oracle_head_probs.restype = ci
        lib.fa_oracle_num_threads.argtypes = []
        lib.fa_oracle_num_threads.restype = ci
        _lib = lib
    return _lib


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact fp64 values of an array of 16-bit floating-point bit patterns (uint16).

    ``dtype`` is "fp16" (IEEE binary16) or "bf16" (the upper half of an IEEE binary32).
    """
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == "fp16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def _check_qkv(q, k, v):
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    if q.ndim != 4 or k.ndim != 4 or v.ndim != 4:
        raise ValueError("q, k, v must be [B, N, H, d]")
    B, Nq, H, d = q.shape
    if k.shape[0] != B or k.shape[2] != H or k.shape[3] != d or v.shape != k.shape:
        raise ValueError(f"shape mismatch: q {q.shape} k {k.shape} v {v.shape}")
    return q, k, v, B, H, Nq, k.shape[1], d


def attention(q, k, v, scale: float, row_block: int = 32, causal: bool = False):
    """Standard attention for every head and row.  Returns ``(O [B,Nq,H,d] fp64, LSE [B,H,Nq] fp64)``.

    ``causal`` applies the optional mask of S (Section 2, footnote): row i sees keys j <= i only.
    """
    q, k, v, B, H, Nq, Nk, d = _check_qkv(q, k, v)
    o = np.empty((B, Nq, H, d), dtype=np.float64)
    lse = np.empty((B, H, Nq), dtype=np.float64)
    rc = _load().fa_oracle_forward_masked(_dptr(q), _dptr(k), _dptr(v), _dptr(o), _dptr(lse), B, H, Nq, Nk, d,
                                          float(scale), int(bool(causal)), int(row_block))
    if rc != 0:
        raise RuntimeError(f"fa_oracle_forward_masked failed with code {rc}")
    return o, lse


def attention_rows(q, k, v, scale: float, rows_bhi, causal: bool = False):
    """Standard attention for sampled query rows.

    ``rows_bhi`` is an ``[n, 3]`` integer array of (batch, head, row).  Returns
    ``(O_rows [n, d] fp64, LSE_rows [n] fp64)``; each row is a complete softmax over all keys.
    """
    q, k, v, B, H, Nq, Nk, d = _check_qkv(q, k, v)
    rows = np.ascontiguousarray(rows_bhi, dtype=np.int32).reshape(-1, 3)
    n = rows.shape[0]
    o = np.empty((n, d), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    rc = _load().fa_oracle_rows_masked(_dptr(q), _dptr(k), _dptr(v),
                                       rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), n, _dptr(o), _dptr(lse),
                                       B, H, Nq, Nk, d, float(scale), int(bool(causal)))
    if rc != 0:
        raise RuntimeError(f"fa_oracle_rows_masked failed with code {rc}")
    return o, lse


def head_probs(q, k, v, scale: float, b: int, h: int):
    """The materialised intermediates of head (b, h): ``(S [Nq,Nk], P [Nq,Nk])`` in fp64."""
    q, k, v, B, H, Nq, Nk, d = _check_qkv(q, k, v)
    s = np.empty((Nq, Nk), dtype=np.float64)
    p = np.empty((Nq, Nk), dtype=np.float64)
    rc = _load().fa_oracle_head_probs(_dptr(q), _dptr(k), _dptr(v), _dptr(s), _dptr(p), B, H, Nq, Nk, d,
                                      float(scale), int(b), int(h))
    if rc != 0:
        raise RuntimeError(f"fa_oracle_head_probs failed with code {rc}")
    return s, p


def num_threads() -> int:
    """Threads a call of :func:`attention` uses (OpenMP's maximum)."""
    return int(_load().fa_oracle_num_threads())
