"""ctypes binding of libfa2's C ABI (see include/fa2.h).  Argument marshalling only.

``fa2_fwd_raw`` takes raw device addresses; ``fa2_fwd`` takes torch CUDA tensors, which are used
purely as owners of device memory (``data_ptr()``) and of the current HIP stream.
"""
from __future__ import annotations

import ctypes
import os

FA2_FP16 = 0
FA2_BF16 = 1
FA2_OK = 0
FA2_ERR_INVALID_ARG = -1
FA2_ERR_UNSUPPORTED = -2
FA2_ERR_LAUNCH = -3
FA2_VARIANT_AUTO = 0
FA2_VARIANT_NARROW = 1
FA2_VARIANT_NARROW8 = 3
FA2_MASK_NONE = 0
FA2_MASK_CAUSAL = 1

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libfa2.so")
_PROBE_PATH = os.path.join(_PKG, "libfa2_probe.so")
_lib = None
_probe = None


class Fa2Error(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"fa2 error {code}: {message}")
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libfa2.so (built in-tree by ``build.build_library``).  A missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is not built; run `python -m paper_2312_11918_amd.build` "
                "(there is no fallback path)")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        lib.fa2_fwd.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ctypes.c_float, ci, vp]
        lib.fa2_fwd.restype = ci
        lib.fa2_fwd_variant.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ctypes.c_float, ci, ci, vp]
        lib.fa2_fwd_variant.restype = ci
        lib.fa2_fwd_masked.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ctypes.c_float, ci, ci, vp]
        lib.fa2_fwd_masked.restype = ci
        lib.fa2_fwd_qk.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ctypes.c_float, ci, ci, vp]
        lib.fa2_fwd_qk.restype = ci
        lib.fa2_strerror.argtypes = [ci]
        lib.fa2_strerror.restype = ctypes.c_char_p
        lib.fa2_tile_shape.argtypes = [ci, ci, ci, ci, ci, ci]
        lib.fa2_tile_shape.restype = ci
        lib.fa2_version.argtypes = []
        lib.fa2_version.restype = ci
        _lib = lib
    return _lib


def probe_library_path() -> str:
    return _PROBE_PATH


def load_probe_library():
    """Load libfa2_probe.so (the MFMA roof probe, see include/fa2_probe.h).  A missing library is an error."""
    global _probe
    if _probe is None:
        if not os.path.exists(_PROBE_PATH):
            raise FileNotFoundError(f"{_PROBE_PATH} is not built; run `python -m paper_2312_11918_amd.build`")
        lib = ctypes.CDLL(_PROBE_PATH)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        lib.fa2_probe_mfma.argtypes = [vp, vp, vp, ci, ci, vp]
        lib.fa2_probe_mfma.restype = ci
        _probe = lib
    return _probe


FA2_PROBE_WORKGROUPS = 512
FA2_PROBE_MFMA_PER_ITER = 16
FA2_PROBE_OPERAND_BYTES = 256 * 4 * 2 * 16


def fa2_probe_mfma_raw(operands_ptr, ticks_ptr, sink_ptr, dtype, iters, stream=None) -> int:
    """Call ``fa2_probe_mfma`` with raw device addresses; returns the C return code."""
    return int(load_probe_library().fa2_probe_mfma(operands_ptr, ticks_ptr, sink_ptr, int(dtype), int(iters), stream))


def fa2_strerror(code: int) -> str:
    return load_library().fa2_strerror(int(code)).decode()


def fa2_tile_shape(B: int, H: int, Nq: int, Nk: int, d: int, mask: int = FA2_MASK_NONE) -> int:
    """The tile shape (``FA2_VARIANT_*``) the library picks for a problem, or a negative error code.  No launch."""
    return int(load_library().fa2_tile_shape(int(B), int(H), int(Nq), int(Nk), int(d), int(mask)))


def fa2_version() -> int:
    return int(load_library().fa2_version())


def fa2_fwd_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, N, d, scale, dtype, stream=None) -> int:
    """Call ``fa2_fwd`` with raw device addresses (ints or None); returns the C return code."""
    return int(load_library().fa2_fwd(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, int(B), int(H), int(N), int(d),
                                      float(scale), int(dtype), stream))


def fa2_fwd_variant_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, N, d, scale, dtype, variant, stream=None) -> int:
    """Call ``fa2_fwd_variant`` (explicit tile shape) with raw device addresses; returns the C return code."""
    return int(load_library().fa2_fwd_variant(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, int(B), int(H), int(N), int(d),
                                              float(scale), int(dtype), int(variant), stream))


def fa2_fwd_masked_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, N, d, scale, dtype, mask, stream=None) -> int:
    """Call ``fa2_fwd_masked`` (optional causal mask of S) with raw device addresses; returns the C return code."""
    return int(load_library().fa2_fwd_masked(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, int(B), int(H), int(N), int(d),
                                             float(scale), int(dtype), int(mask), stream))


def fa2_fwd_qk_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, Nq, Nk, d, scale, dtype, mask, stream=None) -> int:
    """Call ``fa2_fwd_qk`` (Nq queries, Nk keys, optional causal mask) with raw device addresses; returns the C code."""
    return int(load_library().fa2_fwd_qk(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, int(B), int(H), int(Nq), int(Nk), int(d),
                                         float(scale), int(dtype), int(mask), stream))


def fa2_fwd(q, k, v, scale: float, out=None, lse=None, return_lse: bool = True, stream=None,
            variant: int = FA2_VARIANT_AUTO, causal: bool = False):
    """Attention forward on torch CUDA tensors: ``q`` ``[B, Nq, H, d]``, ``k`` and ``v`` ``[B, Nk, H, d]`` (fp16 or
    bf16, contiguous).

    Returns ``(O, LSE)`` with O like ``q`` and LSE ``[B, H, Nq]`` fp32 (``None`` if ``return_lse`` is
    false).  The kernel is enqueued on ``stream`` (a ``torch.cuda.Stream``) or on torch's current stream.
    ``variant`` selects the tile shape (``FA2_VARIANT_*``); the default lets the library choose.
    ``causal`` masks S so that query i sees keys j <= i only (``fa2_fwd_masked``; default tile shape only).
    """
    import torch

    if not (q.is_cuda and k.is_cuda and v.is_cuda):
        raise ValueError("q, k, v must be CUDA tensors (there is no CPU path)")
    if q.dtype == torch.float16:
        dtype = FA2_FP16
    elif q.dtype == torch.bfloat16:
        dtype = FA2_BF16
    else:
        raise ValueError(f"unsupported element type {q.dtype}")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share one element type")
    if (q.dim() != 4 or k.dim() != 4 or v.shape != k.shape or k.shape[0] != q.shape[0] or k.shape[2:] != q.shape[2:]):
        raise ValueError(f"q must be [B, Nq, H, d], k and v [B, Nk, H, d]; got {tuple(q.shape)}, {tuple(k.shape)}, "
                         f"{tuple(v.shape)}")
    if not (q.is_contiguous() and k.is_contiguous() and v.is_contiguous()):
        raise ValueError("q, k, v must be contiguous")
    B, N, H, d = q.shape
    Nk = k.shape[1]
    if out is None:
        out = torch.empty_like(q)
    elif out.shape != q.shape or out.dtype != q.dtype or not out.is_contiguous() or out.device != q.device:
        raise ValueError("out must match q in shape, dtype, device and be contiguous")
    if return_lse:
        if lse is None:
            lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
        elif tuple(lse.shape) != (B, H, N) or lse.dtype != torch.float32 or not lse.is_contiguous():
            raise ValueError("lse must be a contiguous fp32 [B, H, N] tensor")
    else:
        lse = None
    with torch.cuda.device(q.device):
        s = stream if stream is not None else torch.cuda.current_stream()
        ptrs = (q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), None if lse is None else lse.data_ptr())
        if variant != FA2_VARIANT_AUTO:
            if causal or Nk != N:
                raise ValueError("an explicit tile shape runs square, unmasked problems only")
            rc = fa2_fwd_variant_raw(*ptrs, B, H, N, d, scale, dtype, variant, s.cuda_stream)
        elif Nk != N:
            rc = fa2_fwd_qk_raw(*ptrs, B, H, N, Nk, d, scale, dtype, FA2_MASK_CAUSAL if causal else FA2_MASK_NONE,
                                s.cuda_stream)
        elif causal:
            rc = fa2_fwd_masked_raw(*ptrs, B, H, N, d, scale, dtype, FA2_MASK_CAUSAL, s.cuda_stream)
        else:
            rc = fa2_fwd_raw(*ptrs, B, H, N, d, scale, dtype, s.cuda_stream)
    if rc != FA2_OK:
        raise Fa2Error(rc, fa2_strerror(rc))
    return out, lse
