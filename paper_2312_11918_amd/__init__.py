"""FlashAttention-2 forward pass for MI355X (gfx950): a hand-written HIP kernel behind a C ABI.

``fa2_fwd`` and friends are thin ctypes marshalling over ``libfa2.so``; every step of the
attention path runs in the HIP kernel.  The shared library is loaded on first use and a
missing library is an error (there is no CPU fallback).
"""
from .binding import (FA2_BF16, FA2_ERR_INVALID_ARG, FA2_ERR_LAUNCH, FA2_ERR_UNSUPPORTED, FA2_FP16, FA2_MASK_CAUSAL,
                      FA2_MASK_NONE, FA2_OK, FA2_PROBE_MFMA_PER_ITER, FA2_PROBE_OPERAND_BYTES, FA2_PROBE_WORKGROUPS,
                      FA2_VARIANT_AUTO, FA2_VARIANT_NARROW, FA2_VARIANT_NARROW8,
                      Fa2Error, fa2_fwd, fa2_fwd_masked_raw, fa2_fwd_qk_raw, fa2_fwd_raw, fa2_fwd_variant_raw,
                      fa2_probe_mfma_raw, fa2_strerror, fa2_tile_shape, fa2_version, library_path, load_library, load_probe_library,
                      probe_library_path)

__all__ = ["FA2_BF16", "FA2_ERR_INVALID_ARG", "FA2_ERR_LAUNCH", "FA2_ERR_UNSUPPORTED", "FA2_FP16", "FA2_MASK_CAUSAL",
           "FA2_MASK_NONE", "FA2_OK", "FA2_PROBE_MFMA_PER_ITER", "FA2_PROBE_OPERAND_BYTES", "FA2_PROBE_WORKGROUPS",
           "FA2_VARIANT_AUTO", "FA2_VARIANT_NARROW", "FA2_VARIANT_NARROW8",
           "Fa2Error", "fa2_fwd", "fa2_fwd_masked_raw", "fa2_fwd_qk_raw", "fa2_fwd_raw", "fa2_fwd_variant_raw",
           "fa2_probe_mfma_raw", "fa2_strerror", "fa2_tile_shape", "fa2_version", "library_path", "load_library", "load_probe_library",
           "probe_library_path"]
