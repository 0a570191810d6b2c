"""Host-side behaviour of the C ABI that needs no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_2312_11918_amd as fa2

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "fa2.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fa2_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    assert {"fa2_fwd", "fa2_fwd_variant", "fa2_fwd_masked", "fa2_fwd_qk", "fa2_strerror", "fa2_version"} <= set(_declared_functions())


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(fa2.library_path())
    for name in _declared_functions():
        assert hasattr(lib, name), f"{name} is declared in include/fa2.h but not exported"


def test_probe_library_exports_what_its_header_declares():
    text = open(os.path.join(ROOT, "include", "fa2_probe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(fa2_[a-z0-9_]+)\s*\(", text)))
    assert names == ["fa2_probe_mfma"]
    lib = ctypes.CDLL(fa2.probe_library_path())
    for name in names:
        assert hasattr(lib, name)
    # bad arguments are refused before any HIP call
    assert fa2.fa2_probe_mfma_raw(None, 0x1000, 0x1000, 0, 10) == -1
    assert fa2.fa2_probe_mfma_raw(0x1000, 0x1000, 0x1000, 0, 0) == -1
    assert fa2.fa2_probe_mfma_raw(0x1008, 0x1000, 0x1000, 0, 10) == -1
    assert fa2.fa2_probe_mfma_raw(0x1000, 0x1000, 0x1000, 5, 10) == -1


def test_version_and_strerror():
    assert fa2.fa2_version() >= 100
    for code in (fa2.FA2_OK, fa2.FA2_ERR_INVALID_ARG, fa2.FA2_ERR_UNSUPPORTED, fa2.FA2_ERR_LAUNCH, 12345):
        assert isinstance(fa2.fa2_strerror(code), str) and fa2.fa2_strerror(code)


P = 0x1000  # a 16-byte aligned, never dereferenced "device address": validation must reject first


@pytest.mark.parametrize("args,code", [
    (dict(q=None), fa2.FA2_ERR_INVALID_ARG),
    (dict(k=None), fa2.FA2_ERR_INVALID_ARG),
    (dict(v=None), fa2.FA2_ERR_INVALID_ARG),
    (dict(o=None), fa2.FA2_ERR_INVALID_ARG),
    (dict(B=0), fa2.FA2_ERR_INVALID_ARG),
    (dict(H=-1), fa2.FA2_ERR_INVALID_ARG),
    (dict(N=0), fa2.FA2_ERR_INVALID_ARG),
    (dict(d=0), fa2.FA2_ERR_INVALID_ARG),
    (dict(scale=0.0), fa2.FA2_ERR_INVALID_ARG),
    (dict(scale=-0.125), fa2.FA2_ERR_INVALID_ARG),
    (dict(scale=float("nan")), fa2.FA2_ERR_INVALID_ARG),
    (dict(scale=float("inf")), fa2.FA2_ERR_INVALID_ARG),
    (dict(q=P + 8), fa2.FA2_ERR_INVALID_ARG),
    (dict(o=P + 2), fa2.FA2_ERR_INVALID_ARG),
    (dict(lse=P + 2), fa2.FA2_ERR_INVALID_ARG),
    (dict(d=96), fa2.FA2_ERR_UNSUPPORTED),
    (dict(d=512), fa2.FA2_ERR_UNSUPPORTED),
    (dict(N=-128), fa2.FA2_ERR_INVALID_ARG),
    (dict(H=1 << 15, N=1 << 16, d=128), fa2.FA2_ERR_UNSUPPORTED),      # a head's rows span >= 4 GiB: 32-bit offsets
    (dict(dtype=7), fa2.FA2_ERR_UNSUPPORTED),
    (dict(B=1 << 20, N=1 << 20), fa2.FA2_ERR_UNSUPPORTED),
])
def test_bad_arguments_are_rejected_without_a_launch(args, code):
    a = dict(q=P, k=P, v=P, o=P, lse=P, B=1, H=2, N=256, d=64, scale=0.125, dtype=fa2.FA2_FP16)
    a.update(args)
    rc = fa2.fa2_fwd_raw(a["q"], a["k"], a["v"], a["o"], a["lse"], a["B"], a["H"], a["N"], a["d"], a["scale"], a["dtype"])
    assert rc == code


_OKARGS = dict(q=P, k=P, v=P, o=P, lse=P, B=1, H=2, N=256, d=64, scale=0.125, dtype=fa2.FA2_FP16)


@pytest.mark.parametrize("variant,args,code", [
    (99, {}, fa2.FA2_ERR_INVALID_ARG),                                 # unknown tile shape
    (-1, {}, fa2.FA2_ERR_INVALID_ARG),
    (fa2.FA2_VARIANT_NARROW8, dict(N=384), fa2.FA2_ERR_UNSUPPORTED),   # the 256-row shape needs N % 256 == 0
    (2, {}, fa2.FA2_ERR_INVALID_ARG),                                  # values 2 and 4 are not tile shapes
    (4, {}, fa2.FA2_ERR_INVALID_ARG),
    (fa2.FA2_VARIANT_NARROW8, dict(N=128), fa2.FA2_ERR_UNSUPPORTED),
    (fa2.FA2_VARIANT_NARROW, dict(d=32), fa2.FA2_ERR_UNSUPPORTED),
    (fa2.FA2_VARIANT_NARROW8, dict(d=256), fa2.FA2_ERR_UNSUPPORTED),   # d=256 runs on the 128-row shape only
    (fa2.FA2_VARIANT_NARROW, dict(q=None), fa2.FA2_ERR_INVALID_ARG),
])
def test_variant_entry_rejects_bad_arguments_without_a_launch(variant, args, code):
    a = dict(_OKARGS)
    a.update(args)
    rc = fa2.fa2_fwd_variant_raw(a["q"], a["k"], a["v"], a["o"], a["lse"], a["B"], a["H"], a["N"], a["d"], a["scale"],
                                 a["dtype"], variant)
    assert rc == code


@pytest.mark.parametrize("mask,args,code", [
    (2, {}, fa2.FA2_ERR_INVALID_ARG),                                  # unknown mask
    (-1, {}, fa2.FA2_ERR_INVALID_ARG),
    (fa2.FA2_MASK_CAUSAL, dict(k=None), fa2.FA2_ERR_INVALID_ARG),
    (fa2.FA2_MASK_CAUSAL, dict(d=96), fa2.FA2_ERR_UNSUPPORTED),
    (fa2.FA2_MASK_CAUSAL, dict(scale=-1.0), fa2.FA2_ERR_INVALID_ARG),
    (fa2.FA2_MASK_NONE, dict(dtype=3), fa2.FA2_ERR_UNSUPPORTED),
])
def test_masked_entry_rejects_bad_arguments_without_a_launch(mask, args, code):
    a = dict(_OKARGS)
    a.update(args)
    rc = fa2.fa2_fwd_masked_raw(a["q"], a["k"], a["v"], a["o"], a["lse"], a["B"], a["H"], a["N"], a["d"], a["scale"],
                                a["dtype"], mask)
    assert rc == code


@pytest.mark.parametrize("Nq,Nk,mask,args,code", [
    (0, 128, fa2.FA2_MASK_NONE, {}, fa2.FA2_ERR_INVALID_ARG),
    (128, 0, fa2.FA2_MASK_NONE, {}, fa2.FA2_ERR_INVALID_ARG),
    (128, -5, fa2.FA2_MASK_NONE, {}, fa2.FA2_ERR_INVALID_ARG),
    (100, 100, 7, {}, fa2.FA2_ERR_INVALID_ARG),
    (100, 101, fa2.FA2_MASK_CAUSAL, {}, fa2.FA2_ERR_UNSUPPORTED),      # the causal diagonal needs a square S
    (100, 300, fa2.FA2_MASK_NONE, dict(d=80), fa2.FA2_ERR_UNSUPPORTED),
    (100, 300, fa2.FA2_MASK_NONE, dict(v=None), fa2.FA2_ERR_INVALID_ARG),
    (100, 300, fa2.FA2_MASK_NONE, dict(lse=P + 1), fa2.FA2_ERR_INVALID_ARG),
    (1 << 20, 16, fa2.FA2_MASK_NONE, dict(B=1 << 12), fa2.FA2_ERR_UNSUPPORTED),
])
def test_qk_entry_rejects_bad_arguments_without_a_launch(Nq, Nk, mask, args, code):
    a = dict(_OKARGS)
    a.update(args)
    rc = fa2.fa2_fwd_qk_raw(a["q"], a["k"], a["v"], a["o"], a["lse"], a["B"], a["H"], Nq, Nk, a["d"], a["scale"],
                            a["dtype"], mask)
    assert rc == code


def test_torch_wrapper_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 128, 1, 64, dtype=torch.float16)
    with pytest.raises(ValueError):
        fa2.fa2_fwd(x, x, x, 0.125)
