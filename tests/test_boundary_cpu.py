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
    assert {"fa2_fwd", "fa2_fwd_variant", "fa2_fwd_masked", "fa2_fwd_qk", "fa2_tile_shape", "fa2_strerror",
            "fa2_version"} <= set(_declared_functions())


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


def test_tile_shape_choice_follows_the_documented_rule():
    # host logic only: which tile shape the entry points without a `variant` argument take (no launch, no GPU)
    from paper_2312_11918_amd import workloads
    N8, N4 = fa2.FA2_VARIANT_NARROW8, fa2.FA2_VARIANT_NARROW
    expect = {1: N4, 2: N4, 3: N8, 4: N8, 5: N8}   # the five workloads: tiny and N = 512 at d = 64 stay in 128 rows
    for i, w in workloads.CONFIGS.items():
        assert fa2.fa2_tile_shape(w.B, w.H, w.N, w.N, w.d) == expect[i], w.name
    # the paper's shapes
    assert fa2.fa2_tile_shape(4, 32, 4096, 4096, 64) == N8
    assert fa2.fa2_tile_shape(4, 16, 4096, 4096, 128) == N8
    assert fa2.fa2_tile_shape(4, 8, 4096, 4096, 256) == N4          # d = 256 exists in the 128-row shape only
    # whole rounds of the 256 CUs decide: 3 x 16 heads x 8 tiles = 384 tiles is one and a half rounds
    assert fa2.fa2_tile_shape(3, 16, 2048, 2048, 128) == N4
    assert fa2.fa2_tile_shape(4, 16, 2048, 2048, 128) == N8
    # ... unless the tiles are very many (d = 128, N >= 2048)
    assert fa2.fa2_tile_shape(33, 16, 4096, 4096, 128) == N8         # 8448 tiles, 33 rounds
    assert fa2.fa2_tile_shape(33, 16, 1024, 1024, 128) == N4
    # partial tiles, Nq != Nk
    assert fa2.fa2_tile_shape(8, 16, 2047, 2047, 128) == N4
    assert fa2.fa2_tile_shape(8, 16, 2048, 4096, 128) == N4
    # d = 64: only from N = 2048 on
    assert fa2.fa2_tile_shape(16, 32, 1024, 1024, 64) == N4
    assert fa2.fa2_tile_shape(8, 32, 2048, 2048, 64) == N8
    # causal: d = 128 from N = 2048 on (pairs of Q tiles fill the rounds), never at d = 64
    C = fa2.FA2_MASK_CAUSAL
    assert fa2.fa2_tile_shape(8, 16, 2048, 2048, 128, C) == N8
    assert fa2.fa2_tile_shape(16, 16, 1024, 1024, 128, C) == N4
    assert fa2.fa2_tile_shape(1, 32, 16384, 16384, 64, C) == N4
    # refused like the launching entry points refuse
    assert fa2.fa2_tile_shape(1, 1, 128, 128, 96) == fa2.FA2_ERR_UNSUPPORTED
    assert fa2.fa2_tile_shape(1, 1, 128, 256, 64, C) == fa2.FA2_ERR_UNSUPPORTED
    assert fa2.fa2_tile_shape(0, 1, 128, 128, 64) == fa2.FA2_ERR_INVALID_ARG
    assert fa2.fa2_tile_shape(1, 1, 128, 128, 64, 7) == fa2.FA2_ERR_INVALID_ARG
