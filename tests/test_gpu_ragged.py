"""GPU parity for sizes that are not whole tiles and for Nq != Nk (fa2_fwd_qk, and fa2_fwd / fa2_fwd_masked with
a ragged N), against the fp64 CPU oracle on the same seeded bits.  Tolerances are those of the whole-tile path."""
import numpy as np
import pytest

import oracle
import paper_2312_11918_amd as fa2
from paper_2312_11918_amd import workloads
from _gpu_common import TOL_LSE_MAX, TOL_O_MAX, check, torch_gpu

pytestmark = pytest.mark.gpu

SENT16, SENT32 = 0x7E00, np.float32(-12345.0)  # fp16/bf16 NaN pattern as a sentinel; LSE sentinel
PAD = 4096  # sentinel elements on each side of every device tensor


def _guarded(bits, dtype):
    """Device tensor holding `bits` with PAD NaN-pattern elements before and after it; returns (view, whole)."""
    torch = torch_gpu()
    flat = np.full(bits.size + 2 * PAD, SENT16, dtype=np.uint16)
    flat[PAD:PAD + bits.size] = bits.reshape(-1)
    whole = torch.from_numpy(flat.view(np.int16)).cuda()
    tdt = torch.float16 if dtype == "fp16" else torch.bfloat16
    return whole[PAD:PAD + bits.size].view(tdt).view(*bits.shape), whole


def _make(B, H, Nq, Nk, d, dtype, seed, outliers=0.0):
    qb, _, _ = workloads.make_qkv(B, Nq, H, d, dtype, seed)
    _, kb, vb = workloads.make_qkv(B, Nk, H, d, dtype, seed + 1, k_outlier_frac=outliers, k_outlier_gain=6.0)
    return qb, kb, vb


def _run(qb, kb, vb, dtype, scale, causal=False):
    """Runs the library on guarded buffers; checks that no sentinel moved and nothing outside Q, K, V leaked in."""
    torch = torch_gpu()
    B, Nq, H, d = qb.shape
    q, _ = _guarded(qb, dtype)
    k, _ = _guarded(kb, dtype)
    v, _ = _guarded(vb, dtype)
    o, o_whole = _guarded(np.full(qb.shape, SENT16, dtype=np.uint16), dtype)
    lse_whole = torch.full((B * H * Nq + 2 * PAD,), float(SENT32), dtype=torch.float32, device="cuda")
    lse = lse_whole[PAD:PAD + B * H * Nq].view(B, H, Nq)
    fa2.fa2_fwd(q, k, v, scale, out=o, lse=lse, causal=causal)
    torch.cuda.synchronize()
    ow = o_whole.cpu().numpy().view(np.uint16)
    assert np.all(ow[:PAD] == SENT16) and np.all(ow[PAD + qb.size:] == SENT16), "O was written outside its bounds"
    lw = lse_whole.cpu().numpy()
    assert np.all(lw[:PAD] == SENT32) and np.all(lw[PAD + B * H * Nq:] == SENT32), "LSE was written outside its bounds"
    return o.double().cpu().numpy(), lse.double().cpu().numpy()


def _check(o_gpu, lse_gpu, o_ref, lse_ref, what):
    assert not np.any(lse_gpu == SENT32), f"{what}: LSE has unwritten entries"
    check(o_gpu, lse_gpu, o_ref, lse_ref, what)   # non-finite values: unwritten rows or leaked padding


@pytest.mark.parametrize("B,H,Nq,Nk,d,dtype,causal,outliers", [
    (1, 2, 1, 1, 64, "fp16", False, 0.0),        # one query, one key: O = V_0, LSE = scale * q.k
    (1, 1, 1, 1, 128, "bf16", True, 0.0),
    (1, 2, 100, 100, 64, "fp16", False, 0.0),    # less than one Q tile, 2 K/V tiles with a partial one
    (2, 3, 129, 129, 128, "fp16", False, 0.0),   # one row and one key past a tile
    (1, 1, 127, 127, 128, "bf16", False, 0.0),   # one short of a tile
    (1, 2, 63, 65, 64, "fp16", False, 0.0),      # around one K/V tile
    (1, 2, 200, 77, 64, "fp16", False, 0.0),     # Nq > Nk; an odd tile count, so a padding tile is fully masked
    (2, 2, 64, 300, 128, "fp16", False, 0.02),   # Nq < Nk; 5 K/V tiles (odd), large-logit keys
    (1, 3, 333, 1000, 64, "bf16", False, 0.0),
    (1, 2, 1000, 333, 128, "fp16", False, 0.0),
    (1, 2, 256, 192, 64, "fp16", False, 0.0),    # whole Q tiles, Nk a multiple of 64 but not of 128
    (1, 2, 257, 257, 256, "fp16", False, 0.0),   # d = 256
    (1, 1, 130, 70, 256, "bf16", False, 0.0),
    (1, 2, 100, 100, 64, "fp16", True, 0.0),     # causal, one partial Q tile
    (2, 2, 129, 129, 128, "fp16", True, 0.0),    # causal, 2 Q tiles, the second with one row
    (1, 3, 500, 500, 64, "bf16", True, 0.0),     # causal, 4 Q tiles (2 pairs), last partial
    (1, 2, 700, 700, 128, "fp16", True, 0.02),   # causal, 6 Q tiles (3 pairs), large-logit keys
    (1, 2, 321, 321, 256, "fp16", True, 0.0),    # causal, d = 256, 3 Q tiles (one unpaired)
])
def test_ragged_parity_elementwise(B, H, Nq, Nk, d, dtype, causal, outliers):
    seed = 8000 + 3 * Nq + 5 * Nk + d + B
    print(f"ragged case B={B} H={H} Nq={Nq} Nk={Nk} d={d} {dtype} causal={causal} seed={seed}", flush=True)
    qb, kb, vb = _make(B, H, Nq, Nk, d, dtype, seed, outliers)
    scale = float(np.float32(d) ** np.float32(-0.5))
    o_ref, lse_ref = oracle.attention(*(oracle.widen(x, dtype) for x in (qb, kb, vb)), scale, causal=causal)
    o, lse = _run(qb, kb, vb, dtype, scale, causal)
    _check(o, lse, o_ref, lse_ref, f"ragged B{B} H{H} Nq{Nq} Nk{Nk} d{d} {dtype} causal={causal}")


def _random_shapes(count, seed):
    """Seeded draw of problem shapes: sizes spread over 1 .. 900 on a log scale, every head dimension, both types,
    the causal mask on a third of the square ones."""
    r = np.random.Generator(np.random.PCG64(seed))
    shapes = []
    for _ in range(count):
        nq, nk = (int(round(float(np.exp(r.uniform(0.0, np.log(900.0)))))) for _ in range(2))
        causal = bool(r.integers(0, 3) == 0)
        if causal or r.integers(0, 4) == 0:
            nk = nq
        shapes.append((int(r.integers(1, 3)), int(r.integers(1, 4)), nq, nk, int(r.choice([64, 128, 256])),
                       str(r.choice(["fp16", "bf16"])), causal))
    return shapes


def test_seeded_random_shapes_elementwise():
    # forty shapes nobody picked by hand; each on guarded buffers, every element against the oracle
    for n, (B, H, Nq, Nk, d, dtype, causal) in enumerate(_random_shapes(40, 20260417)):
        print(f"random shape {n}: B={B} H={H} Nq={Nq} Nk={Nk} d={d} {dtype} causal={causal}", flush=True)
        qb, kb, vb = _make(B, H, Nq, Nk, d, dtype, 12000 + n)
        scale = float(np.float32(d) ** np.float32(-0.5))
        o_ref, lse_ref = oracle.attention(*(oracle.widen(x, dtype) for x in (qb, kb, vb)), scale, causal=causal)
        o, lse = _run(qb, kb, vb, dtype, scale, causal)
        if dtype == "bf16" and np.abs(o_ref).max() > 2.56:
            # with a handful of keys a row of O is close to one V row: beyond 2.56 in magnitude half an ulp of the
            # bf16 output alone exceeds the absolute bound, so there the bound is max(1e-2, |O| * 2^-7)
            assert np.all(np.isfinite(o)) and not np.any(lse == SENT32)
            assert np.all(np.abs(o - o_ref) <= np.maximum(TOL_O_MAX, np.abs(o_ref) * 2.0 ** -7)), f"random shape {n}"
            assert np.max(np.abs(lse - lse_ref)) <= TOL_LSE_MAX, f"random shape {n}"
        else:
            _check(o, lse, o_ref, lse_ref, f"random shape {n}")


@pytest.mark.parametrize("N,causal", [(2047, False), (2049, False), (2000, True)])
def test_ragged_headline_shape_whole_output(N, causal):
    # the headline shape with a length that is not a whole number of tiles: every element against the oracle
    B, H, d = 8, 16, 128
    print(f"ragged headline N={N} causal={causal}", flush=True)
    qb, kb, vb = workloads.make_qkv(B, N, H, d, "fp16", 9000 + N)
    scale = float(np.float32(d) ** np.float32(-0.5))
    o, lse = _run(qb, kb, vb, "fp16", scale, causal)
    o_ref, lse_ref = oracle.attention(*(oracle.widen(x, "fp16") for x in (qb, kb, vb)), scale, causal=causal)
    _check(o, lse, o_ref, lse_ref, f"B8 H16 N{N} d128 causal={causal} (whole output)")


def test_keys_past_the_end_are_invisible_bitwise():
    # Nq x Nk attention must not depend on what follows K and V in memory: running on the first Nk rows of a longer,
    # different K/V (as its own contiguous tensor) and on guarded buffers gives the same bits as any other padding.
    torch = torch_gpu()
    B, H, Nq, Nk, d = 1, 2, 150, 90, 128
    print("keys past the end", flush=True)
    qb, kb, vb = _make(B, H, Nq, Nk, d, "fp16", 4321)
    q, _ = _guarded(qb, "fp16")
    k1, _ = _guarded(kb, "fp16")
    v1, _ = _guarded(vb, "fp16")
    o1, l1 = fa2.fa2_fwd(q, k1, v1, 0.09)
    # same K/V followed directly by large finite values instead of the NaN guard
    big = torch.full((kb.size + PAD,), 60000.0, dtype=torch.float16, device="cuda")
    k2 = big.clone(); k2[:kb.size] = k1.reshape(-1)
    v2 = big.clone(); v2[:vb.size] = v1.reshape(-1)
    o2, l2 = fa2.fa2_fwd(q, k2[:kb.size].view(B, Nk, H, d), v2[:vb.size].view(B, Nk, H, d), 0.09)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    assert bool(torch.isfinite(o1).all())
