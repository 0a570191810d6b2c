"""GPU parity of the causal mask (fa2_fwd_masked, FA2_MASK_CAUSAL) against the fp64 CPU oracle's masked
standard attention on the same seeded bits.  Tolerances are those of the unmasked path."""
import numpy as np
import pytest

import oracle
import paper_2312_11918_amd as fa2
from paper_2312_11918_amd import workloads
from _gpu_common import TOL_LSE_MAX, check, run_gpu, to_device, torch_gpu

pytestmark = pytest.mark.gpu



def _run_gpu(qb, kb, vb, dtype, scale, causal=True, bits=False):
    return run_gpu(qb, kb, vb, dtype, scale, causal=causal, bits=bits)


@pytest.mark.parametrize("B,H,N,d,dtype,outliers", [
    (1, 2, 128, 64, "fp16", 0.0),     # one Q tile: every K/V tile is a diagonal tile
    (2, 2, 128, 128, "bf16", 0.0),
    (1, 2, 256, 64, "fp16", 0.0),     # workload 1 shape: 2 Q tiles
    (2, 3, 384, 64, "fp16", 0.02),    # 3 Q tiles, large-logit keys
    (1, 2, 640, 128, "fp16", 0.02),   # 5 Q tiles: 2..10 K/V tiles per workgroup
    (1, 3, 896, 128, "bf16", 0.0),
    (1, 5, 1152, 64, "bf16", 0.0),    # 45 workgroups: not a multiple of the 8 XCDs
    (3, 1, 1024, 128, "fp16", 0.0),
    (1, 2, 384, 256, "fp16", 0.0),    # d = 256
    (2, 1, 512, 256, "bf16", 0.0),
    (16, 16, 2304, 128, "fp16", 0.0),  # 256-row shape: 9 Q tiles per head, the middle one unpaired (no chain)
    (4, 16, 4096, 128, "bf16", 0.0),   # 256-row shape: 512 pairs, every workgroup chains two of them
])
def test_causal_parity_elementwise(B, H, N, d, dtype, outliers):
    seed = 3000 + 5 * N + d + B
    print(f"causal case B={B} H={H} N={N} d={d} {dtype} seed={seed}", flush=True)
    qb, kb, vb = workloads.make_qkv(B, N, H, d, dtype, seed, k_outlier_frac=outliers, k_outlier_gain=6.0)
    scale = float(np.float32(d) ** np.float32(-0.5))
    o_ref, lse_ref = oracle.attention(*(oracle.widen(x, dtype) for x in (qb, kb, vb)), scale, causal=True)
    o, lse = _run_gpu(qb, kb, vb, dtype, scale)
    check(o, lse, o_ref, lse_ref, f"causal B{B} H{H} N{N} d{d} {dtype}")
    # the first rows, with the fewest visible keys, are where a mask that is off by one shows most
    check(o[:, :4], lse[:, :, :4], o_ref[:, :4], lse_ref[:, :, :4], "first four rows")


@pytest.mark.parametrize("index", [2, 3, 4, 5])
def test_causal_parity_full_size_workloads(index):
    # the masked Algorithm 1 in fp64 over the whole workload: every element of O and LSE of every workgroup
    w, qb, kb, vb = workloads.make_workload(index)
    print(f"causal workload {index} {w.name} seed={w.seed}", flush=True)
    o, lse = _run_gpu(qb, kb, vb, w.dtype, w.scale)
    q, k, v = (oracle.widen(x, w.dtype) for x in (qb, kb, vb))
    o_ref, lse_ref = oracle.attention(q, k, v, w.scale, causal=True)
    check(o, lse, o_ref, lse_ref, f"causal {w.name} (whole output)")
    # row 0 sees key 0 only: P = 1 exactly, so O_0 is V_0 to the bit and LSE_0 = scale * q_0 . k_0
    assert np.array_equal(o[:, 0], v[:, 0]), "row 0 must reproduce V row 0 exactly"
    s00 = w.scale * np.einsum("bhk,bhk->bh", q[:, 0], k[:, 0])
    assert np.max(np.abs(lse[:, :, 0] - s00)) <= TOL_LSE_MAX


def test_causal_prefix_property_bitwise():
    # Rows 0..M-1 of a causal call never see keys >= M: they must equal, bit for bit, a causal call on the
    # length-M prefix (the kernel visits the same tiles in the same order for them).
    B, H, N, d, M = 2, 4, 2048, 128, 768
    print("causal prefix property", flush=True)
    qb, kb, vb = workloads.make_qkv(B, N, H, d, "fp16", 5151)
    o_full, lse_full = _run_gpu(qb, kb, vb, "fp16", 0.09, bits=True)
    o_pre, lse_pre = _run_gpu(*(np.ascontiguousarray(x[:, :M]) for x in (qb, kb, vb)), "fp16", 0.09, bits=True)
    assert np.array_equal(o_full[:, :M], o_pre)
    assert np.array_equal(lse_full[:, :, :M].view(np.uint32), lse_pre.view(np.uint32))


def test_future_keys_and_values_do_not_matter():
    # Changing K and V at positions > i must leave row i unchanged bit for bit.
    B, H, N, d, cut = 1, 3, 1024, 64, 517
    print("causal independence of the future", flush=True)
    qb, kb, vb = workloads.make_qkv(B, N, H, d, "bf16", 6161)
    kb2, vb2 = kb.copy(), vb.copy()
    _, kx, vx = workloads.make_qkv(B, N, H, d, "bf16", 6162, k_outlier_frac=0.1, k_outlier_gain=8.0)
    kb2[:, cut + 1:] = kx[:, cut + 1:]
    vb2[:, cut + 1:] = vx[:, cut + 1:]
    o1, l1 = _run_gpu(qb, kb, vb, "bf16", 0.125, bits=True)
    o2, l2 = _run_gpu(qb, kb2, vb2, "bf16", 0.125, bits=True)
    assert np.array_equal(o1[:, :cut + 1], o2[:, :cut + 1])
    assert np.array_equal(l1[:, :, :cut + 1].view(np.uint32), l2[:, :, :cut + 1].view(np.uint32))
    assert not np.array_equal(o1[:, cut + 1:], o2[:, cut + 1:])


def test_mask_none_is_the_unmasked_entry_point_and_bad_masks_are_refused():
    torch = torch_gpu()
    B, H, N, d = 1, 2, 384, 128
    print("masked entry with FA2_MASK_NONE", flush=True)
    qb, kb, vb = workloads.make_qkv(B, N, H, d, "fp16", 7171)
    q, k, v = (to_device(x, "fp16") for x in (qb, kb, vb))
    o1, l1 = fa2.fa2_fwd(q, k, v, 0.1)
    o2 = torch.full_like(q, float("nan"))
    l2 = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    rc = fa2.fa2_fwd_masked_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o2.data_ptr(), l2.data_ptr(), B, H, N, d, 0.1,
                                fa2.FA2_FP16, fa2.FA2_MASK_NONE, s)
    assert rc == fa2.FA2_OK
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    o3 = torch.full_like(q, 7.0)
    rc = fa2.fa2_fwd_masked_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o3.data_ptr(), None, B, H, N, d, 0.1,
                                fa2.FA2_FP16, 5, s)
    assert rc == fa2.FA2_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert bool((o3 == 7.0).all()), "a refused call must leave O untouched"
