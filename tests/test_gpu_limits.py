"""GPU parity at the edges of the supported sizes: the longest sequences the workloads use times four, and a
batch entry just under the 4 GiB that the kernel's 32-bit K/V offsets can address."""
import numpy as np
import pytest

import oracle
import paper_2312_11918_amd as fa2
from paper_2312_11918_amd import workloads

pytestmark = pytest.mark.gpu

TOL_O_MAX, TOL_O_MEAN, TOL_LSE_MAX = 1e-2, 1e-3, 1e-3


def _torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _check(o_gpu, lse_gpu, o_ref, lse_ref, what):
    assert np.all(np.isfinite(o_gpu)) and np.all(np.isfinite(lse_gpu)), f"{what}: non-finite values"
    eo = np.abs(o_gpu - o_ref)
    el = np.abs(lse_gpu - lse_ref)
    print(f"{what}: max|dO|={eo.max():.3e} mean|dO|={eo.mean():.3e} max|dLSE|={el.max():.3e}", flush=True)
    assert eo.max() <= TOL_O_MAX and eo.mean() <= TOL_O_MEAN and el.max() <= TOL_LSE_MAX, what


@pytest.mark.parametrize("causal", [False, True])
def test_very_long_sequence_sampled(causal):
    # N = 65536: 1024 K/V tiles per Q tile, 512 Q tiles per head
    torch = _torch()
    B, H, N, d = 1, 2, 65536, 64
    print(f"long sequence N={N} causal={causal}", flush=True)
    qb, kb, vb = workloads.make_qkv(B, N, H, d, "fp16", 65536)
    q, k, v = (torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16) for x in (qb, kb, vb))
    o, lse = fa2.fa2_fwd(q, k, v, 0.125, causal=causal)
    torch.cuda.synchronize()
    o, lse = o.double().cpu().numpy(), lse.double().cpu().numpy()
    r = np.random.Generator(np.random.PCG64(5))
    n = 256
    rows = np.stack([np.zeros(n, dtype=np.int64), r.integers(0, H, n), r.integers(0, N, n)], axis=1).astype(np.int32)
    rows[0], rows[1], rows[2] = (0, 0, 0), (0, H - 1, N - 1), (0, 1, N - 129)
    qf, kf, vf = (oracle.widen(x, "fp16") for x in (qb, kb, vb))
    o_rows, lse_rows = oracle.attention_rows(qf, kf, vf, 0.125, rows, causal=causal)
    _check(o[0, rows[:, 2], rows[:, 1], :], lse[0, rows[:, 1], rows[:, 2]], o_rows, lse_rows, f"N={N} causal={causal}")
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))


@pytest.mark.timeout(600)
def test_batch_entry_just_under_4_gib_sampled_heads():
    # N * H * d * 2 bytes = 2^32 - 2^17: the last K/V rows of the last heads sit at byte offsets just below 2^32,
    # the largest the kernel's 32-bit buffer offsets reach (one more head is refused, checked below).
    torch = _torch()
    B, N, H, d, dtype = 1, 1024, 32767, 64, "bf16"
    base_h = 257
    print(f"large batch entry H={H} N={N} d={d}", flush=True)
    qb0, kb0, vb0 = workloads.make_qkv(1, N, base_h, d, dtype, 40961)   # [1, N, base_h, d]

    def spread(x):
        # head h of the big tensor is head h % base_h of the block, rotated along the sequence by h // base_h rows:
        # every head differs from every other, from 8 MiB of random numbers
        out = np.empty((1, N, H, d), dtype=np.uint16)
        for c in range((H + base_h - 1) // base_h):
            h0, h1 = c * base_h, min((c + 1) * base_h, H)
            out[0, :, h0:h1] = np.roll(x[0, :, :h1 - h0], c, axis=0)
        return out

    big = [spread(x) for x in (qb0, kb0, vb0)]
    q, k, v = (torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16) for x in big)
    scale = 0.125
    o, lse = fa2.fa2_fwd(q, k, v, scale)
    torch.cuda.synchronize()
    heads = np.array([0, 1, base_h, 12345, H - 258, H - 2, H - 1])
    sub = [oracle.widen(np.ascontiguousarray(x[:, :, heads]), dtype) for x in big]
    o_ref, lse_ref = oracle.attention(*sub, scale)
    hidx = torch.from_numpy(heads).cuda()
    o_g = o[:, :, hidx].double().cpu().numpy()
    lse_g = lse[:, hidx].double().cpu().numpy()
    _check(o_g, lse_g, o_ref, lse_ref, f"H={H} sampled heads")
    # a coarse look at everything else: finite, and inside the range of V
    assert bool(torch.isfinite(o).all()) and bool(torch.isfinite(lse).all())
    assert float(o.float().abs().max()) <= float(v.float().abs().max())
    # one more head crosses the 32-bit limit: refused without a launch
    rc = fa2.fa2_fwd_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), None, 1, H + 1, N, d, scale, fa2.FA2_BF16)
    assert rc == fa2.FA2_ERR_UNSUPPORTED
