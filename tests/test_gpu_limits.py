"""GPU parity at the edges of the supported sizes: the longest sequences the workloads use times four, and a
batch entry just under the 4 GiB that the kernel's 32-bit K/V offsets can address."""
import numpy as np
import pytest

import oracle
import paper_2312_11918_amd as fa2
from paper_2312_11918_amd import workloads
from _gpu_common import check, rows_one_per_tile, torch_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("causal", [False, True])
def test_very_long_sequence_one_row_per_query_tile(causal):
    # N = 65536: 1024 K/V tiles per Q tile, 512 Q tiles per head
    torch = torch_gpu()
    B, H, N, d = 1, 2, 65536, 64
    print(f"long sequence N={N} causal={causal}", flush=True)
    qb, kb, vb = workloads.make_qkv(B, N, H, d, "fp16", 65536)
    q, k, v = (torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16) for x in (qb, kb, vb))
    o, lse = fa2.fa2_fwd(q, k, v, 0.125, causal=causal)
    torch.cuda.synchronize()
    o, lse = o.double().cpu().numpy(), lse.double().cpu().numpy()
    # one row in every 128-row query tile of both heads (1024 workgroups, or 512 pairs under the mask), plus corners
    rows = rows_one_per_tile(B, H, N, 128, 5 + int(causal))
    rows[2] = (0, 1, N - 129)
    qf, kf, vf = (oracle.widen(x, "fp16") for x in (qb, kb, vb))
    o_rows, lse_rows = oracle.attention_rows(qf, kf, vf, 0.125, rows, causal=causal)
    check(o[0, rows[:, 2], rows[:, 1], :], lse[0, rows[:, 1], rows[:, 2]], o_rows, lse_rows, f"N={N} causal={causal}")
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))


@pytest.mark.timeout(600)
def test_batch_entry_just_under_4_gib_sampled_heads():
    # N * H * d * 2 bytes = 2^32 - 2^17: the last K/V rows of the last heads sit at byte offsets just below 2^32,
    # the largest the kernel's 32-bit buffer offsets reach (one more head is refused, checked below).
    torch = torch_gpu()
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
    check(o_g, lse_g, o_ref, lse_ref, f"H={H} sampled heads")
    # a coarse look at everything else: finite, and inside the range of V
    assert bool(torch.isfinite(o).all()) and bool(torch.isfinite(lse).all())
    assert float(o.float().abs().max()) <= float(v.float().abs().max())
    # one more head crosses the 32-bit limit: refused without a launch
    rc = fa2.fa2_fwd_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), None, 1, H + 1, N, d, scale, fa2.FA2_BF16)
    assert rc == fa2.FA2_ERR_UNSUPPORTED
