"""Helpers shared by the GPU parity tests: device transfer, one launch through the C ABI, the tolerance check.

Tolerances (fp16/bf16 N(0,1) inputs): max |dO| <= 1e-2, mean |dO| <= 1e-3, max |dLSE| <= 1e-3.
"""
import numpy as np

import paper_2312_11918_amd as fa2

TOL_O_MAX, TOL_O_MEAN, TOL_LSE_MAX = 1e-2, 1e-3, 1e-3


def torch_gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def to_device(bits, dtype):
    """uint16 bit patterns -> device tensor of the 16-bit float type."""
    torch = torch_gpu()
    t = torch.from_numpy(bits.view(np.int16)).cuda()
    return t.view(torch.float16 if dtype == "fp16" else torch.bfloat16)


def run_gpu(qb, kb, vb, dtype, scale, variant=0, causal=False, bits=False):
    """One launch on NaN-prefilled outputs.  Returns (O [B,N,H,d], LSE [B,H,N]) as fp64 numpy arrays, or with
    ``bits`` as (uint16 bit patterns of O, fp32 LSE)."""
    torch = torch_gpu()
    q, k, v = (to_device(x, dtype) for x in (qb, kb, vb))
    o = torch.full_like(q, float("nan"))
    lse = torch.full((q.shape[0], q.shape[2], q.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
    fa2.fa2_fwd(q, k, v, scale, out=o, lse=lse, variant=variant, causal=causal)
    torch.cuda.synchronize()
    if bits:
        return o.view(torch.int16).cpu().numpy().view(np.uint16), lse.cpu().numpy()
    return o.double().cpu().numpy(), lse.double().cpu().numpy()


def check(o_gpu, lse_gpu, o_ref, lse_ref, what):
    """Element-by-element comparison with the oracle's values, to the stated tolerances."""
    assert np.all(np.isfinite(o_gpu)), f"{what}: O has non-finite values"
    assert np.all(np.isfinite(lse_gpu)), f"{what}: LSE has non-finite values"
    eo = np.abs(o_gpu - o_ref)
    el = np.abs(lse_gpu - lse_ref)
    print(f"{what}: max|dO|={eo.max():.3e} mean|dO|={eo.mean():.3e} max|dLSE|={el.max():.3e} "
          f"({eo.size} elements of O, {el.size} of LSE)", flush=True)
    assert eo.max() <= TOL_O_MAX, f"{what}: max |dO| {eo.max():.3e}"
    assert eo.mean() <= TOL_O_MEAN, f"{what}: mean |dO| {eo.mean():.3e}"
    assert el.max() <= TOL_LSE_MAX, f"{what}: max |dLSE| {el.max():.3e}"


def rows_one_per_tile(B, H, N, tile, seed, extra=0):
    """Sampled (batch, head, row) triples with at least one row in EVERY query tile of every head (row = tile start +
    a random offset), plus ``extra`` uniformly drawn rows and the corners."""
    r = np.random.Generator(np.random.PCG64(seed))
    n_tiles = (N + tile - 1) // tile
    b, h, t = np.meshgrid(np.arange(B), np.arange(H), np.arange(n_tiles), indexing="ij")
    i = np.minimum(t * tile + r.integers(0, tile, t.shape), N - 1)
    rows = np.stack([b.ravel(), h.ravel(), i.ravel()], axis=1)
    if extra:
        rows = np.concatenate([rows, np.stack([r.integers(0, B, extra), r.integers(0, H, extra),
                                               r.integers(0, N, extra)], axis=1)])
    corners = np.array([(0, 0, 0), (B - 1, H - 1, N - 1), (0, H - 1, min(127, N - 1)), (B - 1, 0, min(128, N - 1))])
    return np.concatenate([corners, rows]).astype(np.int32)
