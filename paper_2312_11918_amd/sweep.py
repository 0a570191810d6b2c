"""Tile-shape sweep in the manner of the paper's Table 1 (Section 7): times every kernel variant of libfa2
on a list of attention shapes and prints a table of forward TFLOP/s (4*B*H*N^2*d).

Usage:  python -m paper_2312_11918_amd.sweep [--paper] [--workloads] [--iters K]

  --paper      the paper's benchmark shapes: batch 4, N = 4096, (heads, head dim) = (32, 64), (16, 128), (8, 256), fp16
  --workloads  the five synthetic workloads of this repository (the default if nothing is selected)

Inputs are i.i.d. N(0,1), seeded; every variant's output is checked to be finite.
"""
from __future__ import annotations

import argparse
import sys

import numpy as np

VARIANTS = [("128 query rows x 64 keys (4 wavefronts x 32 rows, 2 workgroups/CU)", 1),
            ("256 query rows x 64 keys (8 wavefronts x 32 rows, 1 workgroup/CU, chained Q tiles)", 3),
            ("fa2_fwd's own choice", 0)]
PEAK = 2516.6


def _time(q, k, v, scale, variant, iters):
    import torch
    import paper_2312_11918_amd as fa2

    o = torch.empty_like(q)
    lse = torch.empty((q.shape[0], q.shape[2], q.shape[1]), dtype=torch.float32, device="cuda")
    for _ in range(max(3, iters // 10)):
        fa2.fa2_fwd(q, k, v, scale, out=o, lse=lse, variant=variant)
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fa2.fa2_fwd(q, k, v, scale, out=o, lse=lse, variant=variant)
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / iters)
    assert bool(torch.isfinite(o).all())
    return best


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--paper", action="store_true")
    ap.add_argument("--workloads", action="store_true")
    ap.add_argument("--iters", type=int, default=0, help="timed launches per region (0: about 50 ms worth)")
    args = ap.parse_args(argv)
    import torch
    import paper_2312_11918_amd as fa2
    from paper_2312_11918_amd import workloads

    if not torch.cuda.is_available():
        print("sweep: no GPU visible", file=sys.stderr)
        return 2
    fa2.load_library()
    shapes = []
    if args.paper:
        shapes += [("paper B4 H32 N4096 d64 fp16", 4, 32, 4096, 64, "fp16", 0.0, 1.0, 4096 + 64),
                   ("paper B4 H16 N4096 d128 fp16", 4, 16, 4096, 128, "fp16", 0.0, 1.0, 4096 + 128),
                   ("paper B4 H8 N4096 d256 fp16", 4, 8, 4096, 256, "fp16", 0.0, 1.0, 4096 + 256)]
    if args.workloads or not shapes:
        for i in sorted(workloads.CONFIGS):
            w = workloads.CONFIGS[i]
            shapes.append((w.name, w.B, w.H, w.N, w.d, w.dtype, w.k_outlier_frac, w.k_outlier_gain, w.seed))
    print("| shape | " + " | ".join(name for name, _ in VARIANTS) + f" | best, % of {PEAK} |")
    print("|---|" + "---|" * (len(VARIANTS) + 1))
    for name, B, H, N, d, dtype, frac, gain, seed in shapes:
        qb, kb, vb = workloads.make_qkv(B, N, H, d, dtype, seed, frac, gain)
        tdt = torch.float16 if dtype == "fp16" else torch.bfloat16
        q, k, v = (torch.from_numpy(x.view(np.int16)).cuda().view(tdt) for x in (qb, kb, vb))
        scale = float(np.float32(d) ** np.float32(-0.5))
        flops = 4.0 * B * H * float(N) ** 2 * d
        iters = args.iters or int(min(max(50e-3 / (flops / 0.8e15), 5), 500))
        cells = []
        for _, variant in VARIANTS:
            # only the default shape runs d = 256; the 256-row shape needs whole 256-row tiles
            if variant == 3 and (d > 128 or N % 256 != 0):
                cells.append(None)
                continue
            ms = _time(q, k, v, scale, variant, iters)
            cells.append(flops / (ms * 1e-3) / 1e12)
        best = max(c for c in cells if c is not None)
        print(f"| {name} | " + " | ".join("n/a" if c is None else f"{c:.0f}" for c in cells)
              + f" | {100 * best / PEAK:.1f} |", flush=True)
        del q, k, v
    return 0


if __name__ == "__main__":
    sys.exit(main())
