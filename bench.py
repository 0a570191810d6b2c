#!/usr/bin/env python3
"""Benchmark of the fused attention forward pass (libfa2) on one MI355X.

One "step" is one complete forward pass (one fa2_fwd launch: Q-tile scheduling, K/V staging,
GEMM-I, online softmax, GEMM-II, epilogue) over one synthetic batch that is already resident in
HBM.  The headline workload is B=8, H=16, N=2048, d=128, fp16 (the shape the 50%-of-MFMA-peak
target is stated for); the other four workloads are timed as well and reported under
"workloads".  FLOPs are those of the two matmuls only, 4*B*H*N^2*d (Section 7 of the paper).

Prints ONE JSON line.  `roofline` prices the kernel against the published dense fp16/bf16 MFMA
peak of MI355X; `cpu_baseline` is the fp64 CPU oracle timed on this host on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2516.6      # MI355X dense fp16 = bf16 matrix peak (256 CU x 4096 FLOP/clk x 2.4 GHz)
HBM_PEAK_GBS = 8000.0
HEADLINE = 3

VALU_LANES_PER_CLK_CU = 64.0   # plain (unpacked) fp32 vector rate: 4 SIMDs x 16 lanes per clock
ENGINE_CLOCK_HZ = 2.4e9
N_CUS = 256
# Vector-pipe issue slots per element of S in the steady-state softmax of the kernel as built: fma (1) + exp2 (2: the
# exponential is a half-rate instruction) + rowsum add (1) + half a 16-bit pack (0.5).  (The row maximum is only
# taken on first, masked and overflowing tiles.)
SOFTMAX_VALU_SLOTS_PER_ELEMENT = 4.5

# HBM bytes per launch as profiled with rocprofv3 --pmc (FETCH_SIZE KiB x 2.0 + WRITE_SIZE KiB x 1.0, factors from a
# plain 64 MiB device copy in the same runs); not measured by this script.  Each entry names the summary it is from.
PROFILED_TRAFFIC = {
    "B8_H16_N2048_d128_fp16": {"bytes": 270025349, "algorithmic_bytes": 269484032,
                               "profile": "profiles/fa2_fwd_fp16_d128_B8_H16_N2048.txt"},
    "B32_H16_N512_d64_fp16": {"bytes": 135441756, "algorithmic_bytes": 135266304,
                              "profile": "profiles/fa2_fwd_fp16_d64_B32_H16_N512.txt"},
    "B2_H16_N8192_d128_bf16": {"bytes": 270027304, "algorithmic_bytes": 269484032,
                               "profile": "profiles/fa2_fwd_bf16_d128_B2_H16_N8192.txt"},
    # one head's K and V (4 MiB) equal an XCD's L2 and the 64 query tiles of a head do not all run at once: K/V are
    # fetched about twice per head.  386.5 MiB per 2.3 ms launch is 2 % of the HBM bandwidth.
    "B1_H32_N16384_d64_fp16_koutliers": {"bytes": 405250232, "algorithmic_bytes": 270532608,
                                         "profile": "profiles/fa2_fwd_fp16_d64_B1_H32_N16384_koutliers.txt"},
}


_CUSTOM = {}


def _custom_workload(spec):
    """Registers a workload `B,H,N,d,dtype` (e.g. 4,8,4096,256,fp16) under index 0, same input recipe as the five."""
    from paper_2312_11918_amd import workloads

    B, H, N, d, dtype = spec.split(",")
    B, H, N, d = int(B), int(H), int(N), int(d)
    # index 100 + ... only feeds the seed (SEED_BASE + index); it is not one of the numbered workloads
    _CUSTOM[0] = workloads.Workload(100 + (N + d) % 1000, f"B{B}_H{H}_N{N}_d{d}_{dtype}", B, H, N, d, dtype)
    return 0


def _make(index):
    from paper_2312_11918_amd import workloads

    if index in _CUSTOM:
        w = _CUSTOM[index]
        return (w,) + tuple(workloads.make_qkv(w.B, w.N, w.H, w.d, w.dtype, w.seed))
    return workloads.make_workload(index)


def _device_tensors(index):
    import torch

    w, qb, kb, vb = _make(index)
    tdt = torch.float16 if w.dtype == "fp16" else torch.bfloat16
    q, k, v = (torch.from_numpy(x.view(np.int16)).cuda().view(tdt) for x in (qb, kb, vb))
    return w, q, k, v


def _prepare(index):
    """Device tensors of a workload plus its output buffers."""
    import torch

    w, q, k, v = _device_tensors(index)
    o = torch.empty_like(q)
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
    return w, q, k, v, o, lse


def _launcher(prep, causal):
    import torch
    import paper_2312_11918_amd as fa2

    w, q, k, v, o, lse = prep
    stream = torch.cuda.current_stream()

    def run(n):
        """n back-to-back launches between two HIP events recorded on the launch stream; returns ms per launch."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(n):
            fa2.fa2_fwd(q, k, v, w.scale, out=o, lse=lse, stream=stream, causal=causal)
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / n

    return run


def _time_prepared(prep, steps, warmup, causal=False, n_regions=5, min_region_ms=50.0, settle_ms=100.0):
    """Times one workload.  Returns a dict:
      first_region_ms   ms per launch of the FIRST timed region: exactly `steps` launches right after `warmup`
                        untimed ones (the clock and power state of the chip are still settling then);
      regions_ms        ms per launch of `n_regions` further regions, each of max(steps, enough launches for
                        `min_region_ms`), taken after at least `settle_ms` of launches and once two consecutive
                        regions agree within 2 % (at most 20 tries);
      ms                their median -- the figure reported as ms_per_step;
      wall_ms           host wall clock per launch over the first region (launch overhead included).
    """
    import torch

    run = _launcher(prep, causal)
    for _ in range(max(warmup, 0)):
        run(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    first = run(steps)
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    n = max(steps, int(min_region_ms / max(first, 1e-4)) + 1)
    spent, prev = first * steps, None
    for _ in range(20 if n_regions > 0 else 0):
        cur = run(n)
        spent += cur * n
        if spent >= settle_ms and prev is not None and abs(cur - prev) <= 0.02 * prev:
            break
        prev = cur
    regions = [run(n) for _ in range(n_regions)]
    assert bool(torch.isfinite(prep[4]).all()), "non-finite output"
    return {"ms": float(np.median(regions)) if regions else first, "first_region_ms": first, "regions_ms": sorted(regions),
            "launches_per_region": n, "wall_ms": wall_ms}


def _time_workload(index, steps, warmup, causal=False):
    """Prepares the workload, times it, frees it; returns (workload, timing dict)."""
    import torch

    prep = _prepare(index)
    t = _time_prepared(prep, steps, warmup, causal)
    w = prep[0]
    del prep
    torch.cuda.empty_cache()
    return w, t


def _roofs(w, ms, causal=False):
    """The workload's throughput against the roofs that can bound it: the matrix cores (published dense peak), the
    vector pipe (the softmax's issue slots; binds before the matrix cores when 4 d FLOPs per element of S take less
    matrix time than the softmax takes vector time, i.e. for small d) and HBM (the algorithmic bytes at 8 TB/s)."""
    flops = w.flops * (0.5 if causal else 1.0)
    tf = flops / (ms * 1e-3) / 1e12
    elements = w.B * w.H * float(w.N) ** 2 * (0.5 if causal else 1.0)
    alu_elems_per_s = N_CUS * ENGINE_CLOCK_HZ * VALU_LANES_PER_CLK_CU / SOFTMAX_VALU_SLOTS_PER_ELEMENT
    alu_roof_tf = alu_elems_per_s * 4.0 * w.d / 1e12      # the same FLOP count, at the rate the softmax allows
    alg_bytes = 4 * w.B * w.H * w.N * w.d * 2 + 4 * w.B * w.H * w.N
    hbm_ms = alg_bytes / (HBM_PEAK_GBS * 1e9) * 1e3
    return {"tflops": round(tf, 2), "frac_mfma_peak": round(tf / MFMA_PEAK_TFLOPS, 4),
            "alu_roof_tflops": round(alu_roof_tf, 1), "frac_alu_roof": round(tf / alu_roof_tf, 4),
            "softmax_elements_per_s": round(elements / (ms * 1e-3), 0),
            "hbm_gbs_algorithmic": round(alg_bytes / (ms * 1e-3) / 1e9, 1), "hbm_floor_ms": round(hbm_ms, 5),
            "frac_hbm_roof": round(hbm_ms / ms, 4),
            "binding_roof": min((("mfma", MFMA_PEAK_TFLOPS), ("alu", alu_roof_tf),
                                 ("hbm", flops / (hbm_ms * 1e-3) / 1e12)), key=lambda r: r[1])[0]}


def _mfma_roof(kind, dtype, seed=7):
    """MFMA-only throughput on this box with `kind` operands ("normal": N(0,1) values as in the workloads,
    "constant": all ones), and the engine clock during that run.  Uses libfa2_probe (include/fa2_probe.h)."""
    import torch
    import paper_2312_11918_amd as fa2
    from paper_2312_11918_amd import workloads

    n16 = fa2.FA2_PROBE_OPERAND_BYTES // 2
    if kind == "normal":
        vals = np.random.Generator(np.random.PCG64(seed)).standard_normal(n16, dtype=np.float32)
    else:
        vals = np.ones(n16, dtype=np.float32)
    ops = torch.from_numpy(workloads.round_to_bits(vals, dtype).view(np.int16)).cuda()
    ticks = torch.zeros(4, dtype=torch.int64, device="cuda")
    sink = torch.empty(fa2.FA2_PROBE_WORKGROUPS * 256, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    dt = fa2.FA2_FP16 if dtype == "fp16" else fa2.FA2_BF16
    iters = 20000  # 3.4e12 FLOP per launch, about 2 ms

    def launch():
        rc = fa2.fa2_probe_mfma_raw(ops.data_ptr(), ticks.data_ptr(), sink.data_ptr(), dt, iters, stream.cuda_stream)
        assert rc == 0, f"fa2_probe_mfma returned {rc}"

    for _ in range(3):
        launch()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    e0.record(stream)
    for _ in range(reps):
        launch()
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    flops = fa2.FA2_PROBE_WORKGROUPS * 4 * iters * fa2.FA2_PROBE_MFMA_PER_ITER * 32768.0
    t = ticks.cpu().numpy()
    mhz = 100.0 * float(t[1] - t[0]) / max(float(t[3] - t[2]), 1.0)
    return {"tflops": round(flops / (ms * 1e-3) / 1e12, 1), "clock_mhz": round(mhz)}


def _cpu_baseline(index, target_seconds=15.0):
    """The fp64 oracle, as it stands, on this host's cores, on the first batch entries of the workload."""
    import oracle

    w, qb, kb, vb = _make(index)
    # calibration on one head, then as many whole batch entries as fit the time target
    sl = (slice(0, 1), slice(None), slice(0, 1))
    q1, k1, v1 = (oracle.widen(x[sl], w.dtype) for x in (qb, kb, vb))
    t0 = time.perf_counter()
    oracle.attention(q1, k1, v1, w.scale)
    t_head = time.perf_counter() - t0
    nb = int(max(1, min(w.B, target_seconds / max(t_head * w.H, 1e-9))))
    q, k, v = (oracle.widen(x[:nb], w.dtype) for x in (qb, kb, vb))
    t0 = time.perf_counter()
    oracle.attention(q, k, v, w.scale)
    dt = time.perf_counter() - t0
    flops = 4.0 * nb * w.H * float(w.N) ** 2 * w.d
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"batch entries 0..{nb - 1} of {w.B} (all {w.H} heads, N={w.N}, d={w.d}) of workload "
                      f"{w.name}: {flops / 1e9:.1f} GFLOP in {dt:.2f} s, fp64, gcc -O2 + OpenMP"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=HEADLINE, help="headline workload index (1..5)")
    ap.add_argument("--shape", default=None, metavar="B,H,N,d,dtype",
                    help="time this shape instead of a numbered workload (same seeded N(0,1) recipe), e.g. "
                         "4,8,4096,256,fp16; implies --only-headline")
    ap.add_argument("--causal", action="store_true",
                    help="time fa2_fwd_masked with the causal mask; FLOPs are then counted as 2*B*H*N^2*d")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--no-mfma-roof", action="store_true", help="skip the MFMA-only roof measurement")
    ap.add_argument("--only-headline", action="store_true",
                    help="time the headline launch only: no other workloads, no causal run, no MFMA roof")
    ap.add_argument("--regions", type=int, default=5,
                    help="timed regions after the first one; the reported value is their median (0: report the "
                         "first region, for short profiler runs)")
    ap.add_argument("--min-region-ms", type=float, default=50.0, help="minimum length of each of those regions")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="K",
                    help="first run K plain device copies of the headline Q tensor (a kernel of known HBM "
                         "traffic, for scaling rocprofv3's FETCH_SIZE/WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a single-GPU kernel; run with --gpus 1 "
              "(no multi-GPU sharding or collectives exist here)", file=sys.stderr)
        return 2

    import torch
    import paper_2312_11918_amd as fa2
    from paper_2312_11918_amd import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    fa2.load_library()   # fail loudly if the extension is not built
    if args.shape:
        args.workload = _custom_workload(args.shape)
        args.only_headline = True

    if args.copy_calibration > 0:
        wc, qc, _, _ = _device_tensors(args.workload)
        dst = torch.empty_like(qc)
        for _ in range(args.copy_calibration):
            dst.copy_(qc)
        torch.cuda.synchronize()
        print(f"copy calibration: {args.copy_calibration} copies of {qc.numel() * 2} bytes "
              f"(reads {qc.numel() * 2} B, writes {qc.numel() * 2} B each)", file=sys.stderr)
        del qc, dst

    prep = _prepare(args.workload)
    w = prep[0]
    t = _time_prepared(prep, args.steps, args.warmup, causal=args.causal, n_regions=args.regions,
                       min_region_ms=args.min_region_ms)
    ms = t["ms"]
    flops = w.flops * (0.5 if args.causal else 1.0)
    tflops = flops / (ms * 1e-3) / 1e12
    alg_bytes = 4 * w.B * w.H * w.N * w.d * 2 + 4 * w.B * w.H * w.N
    roofs = _roofs(w, ms, args.causal)

    per_workload = {}
    if not args.only_headline:
        for idx in sorted(workloads.CONFIGS):
            if idx == args.workload:
                wi, ti = w, t
            else:
                wi0 = workloads.CONFIGS[idx]
                si = int(min(max(10e-3 / max(wi0.flops / 0.4e15, 20e-6), 5), 400))
                wi, ti = _time_workload(idx, si, max(3, si // 10))
            entry = {"ms": round(ti["ms"], 5), "first_region_ms": round(ti["first_region_ms"], 5),
                     "launches_per_region": ti["launches_per_region"]}
            entry.update(_roofs(wi, ti["ms"]))
            prof = PROFILED_TRAFFIC.get(wi.name)
            entry["traffic_profiled"] = None if prof is None else prof
            per_workload[wi.name] = entry

    # the same shape under the causal mask (fa2_fwd_masked); FLOPs counted as half of the unmasked product
    causal = None
    if not args.only_headline:
        ct = _time_prepared(prep, args.steps, args.warmup, causal=True, n_regions=args.regions,
                            min_region_ms=args.min_region_ms)
        causal = {"ms": round(ct["ms"], 5), "first_region_ms": round(ct["first_region_ms"], 5),
                  "flops_counted": "2*B*H*N^2*d"}
        causal.update(_roofs(w, ct["ms"], causal=True))

    # the matrix-core roof of this box as measured now, on the workload's kind of operands and on constants
    roof = None
    if not (args.no_mfma_roof or args.only_headline):
        roof = {"normal_operands": _mfma_roof("normal", w.dtype), "constant_operands": _mfma_roof("constant", w.dtype)}
    del prep
    torch.cuda.empty_cache()

    prof = None if args.causal else PROFILED_TRAFFIC.get(w.name)
    out = {
        "metric": "attention fwd TFLOP/s (2*B*H*N^2*d, causal)" if args.causal else "attention fwd TFLOP/s (4*B*H*N^2*d)",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms, 5),
        "first_region_ms": round(t["first_region_ms"], 5),
        "regions": {"n": len(t["regions_ms"]), "launches_each": t["launches_per_region"],
                    "ms_per_launch": [round(x, 5) for x in t["regions_ms"]],
                    "value_is": "median of these regions (each >= --min-region-ms of back-to-back launches, taken "
                                "after the clock has settled); first_region_ms is the region of exactly --steps "
                                "launches right after --warmup"},
        "wall_ms_per_step": round(t["wall_ms"], 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp16" if w.dtype == "fp16" else "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "d": w.d, "causal": bool(args.causal),
                   "scale": "1/sqrt(d)", "inputs": "i.i.d. N(0,1), seeded, resident in HBM"},
        "roofline": {"bound": "mfma", "achieved": round(tflops, 2), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tflops / MFMA_PEAK_TFLOPS, 4),
                     "traffic": None if prof is None else prof["bytes"],
                     "traffic_source": None if prof is None else prof["profile"],
                     "algorithmic_flops_per_launch": flops, "algorithmic_hbm_bytes_per_launch": alg_bytes,
                     "kernel": "fa2_fwd_kernel", "kernel_ms": round(ms, 5),
                     "kernel_ms_is": "HIP events on the launch stream around back-to-back launches, per launch "
                                     "(one step = one launch of this kernel)",
                     "secondary": {k: roofs[k] for k in ("alu_roof_tflops", "frac_alu_roof", "hbm_floor_ms",
                                                          "frac_hbm_roof", "binding_roof")},
                     "mfma_roof_measured": roof,
                     "frac_of_measured_roof": None if roof is None else round(tflops / roof["normal_operands"]["tflops"], 4)},
        "workloads": per_workload,
        "causal_same_shape": causal,
        "paper_context": "H100 PCIe, fp16: 295.7 TFLOP/s best at d=128 (Table 1), 39% of its 756 TFLOP/s peak; not a target",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(args.workload)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
