"""Socket power and engine clock of the GPU while a kernel of this library runs back to back.

The published matrix-core peak of MI355X assumes the 2.4 GHz engine clock; what clock a launch really gets depends
on the power the chip draws, and that depends on the operand data.  This tool makes the dependence visible without
instrumenting any kernel: it keeps one kind of launch running for a few seconds (the attention forward pass or the
MFMA-only probe, on N(0,1) operands or on constants) while a host thread samples the system-management library
(librocm_smi64: socket power, the energy accumulator, the current engine clock, the power cap), and prints one
markdown row per case:

    python -m paper_2312_11918_amd.power_clock [--seconds 4] [--cases fwd3_normal,fwd3_const,...]

Nothing here is on the attention path.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import subprocess
import sys
import threading
import time

import numpy as np


class Smi:
    """The few read-only queries used here, through librocm_smi64's C API."""

    def __init__(self, device=0):
        self.lib = ctypes.CDLL("librocm_smi64.so")
        rc = self.lib.rsmi_init(ctypes.c_uint64(0))
        if rc != 0:
            raise RuntimeError(f"rsmi_init failed with {rc}")
        self.dv = ctypes.c_uint32(device)

        class Freqs(ctypes.Structure):
            _fields_ = [("has_deep_sleep", ctypes.c_bool), ("num_supported", ctypes.c_uint32),
                        ("current", ctypes.c_uint32), ("frequency", ctypes.c_uint64 * 33)]

        self._freqs = Freqs

    def power_w(self):
        p = ctypes.c_uint64(0)
        if self.lib.rsmi_dev_current_socket_power_get(self.dv, ctypes.byref(p)) == 0:
            return p.value / 1e6
        if self.lib.rsmi_dev_power_ave_get(self.dv, ctypes.c_uint32(0), ctypes.byref(p)) == 0:
            return p.value / 1e6
        return None

    def power_cap_w(self):
        p = ctypes.c_uint64(0)
        if self.lib.rsmi_dev_power_cap_get(self.dv, ctypes.c_uint32(0), ctypes.byref(p)) == 0:
            return p.value / 1e6
        return None

    def energy_j(self):
        e, ts, res = ctypes.c_uint64(0), ctypes.c_uint64(0), ctypes.c_float(0)
        if self.lib.rsmi_dev_energy_count_get(self.dv, ctypes.byref(e), ctypes.byref(res), ctypes.byref(ts)) == 0:
            return e.value * res.value * 1e-6  # the counter's unit is `res` micro-joules
        return None

    def sclk_mhz(self):
        f = self._freqs()
        if self.lib.rsmi_dev_gpu_clk_freq_get(self.dv, ctypes.c_int(0), ctypes.byref(f)) == 0 and f.num_supported > 0:
            return f.frequency[min(f.current, f.num_supported - 1)] / 1e6
        return None


def _amd_smi_snapshot():
    """One `amd-smi metric` reading (per-XCD clocks, power), as parsed JSON or None.  Slow (a process start)."""
    try:
        res = subprocess.run(["amd-smi", "metric", "--clock", "--power", "--json"], stdout=subprocess.PIPE,
                             stderr=subprocess.DEVNULL, text=True, timeout=20)
        return json.loads(res.stdout)
    except Exception:
        return None


def _gfx_clocks(snapshot):
    """The GFX clock readings (MHz) found in an amd-smi snapshot."""
    out = []

    def walk(node, path):
        if isinstance(node, dict):
            if "clk" in node and path and path[-1].lower().startswith("gfx"):
                v = node["clk"]
                v = v.get("value") if isinstance(v, dict) else v
                if isinstance(v, (int, float)):
                    out.append(float(v))
            for k, v in node.items():
                walk(v, path + [str(k)])
        elif isinstance(node, list):
            for v in node:
                walk(v, path)

    walk(snapshot, [])
    return out


def _sampler(smi, stop, samples, period):
    while not stop.is_set():
        samples.append((time.perf_counter(), smi.power_w(), smi.sclk_mhz()))
        time.sleep(period)


def _make_case(name):
    """Returns (launch function, FLOPs per launch, description) for a case name."""
    import torch

    import paper_2312_11918_amd as fa2
    from paper_2312_11918_amd import workloads

    kind, data = name.rsplit("_", 1)
    stream = torch.cuda.current_stream()
    if kind.startswith("fwd"):
        index = int(kind[3:])
        w = workloads.CONFIGS[index]
        tdt = torch.float16 if w.dtype == "fp16" else torch.bfloat16
        if data == "normal":
            _, qb, kb, vb = workloads.make_workload(index)
            q, k, v = (torch.from_numpy(x.view(np.int16)).cuda().view(tdt) for x in (qb, kb, vb))
        else:
            q, k, v = (torch.ones((w.B, w.N, w.H, w.d), dtype=tdt, device="cuda") for _ in range(3))
        o = torch.empty_like(q)
        lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")

        def launch():
            fa2.fa2_fwd(q, k, v, w.scale, out=o, lse=lse, stream=stream)

        return launch, w.flops, f"fa2_fwd {w.name}, {'N(0,1)' if data == 'normal' else 'all-ones'} inputs"
    if kind == "probe":
        n16 = fa2.FA2_PROBE_OPERAND_BYTES // 2
        vals = (np.random.Generator(np.random.PCG64(7)).standard_normal(n16, dtype=np.float32) if data == "normal"
                else np.ones(n16, dtype=np.float32))
        ops = torch.from_numpy(workloads.round_to_bits(vals, "fp16").view(np.int16)).cuda()
        ticks = torch.zeros(4, dtype=torch.int64, device="cuda")
        sink = torch.empty(fa2.FA2_PROBE_WORKGROUPS * 256, dtype=torch.float32, device="cuda")
        iters = 4000

        def launch():
            rc = fa2.fa2_probe_mfma_raw(ops.data_ptr(), ticks.data_ptr(), sink.data_ptr(), fa2.FA2_FP16, iters,
                                        stream.cuda_stream)
            assert rc == 0

        flops = fa2.FA2_PROBE_WORKGROUPS * 4 * iters * fa2.FA2_PROBE_MFMA_PER_ITER * 32768.0
        return launch, flops, f"MFMA-only probe, {'N(0,1)' if data == 'normal' else 'all-ones'} fp16 operands"
    raise ValueError(f"unknown case {name!r}")


def run_case(smi, name, seconds, period=0.02):
    import torch

    launch, flops, what = _make_case(name)
    stream = torch.cuda.current_stream()
    for _ in range(10):
        launch()
    torch.cuda.synchronize()
    # chunk length of about 20 ms, found from one timed chunk
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(10):
        launch()
    e1.record(stream)
    torch.cuda.synchronize()
    per = e0.elapsed_time(e1) / 10.0
    chunk = max(1, int(20.0 / per))

    samples, stop = [], threading.Event()
    th = threading.Thread(target=_sampler, args=(smi, stop, samples, period))
    snap_box = []
    snap_th = threading.Thread(target=lambda: (time.sleep(seconds * 0.4), snap_box.append(_amd_smi_snapshot())))
    en0 = smi.energy_j()
    t0 = time.perf_counter()
    th.start()
    snap_th.start()
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record(stream)
    pending = []
    launches = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(chunk):
            launch()
        launches += chunk
        ev = torch.cuda.Event()
        ev.record(stream)
        pending.append(ev)
        if len(pending) > 2:          # at most three chunks queued: the GPU never idles, the queue stays short
            pending.pop(0).synchronize()
    end.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    en1 = smi.energy_j()
    stop.set()
    th.join()
    snap_th.join()
    ms = start.elapsed_time(end)
    # leave out the ramp at both ends
    mid = [(p, c) for (t, p, c) in samples if t0 + 0.5 <= t <= t1 - 0.2]
    powers = [p for p, _ in mid if p is not None]
    clocks = [c for _, c in mid if c is not None]
    xcd = _gfx_clocks(snap_box[0]) if snap_box and snap_box[0] is not None else []
    return {
        "case": name, "what": what, "launches": launches, "seconds": round(ms / 1e3, 3),
        "tflops": round(flops * launches / (ms * 1e-3) / 1e12, 1),
        "power_w_median": None if not powers else round(float(np.median(powers)), 1),
        "power_w_max": None if not powers else round(float(np.max(powers)), 1),
        "power_w_from_energy_counter": None if en0 is None or en1 is None else round((en1 - en0) / (t1 - t0), 1),
        "sclk_mhz_median": None if not clocks else round(float(np.median(clocks))),
        "sclk_mhz_min": None if not clocks else round(float(np.min(clocks))),
        "xcd_gfx_clocks_mhz": [round(x) for x in xcd],
        "samples": len(mid),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seconds", type=float, default=4.0)
    ap.add_argument("--cases", default="fwd3_normal,fwd3_const,probe_normal,probe_const,fwd4_normal,fwd2_normal")
    args = ap.parse_args()
    import torch

    import paper_2312_11918_amd as fa2

    if not torch.cuda.is_available():
        print("power_clock: no GPU visible", file=sys.stderr)
        return 2
    fa2.load_library()
    smi = Smi(0)
    time.sleep(1.0)
    idle = {"power_w": smi.power_w(), "sclk_mhz": smi.sclk_mhz(), "power_cap_w": smi.power_cap_w()}
    print(f"idle: {json.dumps(idle)}", flush=True)
    rows = []
    for name in args.cases.split(","):
        print(f"case {name} ...", flush=True)
        r = run_case(smi, name, args.seconds)
        print(json.dumps(r), flush=True)
        rows.append(r)
        torch.cuda.empty_cache()
        time.sleep(1.0)
    print()
    print(f"power cap {idle['power_cap_w']} W; idle {idle['power_w']} W at {idle['sclk_mhz']} MHz")
    print("| case | TFLOP/s | socket power W (median / max of samples) | W from the energy counter | "
          "engine clock MHz (median / min) | per-XCD GFX clocks MHz (one amd-smi reading) |")
    print("|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['what']} | {r['tflops']} | {r['power_w_median']} / {r['power_w_max']} | "
              f"{r['power_w_from_energy_counter']} | {r['sclk_mhz_median']} / {r['sclk_mhz_min']} | "
              f"{' '.join(str(x) for x in r['xcd_gfx_clocks_mhz']) or '-'} |")
    return 0


if __name__ == "__main__":
    sys.exit(main())
