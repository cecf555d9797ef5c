"""Benchmark of the AdaScale step on one MI355X.

`python bench.py --gpus 1 --steps K --warmup W` times K whole adascale_step calls (mean gradient
and norms, scalars, update: one fused kernel or three) on synthetic gradients already resident in HBM and prints ONE
JSON line.  The workload is the configuration the headline metric is quoted on: d = 25,557,032
parameters in 161 tensors (bottleneck-CNN-like shapes), S = 16 fp32 gradient buffers.

value        = gradient bytes streamed per second (S*d*4 / step time), GB/s
roofline     = the dominant kernel against the 8 TB/s HBM peak, algorithmic bytes of one launch /
               its average duration from HIP events on the launch stream inside the timed region:
               the fused step kernel (whole step, S*d*b + 24*d bytes, 20*d without weight decay) when the library runs the
               step as one persistent launch, else the first kernel of the three-kernel step (the
               gradient sweep: S*d*b read, plus 4*d written for the mean gradient or, in the
               streaming kernel, v read and written and w read under weight decay)
cpu_baseline = the CPU oracle (OpenMP build of the same source) on the host, one step of the
               same workload
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBPS = 8000.0
# HBM bytes one launch of the dominant kernel moves, from the rocprofv3 counter runs summarised under
# profiles/ (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000, the factors a 1 GiB copy calibrates): the
# "traffic" figure of the roofline object for the configurations that were profiled.
TRAFFIC_BYTES = {
    "k_fused_cfg2": 538000000,
    "k_fused_cfg3": 2048400000,
    "k_fused_cfg4": 4962100000,
    "k_reduce_stream_cfg3": 1951900000,
    "k_reduce_stream_cfg5": 47825500000,
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (3 = the headline configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not record per-kernel events inside the timed region")
    ap.add_argument("--lagged", action="store_true",
                    help="time the prior-iteration-gain variant (App. B.3), a single sweep of S*d*b + 16*d bytes")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 1 GiB a few times (the known-size kernel that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import workloads as W
    from paper_2007_05105_amd import AdaScale

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        n = 1 << 28                                   # 2^28 fp32 = 1 GiB read + 1 GiB written per copy
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "torch copy_ kernel", "bytes_read": 4 * n, "bytes_written": 4 * n, "launches": 5}))
        return 0
    wl = W.config(args.config)
    inp = W.Inputs(wl, "cuda:0")
    inp.fill_grads(0)
    gpu = AdaScale(wl.numel, wl.S, wl.lr_table, wl.momentum, wl.weight_decay, wl.theta, wl.eps,
                   wl.grad_dtype, 0, flags=1 if args.lagged else 0)
    arr = lambda ts: (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
    pw, pv = arr(inp.w), arr(inp.v)
    pg = arr([t for g in inp.g for t in g])
    stream = torch.cuda.current_stream()
    sh = int(stream.cuda_stream)

    def run(n: int) -> None:
        for _ in range(n):
            rc = gpu.step_raw(pw, pv, pg, sh)
            if rc != 0:
                raise RuntimeError(gpu.last_error())

    run(args.warmup)
    torch.cuda.synchronize()
    path = gpu.step_path()
    fused = path == "fused"
    # Per-kernel HIP events (recorded by the library on the launch stream) for the three-kernel
    # step.  The fused step is a single kernel per step: one pair of events on the launch stream
    # around the K launches gives its average duration without putting an event between every
    # two launches.
    events = not args.no_kernel_events and not fused
    if events:
        gpu.profile_begin(args.steps)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    run(args.steps)
    ev1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kernel_ms, n_rec = (gpu.profile_end() if events else ((None, None, None), 0))
    sec = (t1 - t0) / args.steps
    dev_ms = ev0.elapsed_time(ev1) / args.steps
    st = gpu.get_state()

    d, S, b = wl.d, wl.S, wl.grad_bytes
    grad_bytes = S * d * b
    # per parameter: 24 bytes (mean gradient or new momentum out and in, w and v in and out); without
    # weight decay the first sweep need not read w, which leaves 20
    total_bytes = grad_bytes + (24 if wl.weight_decay != 0.0 else 20) * d
    value = grad_bytes / sec / 1e9
    # first kernel of the three-kernel step: the general reduce kernel reads the gradients and writes
    # the mean gradient (4 bytes per parameter); the streaming one reads and writes v instead
    # (8 bytes per parameter) and reads w when there is weight decay (4 more)
    if path == "streaming":
        reduce_bytes = grad_bytes + (8 + (4 if wl.weight_decay != 0.0 else 0)) * d
    else:
        reduce_bytes = grad_bytes + 4 * d
    roof = None
    if fused:
        ach = total_bytes / (dev_ms * 1e-3) / 1e9
        traffic = TRAFFIC_BYTES.get(f"k_fused_cfg{args.config}")
        roof = {"bound": "hbm", "kernel": "k_fused (whole step in one launch)", "achieved": round(ach, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "bytes_per_launch": total_bytes, "avg_ms": round(dev_ms, 5),
                "timing": "HIP events on the launch stream around the K launches / K"}
    elif events and kernel_ms[0]:
        ach = reduce_bytes / (kernel_ms[0] * 1e-3) / 1e9
        kname = "k_reduce_stream" if path == "streaming" else "k_reduce"
        traffic = TRAFFIC_BYTES.get(f"{kname}_cfg{args.config}")
        roof = {"bound": "hbm", "kernel": kname, "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "bytes_per_launch": reduce_bytes, "avg_ms": round(kernel_ms[0], 5),
                "other_kernels_ms": {"k_scalars": round(kernel_ms[1], 5),
                                     ("k_apply" if path == "streaming" else "k_update"): round(kernel_ms[2], 5)},
                "update_GBps": round((12 if path == "streaming" else 20) * d / (kernel_ms[2] * 1e-3) / 1e9, 1)
                if kernel_ms[2] else None}

    cpu = None
    if not args.no_cpu_baseline:
        import harness as H
        orc = H.make_oracle(wl, openmp=True)
        w64, v64 = H.params_to_numpy64(inp)
        g_np = H.grads_to_numpy(inp)
        reps, c0 = 0, time.perf_counter()
        while reps < 1 or (time.perf_counter() - c0 < 10.0 and reps < 400):
            orc.step(w64, v64, g_np)
            reps += 1
        csec = (time.perf_counter() - c0) / reps
        cpu = {"value": round(grad_bytes / csec / 1e9, 3), "unit": "GB/s", "cores": orc.threads, "kind": "oracle",
               "sample": f"{reps} full step(s) of the same workload ({S * d / 1e6:.0f}M gradient elements each), "
                         f"OpenMP build of the oracle source, {csec:.3f} s/step"}
        if S * d <= 1 << 30:                          # the single-threaded build as well, one step
            one = H.make_oracle(wl, openmp=False)
            c0 = time.perf_counter()
            one.step(w64, v64, g_np)
            c1 = time.perf_counter() - c0
            cpu["single_thread"] = {"value": round(grad_bytes / c1 / 1e9, 3), "unit": "GB/s", "cores": 1,
                                    "sample": f"1 full step, {c1:.3f} s"}

    out = {
        "metric": "adascale_step gradient GB/s (S*d*b / step time), 1 GPU",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if b == 4 else "bf16->f32", "data": "synthetic",
        "config": {"workload": wl.name, "d": d, "n_tensors": wl.n_tensors, "S": S, "grad_dtype": "fp32" if b == 4 else "bf16",
                   "momentum": wl.momentum, "weight_decay": wl.weight_decay},
        "total_GBps": round(total_bytes / sec / 1e9, 1),
        "pct_hbm_peak": round(100 * total_bytes / sec / 1e9 / HBM_PEAK_GBPS, 2),
        "grad_elements_per_s": round(S * d / sec, 0),
        "algorithmic_bytes_per_step": total_bytes,
        "step_path": {"fused": "fused", "streaming": "three_kernel(streaming reduce)", "general": "three_kernel"}[path]
                     + ("+lagged_gain" if args.lagged else ""),
        "final_state": {"step": st.step, "r": st.r, "tau": st.tau},
        "roofline": roof, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    gpu.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
