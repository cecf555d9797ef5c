"""Benchmark of the AdaScale step on one MI355X.

`python bench.py --gpus 1 --steps K --warmup W` times K whole adascale_step calls (mean gradient
and norms, scalars, update: one fused kernel or three) on synthetic gradients already resident in
HBM and prints ONE JSON line.  The workload is the configuration the headline metric is quoted
on: d = 25,557,032 parameters in 161 tensors (bottleneck-CNN-like shapes), S = 16 fp32 gradient
buffers.

Cold parameters.  In training a step follows a backward pass that has swept the 256 MB
memory-side cache, so no step finds w and v cached.  A loop that steps on the same w and v again
and again does: at d = 25.6 M they are 204 MB.  The timed loop therefore rotates between several
sets of (w, v) buffers (together with the gradient buffers where those are small enough to be
cached as well) so that what a step reads was last touched several cache sizes ago.  The
figure of the plain loop is reported beside it (`frac_warm`).

value        = gradient bytes streamed per second (S*d*b / step time), GB/s, cold loop
roofline     = the dominant kernel against the 8 TB/s HBM peak:
               achieved / frac   algorithmic bytes of one launch / its average duration in the
                                 cold loop, from HIP events on the launch stream;
               frac_warm         the same in the plain loop (w, v served by the memory-side cache);
               moved_bytes       bytes the kernel really reads and writes (the library counts them
                                 from its tile tables: the mean gradient that stays on chip is
                                 never written or read back), frac_moved = moved / time / peak:
                                 how close the kernel runs to the memory system, where `frac`
                                 says how close the step is to a design that moves the
                                 algorithmic bytes at peak;
               traffic           the same from rocprofv3 FETCH_SIZE / WRITE_SIZE counters, read
                                 out of the summary under profiles/ named in traffic_source.
               The kernel is the fused step (whole step, S*d*b + 24*d bytes, 20*d without weight
               decay) when the library runs the step as one persistent launch, else the first
               kernel of the three-kernel step (the gradient sweep).
graph_replay = the same cold loop captured once into a HIP graph and replayed (launch gaps shrink;
               reported beside the headline, which stays the directly launched loop)
other_configs = the other benchmark configurations, timed the same way (cold), without a CPU leg
cpu_baseline = the CPU oracle (OpenMP build of the same source) on the host, steps of the same
               workload for about ten seconds
"""
from __future__ import annotations

import argparse
import ctypes as C
import gc
import json
import math
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBPS = 8000.0
CACHE_BYTES = 256 << 20          # memory-side cache of the MI355X
MAX_SETS = 8                     # pointer tables the library keeps on the device
# rocprofv3 summaries holding the measured HBM traffic of the dominant kernel per launch
# (a line `traffic_bytes_per_launch[<key>] = N`), by workload number and step path
PROFILE_OF = {
    ("fused", 2): "k_fused_cfg3_resnet50like_S16.md",
    ("fused", 3): "k_fused_cfg3_resnet50like_S16.md",
    ("fused", 4): "k_fused_cfg3_resnet50like_S16.md",
    ("fused", 5): "k_fused_cfg3_resnet50like_S16.md",
    ("streaming", 3): "three_kernel_step_cfg3_resnet50like_S16.md",
    ("streaming", 5): "three_kernel_streaming_cfg5_transformer350M_S64_bf16.md",
}


def profiled_traffic(path: str, cfg: int):
    """(bytes per launch, source file) from the committed profile summary, or (None, None)."""
    name = PROFILE_OF.get((path, cfg))
    if not name:
        return None, None
    try:
        text = open(os.path.join(ROOT, "profiles", name)).read()
    except OSError:
        return None, None
    m = re.search(r"traffic_bytes_per_launch\[cfg%d\]\s*=\s*([0-9,]+)" % cfg, text)
    return (int(m.group(1).replace(",", "")), "profiles/" + name) if m else (None, None)


class Loop:
    """One workload resident on the GPU, with `n_sets` rotating sets of parameter (and, for small
    workloads, gradient) buffers, and the library context stepping on them."""

    def __init__(self, cfg: int, lagged: bool, cold: bool, force_path: str = "none"):
        import torch
        import workloads as W
        from paper_2007_05105_amd import AdaScale, Tuning
        self.torch = torch
        wl = self.wl = W.config(cfg)
        self.cfg = cfg
        inp = self.inp = W.Inputs(wl, "cuda:0")
        inp.fill_grads(0)
        wv_bytes = 8 * wl.d
        g_bytes = wl.S * wl.d * wl.grad_bytes
        self.rotate_grads = cold and g_bytes < (1 << 30)     # small enough to be cached in part
        set_bytes = wv_bytes + (g_bytes if self.rotate_grads else 0)
        if not cold or wv_bytes >= 4 * CACHE_BYTES:           # cold by itself: a step sweeps the cache many times
            self.n_sets = 1
        else:
            self.n_sets = min(MAX_SETS, max(3, math.ceil(3 * CACHE_BYTES / set_bytes)))
        self.cold = cold and (self.n_sets * set_bytes >= 3 * CACHE_BYTES or self.n_sets == 1)
        arr = lambda ts: (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
        self.keep = []
        self.sets = []
        for j in range(self.n_sets):
            if j == 0:
                w, v, g = inp.w, inp.v, inp.g
            else:
                wf, vf = inp.w_flat.clone(), inp.v_flat.clone()
                w, v = W.views(wf, wl.numel, inp.offs32), W.views(vf, wl.numel, inp.offs32)
                g = inp.g
                if self.rotate_grads:
                    other = W.Inputs(wl, "cuda:0")
                    other.fill_grads(j)
                    g = other.g
                    self.keep.append(other)
                self.keep += [wf, vf]
            self.sets.append((arr(w), arr(v), arr([t for gi in g for t in gi])))
        self.gpu = AdaScale(wl.numel, wl.S, wl.lr_table, wl.momentum, wl.weight_decay, wl.theta, wl.eps,
                            wl.grad_dtype, 0, flags=1 if lagged else 0,
                            tuning=None if force_path == "none" else
                            Tuning(force_path={"general": 1, "fused": 2, "streaming": 3}[force_path]))
        self.stream = torch.cuda.current_stream()
        self.sh = int(self.stream.cuda_stream)
        self.t = 0

    def run(self, n: int, sets=None, stream_handle=None) -> None:
        k = self.n_sets if sets is None else sets
        sh = self.sh if stream_handle is None else stream_handle
        for _ in range(n):
            pw, pv, pg = self.sets[self.t % k]
            self.t += 1
            rc = self.gpu.step_raw(pw, pv, pg, sh)
            if rc != 0:
                raise RuntimeError(self.gpu.last_error())

    def graph_ms(self, n: int, rounds: int = 5):
        """The same cold loop launched as a HIP graph: `rounds` rotations through the sets of
        buffers captured once (every set has been stepped on before, so its pointer table is on
        the device), replayed until at least n steps have run.  (ms per step, steps per graph)."""
        torch = self.torch
        per_graph = rounds * self.n_sets
        self.t = 0
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            self.run(per_graph, stream_handle=int(torch.cuda.current_stream().cuda_stream))
        replays = max(1, -(-n // per_graph))
        graph.replay()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(self.stream)
        for _ in range(replays):
            graph.replay()
        ev1.record(self.stream)
        torch.cuda.synchronize()
        del graph
        return ev0.elapsed_time(ev1) / (replays * per_graph), per_graph

    def timed(self, n: int, sets=None, kernel_events: bool = False):
        """(host seconds per step, device ms per step, per-kernel ms or None) over n steps."""
        torch = self.torch
        if kernel_events:
            self.gpu.profile_begin(n)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record(self.stream)
        self.run(n, sets)
        ev1.record(self.stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        kms = self.gpu.profile_end()[0] if kernel_events else None
        return (t1 - t0) / n, ev0.elapsed_time(ev1) / n, kms

    def median_ms(self, n: int) -> float:
        """Median over n steps of the time between events recorded before each step (a pass of its
        own: the main timed region has no events between its launches)."""
        torch = self.torch
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        torch.cuda.synchronize()
        for i in range(n):
            ev[i].record(self.stream)
            self.run(1)
        ev[n].record(self.stream)
        torch.cuda.synchronize()
        return statistics.median(ev[i].elapsed_time(ev[i + 1]) for i in range(n))

    def close(self) -> None:
        self.gpu.close()
        self.sets = self.keep = self.inp = None
        gc.collect()
        self.torch.cuda.empty_cache()


def measure(cfg: int, steps: int, warmup: int, lagged: bool, kernel_events: bool, warm_too: bool, median_steps: int,
            force_path: str = "none", with_graph: bool = False):
    """Time one workload; returns (record for the JSON line, the Loop, still open)."""
    lp = Loop(cfg, lagged, cold=True, force_path=force_path)
    wl, gpu = lp.wl, lp.gpu
    lp.run(warmup)
    lp.torch.cuda.synchronize()
    path = gpu.step_path()
    fused = path == "fused"
    # Per-kernel HIP events (recorded by the library on the launch stream) for the three-kernel
    # step.  The fused step is a single kernel per step: one pair of events on the launch stream
    # around the K launches gives its average duration without an event between every two launches.
    events = kernel_events and not fused
    sec, dev_ms, kms = lp.timed(steps, kernel_events=events)
    warm = None
    if warm_too and lp.n_sets > 1:
        lp.run(max(3, warmup // 2), sets=1)
        _, warm_dev_ms, warm_kms = lp.timed(steps, sets=1, kernel_events=events)
        warm = (warm_dev_ms, warm_kms)
    med = lp.median_ms(median_steps) if median_steps > 0 else None
    graph = lp.graph_ms(max(steps, 100)) if with_graph else None

    d, S, b = wl.d, wl.S, wl.grad_bytes
    grad_bytes = S * d * b
    total_bytes = gpu.step_bytes()                    # S*d*b + 24*d, 20*d without weight decay
    moved_step = gpu.step_moved_bytes()
    per_param_sweep = 8 + (4 if wl.weight_decay != 0.0 else 0)
    if fused:
        kname, k_bytes, k_moved, k_ms = "k_fused (whole step in one launch)", total_bytes, moved_step, dev_ms
        k_ms_warm = warm[0] if warm else None
        timing = "HIP events on the launch stream around the K launches / K"
    else:
        # first kernel of the three-kernel step: the streaming one reads the gradients, reads and
        # writes v and reads w under weight decay; the general one writes the mean gradient instead
        kname = "k_reduce_stream" if path == "streaming" else "k_reduce"
        k_bytes = grad_bytes + (per_param_sweep if path == "streaming" else 4) * d
        k_moved = moved_step - 12 * d if path == "streaming" else k_bytes      # the rest is k_apply's
        k_ms = kms[0] if kms else None
        k_ms_warm = warm[1][0] if warm and warm[1] else None
        timing = "HIP events on the launch stream before and after every launch, averaged"
    roof = None
    if k_ms:
        ach = k_bytes / (k_ms * 1e-3) / 1e9
        traffic, source = (None, None) if lagged else profiled_traffic(path, cfg)
        roof = {"bound": "hbm", "kernel": kname, "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBPS, 4),
                "frac_warm": round(k_bytes / (k_ms_warm * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4) if k_ms_warm else None,
                "traffic": traffic, "traffic_source": source,
                "bytes_per_launch": k_bytes, "moved_bytes": k_moved,
                "frac_moved": round(k_moved / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "avg_ms": round(k_ms, 5), "avg_ms_warm": round(k_ms_warm, 5) if k_ms_warm else None,
                "timing": timing,
                "cold": f"{lp.n_sets} rotating set(s) of w, v" + (" and gradients" if lp.rotate_grads else "")
                        + ("" if lp.cold else " (still cache resident: not an HBM measurement)")}
        if not fused and kms:
            roof["other_kernels_ms"] = {"k_scalars": round(kms[1], 5),
                                        ("k_apply" if path == "streaming" else "k_update"): round(kms[2], 5)}
            if kms[2]:
                roof["update_GBps"] = round((12 if path == "streaming" else 20) * d / (kms[2] * 1e-3) / 1e9, 1)
    rec = {
        "workload": wl.name, "d": d, "n_tensors": wl.n_tensors, "S": S, "grad_dtype": "fp32" if b == 4 else "bf16",
        "ms_per_step": round(sec * 1e3, 5), "device_ms_per_step": round(dev_ms, 5),
        "median_ms_per_step": round(med, 5) if med else None,
        "graph_replay": {"ms_per_step": round(graph[0], 5), "steps_per_graph": graph[1],
                         "pct_hbm_peak": round(100 * total_bytes / (graph[0] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
                         "note": "the same cold loop captured once into a HIP graph and replayed"} if graph else None,
        "grad_GBps": round(grad_bytes / sec / 1e9, 1),
        "algorithmic_bytes": total_bytes, "pct_hbm_peak": round(100 * total_bytes / sec / 1e9 / HBM_PEAK_GBPS, 2),
        "moved_bytes": moved_step, "pct_hbm_peak_moved": round(100 * moved_step / sec / 1e9 / HBM_PEAK_GBPS, 2),
        "step_path": {"fused": "fused", "streaming": "three_kernel(streaming reduce)", "general": "three_kernel"}[path]
                     + ("+lagged_gain" if lagged else ""),
        "cold_parameters": lp.cold, "rotating_sets": lp.n_sets, "roofline": roof,
    }
    return rec, lp


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (3 = the headline configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true", help="do not time the other configurations afterwards")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the cold loop")
    ap.add_argument("--no-warm-loop", action="store_true", help="skip the plain loop on one set of w, v (frac_warm)")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not record per-kernel events inside the timed region")
    ap.add_argument("--lagged", action="store_true",
                    help="time the prior-iteration-gain variant (App. B.3), a single sweep of S*d*b + 16*d bytes")
    ap.add_argument("--force-path", choices=["none", "fused", "streaming", "general"], default="none",
                    help="take this implementation of the step where the library would choose another (measurements)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 1 GiB a few times (the known-size kernel that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch

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

    rec, lp = measure(args.config, args.steps, args.warmup, args.lagged, not args.no_kernel_events,
                      not args.no_warm_loop, median_steps=max(50, min(args.steps, 200)), force_path=args.force_path,
                      with_graph=not args.no_graph)
    wl, inp = lp.wl, lp.inp
    st = lp.gpu.get_state()
    d, S, b = wl.d, wl.S, wl.grad_bytes
    grad_bytes = S * d * b

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
        del w64, v64, g_np
    lp.close()

    others = []
    if not args.headline_only:
        for cfg in (1, 2, 4, 5):
            if cfg == args.config:
                continue
            o, olp = measure(cfg, 30 if cfg == 5 else 100, 5 if cfg == 5 else 10, args.lagged, not args.no_kernel_events,
                             False, median_steps=0, force_path=args.force_path, with_graph=not args.no_graph)
            olp.close()
            r = o.pop("roofline")
            if r:
                o["dominant_kernel"] = {k: r[k] for k in ("kernel", "frac", "frac_moved", "avg_ms", "traffic",
                                                          "traffic_source", "cold")}
            others.append(o)

    out = {
        "metric": "adascale_step gradient GB/s (S*d*b / step time), 1 GPU",
        "value": rec["grad_GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rec["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if b == 4 else "bf16->f32", "data": "synthetic",
        "config": {"workload": wl.name, "d": d, "n_tensors": wl.n_tensors, "S": S, "grad_dtype": rec["grad_dtype"],
                   "momentum": wl.momentum, "weight_decay": wl.weight_decay,
                   "cold_parameters": rec["cold_parameters"], "rotating_sets_of_w_v": rec["rotating_sets"]},
        "median_ms_per_step": rec["median_ms_per_step"], "graph_replay": rec["graph_replay"],
        "total_GBps": round(rec["algorithmic_bytes"] / (rec["ms_per_step"] * 1e-3) / 1e9, 1),
        "pct_hbm_peak": rec["pct_hbm_peak"],
        "pct_hbm_peak_moved": rec["pct_hbm_peak_moved"],
        "grad_elements_per_s": round(S * d / (rec["ms_per_step"] * 1e-3), 0),
        "algorithmic_bytes_per_step": rec["algorithmic_bytes"], "moved_bytes_per_step": rec["moved_bytes"],
        "step_path": rec["step_path"],
        "final_state": {"step": st.step, "r": st.r, "tau": st.tau},
        "roofline": rec["roofline"], "cpu_baseline": cpu, "other_configs": others,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
