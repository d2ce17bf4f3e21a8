#!/usr/bin/env python3
"""Benchmark of the gossip-BMUF synchronisation step on one MI355X.

A step is one whole sync (neighbour sampling + fused gather-average-momentum kernel) over
all components of all K workers of a synthetic LSTM-LM-shaped parameter set that is already
resident in HBM.  Prints ONE JSON line: whole-job worker-params/s of the headline workload
(the largest benchmark configuration, K = 64), the HBM roofline of the fused kernel
(algorithmic bytes = 24 B per worker-param, launch durations measured live with events on the
launch stream around the very launches that are timed), the same figures for the other large
configurations, and the CPU oracle timed on this machine's host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME|INDEX] [--layout L]
                    [--only [--entry-points]] [--all] [--no-cpu] [--calibrate]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0            # MI355X HBM3E, published
BYTES_PER_WORKER_PARAM = 24       # read theta, omega, Delta + write theta', omega', Delta'


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(workload: str):
    """HBM bytes per fused-kernel launch from the committed rocprofv3 --pmc summary of this
    workload (a stored figure of an earlier profiled run, not of this run), and its file."""
    rel = os.path.join("profiles", f"sync_kernel_{workload}_pmc.md")
    try:
        m = re.search(r"^traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(os.path.join(ROOT, rel)).read(), re.M)
        return (float(m.group(1)), rel) if m else (None, None)
    except OSError:
        return None, None


def timed_launches(torch, stream, fn, n):
    """n launches of fn(i) with an event on the launch stream before the first, between
    consecutive ones and after the last; mean ms from one event to the next."""
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    marks[0].record(stream)
    for i in range(n):
        fn(i)
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    return sum(a.elapsed_time(b) for a, b in zip(marks[:-1], marks[1:])) / max(n, 1)


def run_gpu(w, steps: int, warmup: int, layout: str = "blocked", entry_points: bool = False):
    import torch

    from paper_1909_09010_amd import binding, workloads

    dev = "cuda:0"
    off = workloads.component_offsets(w)
    P = int(off[-1])
    m = len(off) - 1
    t0 = time.perf_counter()
    H = workloads.periods(w)
    plan = binding.Plan(off, w.K, w.q, w.p, seed=w.seed, periods=H)
    st = workloads.init_state(w, dev, layout=layout, plan=plan)
    torch.cuda.synchronize()
    log(f"[bench] {w.name}: K={w.K} q={w.q} p={plan.info.p} P={P} m={m} layout={layout} "
        f"state={3 * w.K * P * 4 / 1e9:.1f} GB in {st.bytes / 1e9:.1f} GB of HBM, init {time.perf_counter() - t0:.1f}s")
    stream = torch.cuda.current_stream()
    tick = int(H.min()) if H is not None else 1   # with periods a step is one sync of the components that are due

    def sync(rnd):
        if st.layout == "separate":
            t, o, d = st.arrays
            if H is None:
                plan.sync(t, o, d, st.worker_stride, w.eta, w.zeta, w.mode, rnd, stream)
            else:
                plan.sync_step(t, o, d, st.worker_stride, w.eta, w.zeta, w.mode, (rnd + 1) * tick, stream)
        elif H is None:
            plan.sync_state(st.desc(), w.eta, w.zeta, w.mode, rnd, stream)
        else:
            plan.sync_step_state(st.desc(), w.eta, w.zeta, w.mode, (rnd + 1) * tick, stream)

    for r in range(warmup):
        sync(r)
    torch.cuda.synchronize()
    # the timed region: `steps` whole syncs back to back, with an event on the launch stream at
    # every boundary between syncs, which gives the launch durations of the very same syncs
    t0 = time.perf_counter()
    launch_ms = timed_launches(torch, stream, lambda i: sync(warmup + i), steps)
    elapsed = time.perf_counter() - t0
    synced = 0
    for i in range(steps):
        if H is None:
            synced += P
        else:
            synced += int((off[1:] - off[:-1])[((warmup + i + 1) * tick) % H == 0].sum())
    finite = all(bool(torch.isfinite(st.get_row(0, k)).all()) for k in (0, w.K - 1))
    res = dict(P=P, m=m, K=w.K, synced_per_step=synced / max(steps, 1), elapsed=elapsed, launch_ms=launch_ms,
               finite=finite, layout=layout, hbm_bytes=st.bytes, steps=steps,
               tile_columns=plan.info.tile_columns_blocked if layout == "blocked" else plan.info.tile_columns)
    if entry_points:
        # the two further kernels on the same state: the gossip-MA branch (theta only: 8 B per
        # worker-param, sampler included) and the final model average (4(K+1) B per parameter)
        out = torch.empty(P, device=dev)
        ma_desc = st.desc(gossip_ma=True)
        rows = st.layout == "separate"

        def ma(i):
            if rows:
                plan.sync(st.arrays[0], None, None, st.worker_stride, 0.0, 1.0, binding.MODE_GOSSIP_MA, i, stream)
            else:
                plan.sync_state(ma_desc, 0.0, 1.0, binding.MODE_GOSSIP_MA, i, stream)

        def fa(i):
            if rows:
                plan.final_average(st.arrays[0], st.worker_stride, out, stream)
            else:
                plan.final_average_state(ma_desc, out, stream)

        ma(0), fa(0)
        ma_ms = timed_launches(torch, stream, ma, 5)
        fa_ms = timed_launches(torch, stream, fa, 5)
        res["entry_points"] = {
            "gossip_ma": {"ms": ma_ms, "algorithmic_bytes": 8 * w.K * P, "GBps": 8 * w.K * P / ma_ms / 1e6,
                          "frac": 8 * w.K * P / ma_ms / 1e6 / HBM_PEAK_GBPS, "note": "whole sync: sampler + kernel"},
            "final_average": {"ms": fa_ms, "algorithmic_bytes": 4 * (w.K + 1) * P, "GBps": 4 * (w.K + 1) * P / fa_ms / 1e6,
                              "frac": 4 * (w.K + 1) * P / fa_ms / 1e6 / HBM_PEAK_GBPS}}
        del out
    plan.destroy()
    del st
    torch.cuda.empty_cache()
    return res


def run_copy_probe(n_floats: int = 1 << 28, launches: int = 3):
    """gbmuf_probe_copy on two 1 GiB buffers: 4*n bytes read and 4*n bytes written per launch."""
    import torch

    from paper_1909_09010_amd import binding

    src = torch.randn(n_floats, device="cuda:0")
    dst = torch.empty_like(src)
    stream = torch.cuda.current_stream()
    binding.probe_copy(dst, src, n_floats, 0, stream)
    ms = timed_launches(torch, stream, lambda i: binding.probe_copy(dst, src, n_floats, 0, stream), launches)
    assert torch.equal(src, dst)
    return {"bytes_read": 4 * n_floats, "bytes_written": 4 * n_floats, "ms": ms, "GBps": 8 * n_floats / ms / 1e6}


def run_cpu_baseline(w, target_seconds: float = 15.0):
    """The oracle as it stands, on this machine's host cores, on a bounded sample of the workload:
    the leading stripe of every component (same K, q, m, neighbour tables and scalars)."""
    import numpy as np

    import oracle
    from paper_1909_09010_amd import workloads

    off = workloads.component_offsets(w)
    P = int(off[-1])
    budget = 16_000_000 // w.K * 4                      # sampled parameters per worker (64 M worker-params)
    frac = min(1.0, budget / P)
    sizes = np.maximum(1, np.floor((off[1:] - off[:-1]) * frac)).astype(np.int64)
    sizes = np.minimum(sizes, off[1:] - off[:-1])
    red = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    Ps = int(red[-1])
    rng = np.random.default_rng(w.seed)
    w0 = (rng.normal(0, w.w0_scale, Ps) if w.w0_dist == "normal" else rng.uniform(-w.w0_scale, w.w0_scale, Ps))
    theta = (w0 + rng.normal(0, w.drift_std, (w.K, Ps))).astype(np.float32)
    omega = np.tile(w0.astype(np.float32), (w.K, 1))
    delta = (rng.normal(0, w.delta_std, (w.K, Ps)) if w.delta_std > 0 else np.zeros((w.K, Ps))).astype(np.float32)
    p = oracle.default_p(w.K) if w.p == 0 else w.p
    eta, zeta = np.float32(w.eta), np.float32(w.zeta)
    t0 = time.perf_counter()
    oracle.sync(red, w.K, p, w.q, w.seed, 0, theta, omega, delta, eta, zeta, w.mode)
    one = time.perf_counter() - t0
    rounds = int(max(1, min(200, round(target_seconds / max(one, 1e-3)))))
    t0 = time.perf_counter()
    for r in range(1, rounds + 1):
        oracle.sync(red, w.K, p, w.q, w.seed, r, theta, omega, delta, eta, zeta, w.mode)
    dt = time.perf_counter() - t0
    return {"value": w.K * Ps * rounds / dt, "unit": "worker-params/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"leading {frac:.4f} of each of the {len(sizes)} components of {w.name} "
                      f"({Ps} params/worker, K={w.K}), {rounds} rounds in {dt:.1f}s, fp32 C oracle with OpenMP"}


def summary(w, g):
    """One workload's figures: whole-sync throughput and the launch-duration roofline."""
    wp_synced = g["K"] * g["synced_per_step"]
    v = wp_synced * g["steps"] / g["elapsed"]
    # the launch covers the tiles of the components that were due: its algorithmic bytes
    gbps = BYTES_PER_WORKER_PARAM * wp_synced / (g["launch_ms"] * 1e-3) / 1e9
    return {"workload": w.name, "K": w.K, "q": w.q, "params_per_worker": g["P"], "components": g["m"],
            "layout": g["layout"], "state_GB": 3 * w.K * g["P"] * 4 / 1e9, "arena_GB": g["hbm_bytes"] / 1e9,
            "value": v, "ms_per_step": g["elapsed"] / g["steps"] * 1e3, "kernel_ms": g["launch_ms"],
            "kernel_GBps": gbps, "kernel_frac": gbps / HBM_PEAK_GBPS, "steps": g["steps"]}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="k64",
                    help="name or index into the benchmark configurations (default: configs[4], k64, the largest)")
    ap.add_argument("--layout", default="blocked", choices=["blocked", "rows", "separate"],
                    help="state placement: the library's blocked arena (default), its rows arena, or three separate tensors")
    ap.add_argument("--only", action="store_true", help="time the headline workload only (what the profiles run)")
    ap.add_argument("--entry-points", action="store_true",
                    help="with --only: still time the gossip-MA branch and the final average on the headline state")
    ap.add_argument("--all", action="store_true", help="also time configs[0], [1] and the paper-shaped (16,128) schedule")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch the library's plain copy probe (1 GiB read + 1 GiB written per launch): "
                         "the known-traffic kernel that rocprofv3 byte counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (K workers are replicas in one GPU's HBM); "
              "--gpus N with N > 1 is not supported.", file=sys.stderr)
        return 2

    import torch

    from paper_1909_09010_amd import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        return 3

    w = workloads.get(args.workload)
    g = run_gpu(w, args.steps, args.warmup, args.layout, entry_points=args.entry_points or not args.only)
    head = summary(w, g)
    assert head["kernel_ms"] <= head["ms_per_step"] * 1.001, "event-timed launches cannot exceed the wall clock around them"
    algo_bytes = BYTES_PER_WORKER_PARAM * w.K * g["P"]
    traffic, traffic_src = measured_traffic(w.name) if args.layout == "blocked" else (None, None)
    out = {
        "metric": "gossip_bmuf_sync_worker_params_per_s",
        "value": head["value"],
        "unit": "worker-params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "K": w.K, "q": w.q, "params_per_worker": g["P"], "components": g["m"],
                   "eta": w.eta, "zeta": w.zeta, "mode": "nesterov" if w.mode == 1 else str(w.mode),
                   "state_GB": head["state_GB"], "arena_GB": head["arena_GB"], "layout": g["layout"],
                   "tile_columns": g["tile_columns"]},
        "effective_GBps": BYTES_PER_WORKER_PARAM * head["value"] / 1e9,
        "pct_of_hbm_peak": 100.0 * BYTES_PER_WORKER_PARAM * head["value"] / 1e9 / HBM_PEAK_GBPS,
        "finite": g["finite"],
        "roofline": {"bound": "hbm", "achieved": head["kernel_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": head["kernel_frac"], "traffic": traffic, "traffic_source": traffic_src,
                     "kernel": "sync_vec4_kernel", "kernel_ms": head["kernel_ms"], "algorithmic_bytes": algo_bytes,
                     "timing": "mean over the timed syncs, from events on the launch stream at the boundaries "
                               "between them (the few-microsecond sampler launch of a sync is inside)"},
    }
    if "entry_points" in g:
        out["other_entry_points"] = g["entry_points"]
    if not args.only:
        names = ["large_vocab", "large_vocab_chunked", "k64", "k64_4layer"]
        if args.all:
            names += ["tiny", "medium", "paper_shaped"]
        others = []
        for name in names:
            if name == w.name:
                continue
            ww = workloads.get(name)
            others.append(summary(ww, run_gpu(ww, min(args.steps, ww.rounds, 10), args.warmup, args.layout)))
        out["other_workloads"] = others
        if args.layout == "blocked":
            # what a caller with three plain [K, P] tensors gets (rows: 3K address streams; the
            # figure then depends on where the driver happened to place the tensors)
            sep = summary(w, run_gpu(w, min(args.steps, 5), args.warmup, "separate"))
            out["separate_tensors_layout"] = {k: sep[k] for k in ("kernel_ms", "kernel_GBps", "kernel_frac", "arena_GB")}
    if args.calibrate:
        out["copy_probe"] = run_copy_probe()
    if not args.no_cpu:
        out["cpu_baseline"] = run_cpu_baseline(w)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
