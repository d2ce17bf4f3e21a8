#!/usr/bin/env python3
"""Benchmark of the gossip-BMUF synchronisation step on one MI355X.

A step is one whole sync (neighbour sampling + fused gather-average-momentum kernel) over
all components of all K workers of a synthetic LSTM-LM-shaped parameter set that is already
resident in HBM.  Prints ONE JSON line: whole-job worker-params/s, the HBM roofline of the
fused kernel (algorithmic bytes = 24 B per worker-param, launch durations measured live
with events on the launch stream) and the CPU oracle timed on this machine's host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME|INDEX] [--all]
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
    """HBM bytes per fused-kernel launch from the committed rocprofv3 --pmc summary, if any."""
    path = os.path.join(ROOT, "profiles", f"sync_kernel_{workload}_pmc.md")
    try:
        m = re.search(r"^traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def run_gpu(w, steps: int, warmup: int, contiguous: bool = False):
    import numpy as np
    import torch

    from paper_1909_09010_amd import binding, workloads

    dev = "cuda:0"
    off = workloads.component_offsets(w)
    P = int(off[-1])
    m = len(off) - 1
    t0 = time.perf_counter()
    span = None if contiguous else workloads.default_span_bytes(dev, 3 * w.K * workloads.padded_stride(P) * 4)
    theta, omega, delta = workloads.init_state(w, dev, span_bytes=span)
    stride = theta.stride(0)
    plan = binding.Plan(off, w.K, w.q, w.p, seed=w.seed)
    torch.cuda.synchronize()
    log(f"[bench] {w.name}: K={w.K} q={w.q} p={plan.info.p} P={P} m={m} tiles={plan.info.n_tiles} "
        f"state={3 * w.K * theta.shape[1] * 4 / 1e9:.1f} GB, row stride {stride * 4 / 1e9:.2f} GB, "
        f"HBM span {(w.K - 1) * stride * 4 / 1e9 + 3 * theta.shape[1] * 4 / 1e9:.0f} GB, init {time.perf_counter() - t0:.1f}s")
    stream = torch.cuda.current_stream()

    H = workloads.periods(w)
    if H is not None:
        plan.set_periods(H)                     # Algorithm 1's per-component periods; a step is then one
        tick = int(H.min())                     # sync of the components that are due (counter += min H_i)

    rnd = 0
    for _ in range(warmup):
        if H is None:
            plan.sync(theta, omega, delta, stride, w.eta, w.zeta, w.mode, rnd, stream)
        else:
            plan.sync_step(theta, omega, delta, stride, w.eta, w.zeta, w.mode, (rnd + 1) * tick, stream)
        rnd += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    synced = 0
    for _ in range(steps):
        if H is None:
            plan.sync(theta, omega, delta, stride, w.eta, w.zeta, w.mode, rnd, stream)
            synced += P
        else:
            plan.sync_step(theta, omega, delta, stride, w.eta, w.zeta, w.mode, (rnd + 1) * tick, stream)
            active = ((rnd + 1) * tick) % H == 0
            synced += int((off[1:] - off[:-1])[active].sum())
        rnd += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # the dominant kernel alone: same kernel and launch shape through gbmuf_sync_table, with the
    # round's table drawn beforehand; one event pair per launch on the launch stream
    nbr = torch.zeros((m, w.K, max(w.q, 1)), dtype=torch.int32, device=dev)
    pairs = []
    for _ in range(steps):
        plan.neighbours_device(rnd, nbr, stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        plan.sync_table(nbr, theta, omega, delta, stride, w.eta, w.zeta, w.mode, stream)
        e1.record(stream)
        pairs.append((e0, e1))
        rnd += 1
    torch.cuda.synchronize()
    kernel_ms = float(np.mean([a.elapsed_time(b) for a, b in pairs]))
    finite = bool(torch.isfinite(theta[:, :P]).all())
    plan.destroy()
    del theta, omega, delta, nbr
    torch.cuda.empty_cache()
    return dict(P=P, m=m, K=w.K, stride=stride, synced_per_step=synced / max(steps, 1), padded=workloads.padded_stride(P), elapsed=elapsed,
                kernel_ms=kernel_ms, finite=finite, layout="contiguous" if span is None else "interleaved_rows")


def run_other_entry_points(w, launches: int = 5):
    """The two further kernels on the same workload: the gossip-MA branch (theta only: 8 B per
    worker-param) and the final model average (4(K+1) B per parameter)."""
    import numpy as np
    import torch

    from paper_1909_09010_amd import binding, workloads

    dev = "cuda:0"
    off = workloads.component_offsets(w)
    P = int(off[-1])
    span = workloads.default_span_bytes(dev, 3 * w.K * workloads.padded_stride(P) * 4)
    theta, _, _, stride = workloads.alloc_state(w.K, P, dev, span_bytes=span)
    theta.normal_(0, 0.02)
    out = torch.empty(P, device=dev)
    plan = binding.Plan(off, w.K, w.q, w.p, seed=w.seed)
    stream = torch.cuda.current_stream()

    def timed(fn):
        fn(0)
        pairs = []
        for r in range(1, launches + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn(r)
            e1.record(stream)
            pairs.append((e0, e1))
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in pairs]))

    ma = timed(lambda r: plan.sync(theta, None, None, stride, 0.0, 1.0, binding.MODE_GOSSIP_MA, r, stream))
    fa = timed(lambda r: plan.final_average(theta, stride, out, stream))
    plan.destroy()
    res = {"gossip_ma": {"ms": ma, "algorithmic_bytes": 8 * w.K * P, "GBps": 8 * w.K * P / ma / 1e6,
                         "frac": 8 * w.K * P / ma / 1e6 / HBM_PEAK_GBPS, "note": "whole sync: sampler + kernel"},
           "final_average": {"ms": fa, "algorithmic_bytes": 4 * (w.K + 1) * P, "GBps": 4 * (w.K + 1) * P / fa / 1e6,
                             "frac": 4 * (w.K + 1) * P / fa / 1e6 / HBM_PEAK_GBPS}}
    del theta, out
    torch.cuda.empty_cache()
    return res


def run_copy_probe(n_floats: int = 1 << 28, launches: int = 3):
    """gbmuf_probe_copy on two 1 GiB buffers: 4*n bytes read and 4*n bytes written per launch."""
    import numpy as np
    import torch

    from paper_1909_09010_amd import binding

    src = torch.randn(n_floats, device="cuda:0")
    dst = torch.empty_like(src)
    stream = torch.cuda.current_stream()
    binding.probe_copy(dst, src, n_floats, 0, stream)
    pairs = []
    for _ in range(launches):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        binding.probe_copy(dst, src, n_floats, 0, stream)
        e1.record(stream)
        pairs.append((e0, e1))
    torch.cuda.synchronize()
    ms = float(np.mean([a.elapsed_time(b) for a, b in pairs]))
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
    budget = 4_000_000                                  # sampled parameters per worker
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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="large_vocab",
                    help="name or index into the benchmark configurations (default: configs[2], large_vocab)")
    ap.add_argument("--all", action="store_true", help="also time configs[1], [3], [4] and the 4-layer K=64 variant")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch the library's plain copy probe (1 GiB read + 1 GiB written per launch): "
                         "the known-traffic kernel that rocprofv3 byte counters are scaled by")
    ap.add_argument("--contiguous", action="store_true",
                    help="three separate contiguous [K, P] tensors instead of the HBM-spanning row layout")
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
    gc = None
    if args.all and not args.contiguous:
        # the same workload with the rows side by side, measured first: physical placement depends on
        # what the process allocated before, and a fresh process is what a caller of this layout gets
        gc = run_gpu(w, min(args.steps, 5), args.warmup, contiguous=True)
    g = run_gpu(w, args.steps, args.warmup, args.contiguous)
    wp = g["K"] * g["P"]
    value = wp * args.steps / g["elapsed"]
    algo_bytes = BYTES_PER_WORKER_PARAM * wp
    achieved = algo_bytes / (g["kernel_ms"] * 1e-3) / 1e9
    out = {
        "metric": "gossip_bmuf_sync_worker_params_per_s",
        "value": value,
        "unit": "worker-params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": g["elapsed"] / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "K": w.K, "q": w.q, "params_per_worker": g["P"], "components": g["m"],
                   "eta": w.eta, "zeta": w.zeta, "mode": "nesterov" if w.mode == 1 else str(w.mode),
                   "state_GB": 3 * w.K * g["padded"] * 4 / 1e9, "layout": g["layout"],
                   "row_stride_GB": g["stride"] * 4 / 1e9},
        "effective_GBps": BYTES_PER_WORKER_PARAM * value / 1e9,
        "pct_of_hbm_peak": 100.0 * BYTES_PER_WORKER_PARAM * value / 1e9 / HBM_PEAK_GBPS,
        "finite": g["finite"],
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic(w.name),
                     "kernel": "sync_vec4_kernel", "kernel_ms": g["kernel_ms"], "algorithmic_bytes": algo_bytes},
    }
    if args.all:
        others = []
        for name in ("tiny", "medium", "large_vocab_chunked", "k64", "k64_4layer", "paper_shaped"):
            if name == w.name:
                continue
            ww = workloads.get(name)
            steps = min(args.steps, ww.rounds)
            gg = run_gpu(ww, steps, args.warmup, args.contiguous)
            v = gg["K"] * gg["synced_per_step"] * steps / gg["elapsed"]   # worker-params actually synced
            kb = BYTES_PER_WORKER_PARAM * gg["K"] * gg["P"] / (gg["kernel_ms"] * 1e-3) / 1e9
            others.append({"workload": name, "value": v, "ms_per_step": gg["elapsed"] / steps * 1e3,
                           "effective_GBps": BYTES_PER_WORKER_PARAM * v / 1e9, "kernel_GBps": kb,
                           "kernel_frac": kb / HBM_PEAK_GBPS})
        out["other_workloads"] = others
        out["other_entry_points"] = run_other_entry_points(w)
        if gc is not None:
            out["contiguous_layout"] = {"kernel_ms": gc["kernel_ms"],
                                        "kernel_frac": BYTES_PER_WORKER_PARAM * wp / (gc["kernel_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    if args.calibrate:
        out["copy_probe"] = run_copy_probe()
    if not args.no_cpu:
        out["cpu_baseline"] = run_cpu_baseline(w)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
