"""Benchmark of the hierarchical recursive-doubling all-reduce on one MI355X.

One "step" = one whole all-reduce (reduce-scatter, log2 N exchange-and-sum steps,
all-gather) over all P virtual ranks.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak
COPY_PROBE_BYTES = 256 << 20  # the known-size copy that rocprof's byte counters are scaled by
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "fused_kernel_c4_traffic.json")


def algorithmic_bytes(P: int, G: int, N: int, msg_bytes: int) -> int:
    """Bytes the schedule itself must move: per rank 2M + (3L + 2) M/G (reads M + L*2M/G + M/G,
    writes M/G + L*M/G + M), every partial materialised because it crosses a network in the
    real method."""
    L = N.bit_length() - 1
    return P * (2 * msg_bytes + (3 * L + 2) * msg_bytes // G)


def device_bufs(x):
    import numpy as np
    import torch
    if x.dtype == np.uint16:
        return [torch.from_numpy(x[p].view(np.int16).copy()).view(torch.bfloat16).to("cuda:0") for p in range(x.shape[0])]
    return [torch.from_numpy(x[p].copy()).to("cuda:0") for p in range(x.shape[0])]


def time_calls(fn, warmup: int, steps: int):
    """(wall seconds, event milliseconds) for `steps` calls after `warmup` calls."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return time.perf_counter() - t0, e0.elapsed_time(e1)


def time_graph(ar, bufs, calls_per_graph: int, warmup: int, replays: int) -> float:
    """Mean microseconds per all-reduce with `calls_per_graph` calls captured in one HIP graph."""
    import torch
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        ar(bufs, stream)
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(calls_per_graph):
                ar(bufs, stream)
    torch.cuda.synchronize()
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1000.0 / (replays * calls_per_graph)


def copy_probe(times: int = 3) -> None:
    """Launch the library's plain copy kernel on COPY_PROBE_BYTES (so that a rocprofv3 --pmc run
    of this script sees a kernel whose HBM traffic is known: that many bytes read and written)."""
    import torch
    import paper_2511_09557_amd as rar
    src = torch.full((COPY_PROBE_BYTES,), 3, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(times):
        rar.rar_copy_probe(dst.data_ptr(), src.data_ptr(), COPY_PROBE_BYTES, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()


def measured_traffic(workload: str):
    """HBM bytes per fused launch from the committed rocprofv3 --pmc summary (None if absent or
    for another workload).  bench.py cannot collect hardware counters itself."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
        return t["bytes_per_launch"] if t.get("workload") == workload else None
    except (OSError, ValueError, KeyError):
        return None


def bench_workload(name: str, warmup: int, steps: int, extras: bool):
    import paper_2511_09557_amd as rar
    import rar_inputs as ri
    w = ri.WORKLOADS[name]
    x = ri.make_inputs(w)
    dtype = rar.RAR_BF16 if w.dtype == "bf16" else rar.RAR_F32
    out = {"P": w.P, "G": w.G, "N": w.N, "bytes_per_rank": w.bytes_per_rank,
           "algorithmic_bytes": algorithmic_bytes(w.P, w.G, w.N, w.bytes_per_rank)}
    bufs = device_bufs(x)
    ar = rar.AllReduce(w.P, w.G, w.n, dtype, rar.RAR_MODE_FUSED)
    wall, ev_ms = time_calls(lambda: ar(bufs), warmup, steps)
    assert ar.status() == 0
    out["fused_us"] = ev_ms * 1000.0 / steps
    out["fused_wall_us"] = wall * 1e6 / steps
    out["tuning"] = dict(zip(("B_s", "C_s"), ar.tuning()))
    if extras:
        ar.set_mode(rar.RAR_MODE_STEPWISE)
        _, ev = time_calls(lambda: ar(bufs), warmup // 4 + 1, max(steps // 4, 10))
        out["stepwise_us"] = ev * 1000.0 / max(steps // 4, 10)
        ar.set_mode(rar.RAR_MODE_FUSED)
        _, ev = time_calls(lambda: ar.launch_floor(), warmup, steps)
        out["launch_floor_us"] = ev * 1000.0 / steps
        _, ev = time_calls(lambda: ar.barrier_only(), warmup, steps)
        out["barrier_only_us"] = ev * 1000.0 / steps
        out["graph100_us"] = time_graph(ar, bufs, 100, 2, 10)
        assert ar.status() == 0
    ar.close()
    return out


def cpu_baseline(name: str):
    """The oracle as it stands, on the host cores of this machine, on one whole all-reduce of the
    workload (repeated until about 10 s have passed)."""
    import oracle
    import rar_inputs as ri
    w = ri.WORKLOADS[name]
    x = ri.make_inputs(w)
    want = min(16, os.cpu_count() or 1)
    cores = oracle.threads_used(want)
    oracle.allreduce(x, w.G, threads=cores)
    t0 = time.perf_counter()
    reps = 0
    while True:
        oracle.allreduce(x, w.G, threads=cores)
        reps += 1
        if time.perf_counter() - t0 > 10.0 or reps >= 50:
            break
    per = (time.perf_counter() - t0) / reps
    return {"value": per * 1e6, "unit": "us per all-reduce", "cores": cores, "kind": "oracle",
            "sample": f"{reps} whole all-reduces of workload {name} (P={w.P}, {w.bytes_per_rank} B per rank)"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4"])
    ap.add_argument("--no-extras", action="store_true", help="only the headline workload, fused mode")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build emulates all P ranks on ONE GPU; --gpus must be 1 "
              "(no multi-GPU path exists, see DESIGN.md 'More than one GPU')", file=sys.stderr)
        return 2

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    import rar_inputs as ri

    head = bench_workload(args.workload, args.warmup, args.steps, extras=not args.no_extras)
    copy_probe()
    w = ri.WORKLOADS[args.workload]
    us = head["fused_us"]
    achieved = head["algorithmic_bytes"] / (us * 1e-6) / 1e9
    line = {
        "metric": "us per all-reduce (fused schedule, bf16, P virtual ranks on one GPU); achieved HBM GB/s vs peak",
        "value": us,
        "unit": "us",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["fused_wall_us"] / 1000.0,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 storage, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: P={w.P} (G={w.G} x N={w.N}), {w.bytes_per_rank} B bf16 per rank, fused mode",
                   "tuning": head["tuning"]},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic(args.workload),
                     "kernel": "fused_kernel", "algorithmic_bytes_per_launch": head["algorithmic_bytes"],
                     "avg_launch_us": us},
    }
    if not args.no_extras:
        detail = {args.workload: head}
        for other in ("c1", "c2", "c3", "c4"):
            if other != args.workload:
                detail[other] = bench_workload(other, args.warmup, max(args.steps // 2, 10), extras=True)
        for k, v in detail.items():
            v["achieved_GBps"] = v["algorithmic_bytes"] / (v["fused_us"] * 1e-6) / 1e9
        line["detail"] = detail
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
