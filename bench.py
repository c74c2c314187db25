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
SWEEP_SEED = 20251109 * 1000 + 400
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "fused_kernel_{workload}_traffic.json")


def algorithmic_bytes(P: int, G: int, N: int, msg_bytes: int) -> int:
    """Bytes the schedule itself must move: per rank 2M + (3L + 2) M/G (reads M + L*2M/G + M/G,
    writes M/G + L*M/G + M), every partial materialised because it crosses a network in the
    real method."""
    L = N.bit_length() - 1
    return P * (2 * msg_bytes + (3 * L + 2) * msg_bytes // G)


def moved_bytes(P: int, G: int, N: int, msg_bytes: int) -> int:
    """Bytes the fused kernel has to move for one all-reduce (N a power of two): per rank it reads
    the G local messages' chunk (M) and one peer partial per step (L * M/G), and writes its own
    partial for every step but the last (L * M/G: S_0 .. S_{L-1}) and the gathered result (M):
    2M + 2L * M/G.  A rank's own partial stays in registers from step to step and the last
    partial is never written out, which is what separates this from the schedule's count above."""
    L = N.bit_length() - 1
    return P * (2 * msg_bytes + 2 * L * msg_bytes // G)


MIN_CALLS_SHORT = 300   # kernels of a few microseconds are timed over at least this many calls


def device_bufs(x):
    """x[P, n] on the host -> P rank buffers on the device, as the rows of ONE allocation.
    (The library takes any P pointers; rows of a single allocation measured 10-15 % faster than
    P separately allocated tensors, whose physical placement is up to the allocator.)"""
    import numpy as np
    import torch
    if x.dtype == np.uint16:
        whole = torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).to("cuda:0")
    else:
        whole = torch.from_numpy(x.copy()).to("cuda:0")
    return [whole[p] for p in range(x.shape[0])]


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


def time_graph(enqueue, calls_per_graph: int, warmup: int, replays: int) -> float:
    """Mean microseconds per call with `calls_per_graph` calls of enqueue(stream) captured in one
    HIP graph (the paper's micro-benchmark protocol, Section 5: 100 all-reduces per graph)."""
    import torch
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        enqueue(stream)                      # eager call first: one-time set-up stays out of the graph
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(calls_per_graph):
                enqueue(stream)
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


def time_graph_two_chains(enqueue_a, enqueue_b, calls_per_chain: int, warmup: int, replays: int) -> float:
    """Mean microseconds per call when two independent chains of calls (two plans, two sets of
    buffers) run side by side on two streams inside one HIP graph: a call of one chain may start
    while a call of the other is still finishing."""
    import torch
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(main):
        enqueue_a(main)
        enqueue_b(main)
        main.synchronize()
        with torch.cuda.graph(graph, stream=main):
            side.wait_stream(main)
            for _ in range(calls_per_chain):
                enqueue_a(main)
                enqueue_b(side)
            main.wait_stream(side)
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
    return e0.elapsed_time(e1) * 1000.0 / (replays * 2 * calls_per_chain)


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


def streaming_ceilings():
    """What plain streaming kernels reach on this device, beyond the 256 MiB memory-side cache: a
    read-only pass over 1 GiB and a copy of 512 MiB (bytes counted = read + written)."""
    import torch
    import paper_2511_09557_amd as rar
    st = torch.cuda.current_stream().cuda_stream
    big = torch.full((1 << 30,), 5, dtype=torch.uint8, device="cuda:0")
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    half = 512 << 20
    _, ev = time_calls(lambda: rar.rar_read_probe(sink.data_ptr(), big.data_ptr(), 1 << 30, st), 3, 20)
    read = (1 << 30) / (ev / 20 * 1e-3) / 1e9
    _, ev = time_calls(lambda: rar.rar_copy_probe(big.data_ptr() + half, big.data_ptr(), half, st), 3, 20)
    copy = 2 * half / (ev / 20 * 1e-3) / 1e9
    del big
    torch.cuda.empty_cache()
    return {"read_only_GBps": read, "copy_GBps": copy,
            "note": "library probes rar_read_probe (1 GiB) and rar_copy_probe (512 MiB -> 512 MiB), 16-byte vectors, 20 calls each"}


def cold_leg(ar, stream_calls: int = 20, replays: int = 5):
    """The bound all-reduce with the memory-side cache swept before every call: HIP graphs of
    `stream_calls` x (256 MiB copy, all-reduce) against graphs of the copies alone; the difference
    is the all-reduce on cold caches.  Returns microseconds per call."""
    import torch
    import paper_2511_09557_amd as rar
    src = torch.full((COPY_PROBE_BYTES,), 3, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)

    def sweep_caches(st):
        rar.rar_copy_probe(dst.data_ptr(), src.data_ptr(), COPY_PROBE_BYTES, st.cuda_stream)

    def both(st):
        sweep_caches(st)
        ar.launch(st)
    alone = min(time_graph(sweep_caches, stream_calls, 1, replays) for _ in range(2))
    pair = min(time_graph(both, stream_calls, 1, replays) for _ in range(2))
    # the all-reduce alone between two events, launched eagerly right behind the copy (its launch
    # is queued while the copy runs): the kernel's own duration plus the gap before it
    cur = torch.cuda.current_stream()
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(40)]
    for e0, e1 in pairs:
        sweep_caches(cur)
        e0.record()
        ar.launch(cur.cuda_stream)
        e1.record()
    torch.cuda.synchronize()
    bracketed = sorted(e0.elapsed_time(e1) * 1000.0 for e0, e1 in pairs[5:])
    bracketed_us = bracketed[len(bracketed) // 2]
    del dst
    # the same with a sweep that only reads (512 MiB): the caches then hold clean lines of other
    # data, where the copy above leaves 256 MiB of modified lines that have to be written back
    # while the all-reduce runs
    big = torch.full((2 * COPY_PROBE_BYTES,), 7, dtype=torch.uint8, device="cuda:0")
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda:0")

    def sweep_reading(st):
        rar.rar_read_probe(sink.data_ptr(), big.data_ptr(), 2 * COPY_PROBE_BYTES, st.cuda_stream)

    def both_reading(st):
        sweep_reading(st)
        ar.launch(st)
    alone_r = min(time_graph(sweep_reading, stream_calls, 1, replays) for _ in range(2))
    pair_r = min(time_graph(both_reading, stream_calls, 1, replays) for _ in range(2))
    del src, big
    return pair - alone, alone, pair_r - alone_r, bracketed_us


def bench_chain(ar, K: int = 100, launches: int = 10):
    """Microseconds per all-reduce when K of them run in ONE persistent launch (rar_allreduce_chain)."""
    import torch
    cur = torch.cuda.current_stream().cuda_stream
    ar.launch_chain(2, cur)
    _, ev = time_calls(lambda: ar.launch_chain(K, cur), 2, launches)
    return ev * 1000.0 / (launches * K)


def bench_step_combine(warmup: int, steps: int):
    """rar_step_combine (one rank's exchange-and-sum, 3 * n * 2 bytes of traffic) on c4's per-step
    message (512 KiB, launch-bound) and on 128 MiB (bandwidth-bound; beyond the memory-side cache)."""
    import torch
    import paper_2511_09557_amd as rar
    out = {}
    st = torch.cuda.current_stream().cuda_stream
    for label, n in (("512KiB", 262144), ("128MiB", 64 << 20)):
        dst = torch.zeros(n, dtype=torch.bfloat16, device="cuda:0")
        src = torch.ones(n, dtype=torch.bfloat16, device="cuda:0")
        k = max(steps // 10, 10) if n > (1 << 22) else steps
        _, ev = time_calls(lambda: rar.rar_step_combine(dst.data_ptr(), src.data_ptr(), 0, n, rar.RAR_BF16, st), min(warmup, 20), k)
        us = ev * 1000.0 / k
        out[label] = {"elements": n, "us": us, "GBps": 3 * n * 2 / (us * 1e-6) / 1e9}
        del dst, src
    return out


def measured_traffic(workload: str):
    """HBM bytes per fused launch from the committed rocprofv3 --pmc summary (None if absent or
    for another workload).  bench.py cannot collect hardware counters itself."""
    try:
        with open(TRAFFIC_FILE.format(workload=workload)) as f:
            t = json.load(f)
        return t["bytes_per_launch"] if t.get("workload") == workload else None
    except (OSError, ValueError, KeyError):
        return None


def prepare_workload(name: str, mode: str = "fused"):
    """Inputs in device memory and a plan with its scratch, bound: (rank buffers, AllReduce)."""
    import paper_2511_09557_amd as rar
    import rar_inputs as ri
    w = ri.WORKLOADS[name]
    bufs = device_bufs(ri.make_inputs(w))
    ar = rar.AllReduce(w.P, w.G, w.n, rar.RAR_BF16 if w.dtype == "bf16" else rar.RAR_F32, rar.RAR_MODE_FUSED)
    if mode != "fused":     # only with --no-extras: the headline call in another mode (for per-kernel profiles)
        ar.set_mode({"stepwise": rar.RAR_MODE_STEPWISE, "packed": rar.RAR_MODE_FUSED_PACKED, "auto": rar.RAR_MODE_AUTO}[mode])
    ar.bind(bufs)
    return bufs, ar


def bench_workload(name: str, warmup: int, steps: int, extras: bool, mode: str = "fused", headline: bool = True, prepared=None):
    """One workload.  The headline workload's fused call is timed over exactly `steps` calls after
    `warmup` (the figure of the JSON line); every other figure uses its own number of calls, at
    least MIN_CALLS_SHORT for kernels of a few microseconds, so that no figure is a 10-call sample.
    `prepared`: what prepare_workload returned earlier for this workload (else it is called now)."""
    import torch
    import paper_2511_09557_amd as rar
    import rar_inputs as ri
    w = ri.WORKLOADS[name]
    out = {"P": w.P, "G": w.G, "N": w.N, "bytes_per_rank": w.bytes_per_rank,
           "algorithmic_bytes": algorithmic_bytes(w.P, w.G, w.N, w.bytes_per_rank),
           "moved_bytes": moved_bytes(w.P, w.G, w.N, w.bytes_per_rank)}
    bufs, ar = prepared if prepared is not None else prepare_workload(name, mode)
    cur = torch.cuda.current_stream().cuda_stream   # looked up once: the timed calls pass the handle
    short = w.bytes_per_rank <= (1 << 20)           # c1-c3: a few microseconds per call
    calls = steps if headline else max(steps, MIN_CALLS_SHORT if short else 100)
    warm = warmup if headline else max(warmup, 50)
    sub_calls = max(steps, MIN_CALLS_SHORT) if short else max(min(steps, 500), 100)   # for the side measurements
    wall, ev_ms = time_calls(lambda: ar.launch(cur), warm, calls)
    assert ar.status() == 0
    out["fused_us"] = ev_ms * 1000.0 / calls
    out["fused_wall_us"] = wall * 1e6 / calls
    out["fused_calls_timed"] = calls
    if extras:  # two more repetitions of the same timed region, to show the spread
        reps = [out["fused_us"]] + [time_calls(lambda: ar.launch(cur), 10, calls)[1] * 1000.0 / calls for _ in range(2)]
        out["fused_us_repetitions"] = reps
    out["tuning"] = dict(zip(("B_s", "C_s"), ar.tuning()))
    if extras:
        out["side_calls_timed"] = sub_calls
        ar.set_mode(rar.RAR_MODE_STEPWISE)
        k = max(sub_calls // 3, 100)
        _, ev = time_calls(lambda: ar.launch(cur), 20, k)
        out["stepwise_us"] = ev * 1000.0 / k
        ar.set_mode(rar.RAR_MODE_FUSED)
        _, ev = time_calls(lambda: ar.launch_floor(cur), 50, sub_calls)
        out["launch_floor_us"] = ev * 1000.0 / sub_calls
        _, ev = time_calls(lambda: ar.barrier_only(cur), 50, sub_calls)
        out["barrier_only_us"] = ev * 1000.0 / sub_calls
        # the same three things inside HIP graphs of 100 calls: the device-side cost without
        # the host's launch rate.  floor = launch only; barrier = flags only; fused = everything
        out["graph100_us"] = time_graph(lambda st: ar.launch(st), 100, 2, 10)
        out["graph100_launch_floor_us"] = time_graph(lambda st: ar.launch_floor(st), 100, 2, 10)
        out["graph100_barrier_only_us"] = time_graph(lambda st: ar.barrier_only(st), 100, 2, 10)
        ar.set_mode(rar.RAR_MODE_STEPWISE)
        out["graph100_stepwise_us"] = time_graph(lambda st: ar.launch(st), 100, 2, 10)
        ar.set_mode(rar.RAR_MODE_FUSED)
        # 100 all-reduces in ONE persistent launch (rar_allreduce_chain): a workgroup starts call
        # k+1 as soon as its own slices of call k are gathered; per-call time
        out["chain100_us"] = bench_chain(ar)
        # the memory-side cache swept before every call (256 MiB copy in between, copy time subtracted)
        cold, sweep_us, cold_clean, cold_events = cold_leg(ar)
        out["cold_us"] = cold
        out["cold_between_events_us"] = cold_events
        out["cold_sweep_copy_us"] = sweep_us
        out["cold_after_read_sweep_us"] = cold_clean
        # back-to-back calls versus calls with compute in between (the paper's Appendix B runs a
        # synthetic matmul between all-reduces).  The compute here is what precedes the all-reduce
        # in a tensor-parallel layer: every rank's row-parallel product, tokens x hidden/P @
        # hidden/P x hidden in bf16, written straight into that rank's message (one batched product
        # for all P emulated ranks; its weights, hidden x hidden in total, sweep the caches).  The
        # all-reduce's share is the difference to the products alone.
        hidden = 8192 if w.bytes_per_rank <= (256 << 10) else 16384
        tokens = max(w.n // hidden, 1)
        whole = bufs[0]._base.view(w.P, tokens, hidden)
        a_sh = torch.randn(w.P, tokens, hidden // w.P, device="cuda:0", dtype=torch.bfloat16)
        w_sh = torch.randn(w.P, hidden // w.P, hidden, device="cuda:0", dtype=torch.bfloat16) / hidden ** 0.5
        torch.bmm(a_sh, w_sh, out=whole)
        mm = time_graph(lambda st: torch.bmm(a_sh, w_sh, out=whole), 100, 2, 10)

        def mm_then_ar(st):
            torch.bmm(a_sh, w_sh, out=whole)
            ar.launch(st)
        ar.set_mode(rar.RAR_MODE_AUTO)      # as a caller who sets nothing would run it
        both = time_graph(mm_then_ar, 100, 2, 10)
        # the all-reduce alone between two events, launched eagerly right behind the product (its
        # launch is queued while the product runs): the kernel's own duration plus the gap before it
        brackets = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(40)]
        for e0, e1 in brackets:
            torch.bmm(a_sh, w_sh, out=whole)
            e0.record()
            ar.launch(cur)
            e1.record()
        torch.cuda.synchronize()
        between = sorted(e0.elapsed_time(e1) * 1000.0 for e0, e1 in brackets[5:])
        ar.set_mode(rar.RAR_MODE_FUSED)
        out["graph100_matmul_us"] = mm
        out["graph100_interleaved_allreduce_us"] = both - mm
        out["interleaved_between_events_us"] = between[len(between) // 2]
        del a_sh, w_sh, whole
        # the data+flag ("packed") exchange of Section 4.2.2, where the planner offers it
        try:
            ar.set_mode(rar.RAR_MODE_FUSED_PACKED)
        except rar.RarError:
            out["packed_us"] = out["graph100_packed_us"] = out["chain100_packed_us"] = None
        else:
            _, ev = time_calls(lambda: ar.launch(cur), 50, sub_calls)
            out["packed_us"] = ev * 1000.0 / sub_calls
            out["graph100_packed_us"] = time_graph(lambda st: ar.launch(st), 100, 2, 10)
            out["chain100_packed_us"] = bench_chain(ar)
            out["packed_tuning"] = dict(zip(("B_s", "C_s"), ar.tuning()))
            ar.set_mode(rar.RAR_MODE_FUSED)
        # two independent chains of calls side by side (two plans, two sets of buffers, two streams
        # in one graph): what per-step buffers and sequence numbers buy in the paper, a call that
        # starts before the previous one has finished everywhere, shows here as overlap of kernels
        bufs_b, ar_b = prepare_workload(name)
        ar_b.set_mode(rar.RAR_MODE_AUTO)
        ar.set_mode(rar.RAR_MODE_AUTO)
        rar.rar_plan_set_concurrency(ar.plan, 2)       # each chain sizes its grid for half the device
        rar.rar_plan_set_concurrency(ar_b.plan, 2)
        out["graph100_two_chains_us"] = time_graph_two_chains(lambda st: ar.launch(st), lambda st: ar_b.launch(st), 50, 2, 10)
        assert ar.status() == 0 and ar_b.status() == 0
        ar_b.close()
        del bufs_b
        rar.rar_plan_set_concurrency(ar.plan, 1)
        # what a caller who sets nothing gets (the library's automatic choice between the two),
        # timed on its own, eagerly and in graphs
        packed = ar.effective_mode() == rar.RAR_MODE_FUSED_PACKED
        out["auto_mode"] = "fused_packed" if packed else "fused"
        _, ev = time_calls(lambda: ar.launch(cur), 50, sub_calls)
        out["auto_us"] = ev * 1000.0 / sub_calls
        out["graph100_auto_us"] = time_graph(lambda st: ar.launch(st), 100, 2, 10)
        out["chain100_auto_us"] = bench_chain(ar)
        ar.set_mode(rar.RAR_MODE_FUSED)
        assert ar.status() == 0
    ar.close()
    return out


def sweep(path: str) -> None:
    """Message-size sweep (8 KiB .. 64 MiB per rank, P in {8,16,32,64,128} with G=4, plus
    64 = 8x8; bf16 and fp32; N(0,1) values drawn on the device from a seeded generator).
    Writes one JSON object per point to `path` and prints a table."""
    import torch
    import paper_2511_09557_amd as rar
    gen = torch.Generator(device="cuda:0")
    rows = []
    with open(path, "w") as f:
        for dtype, code, es, tdt in (("bf16", rar.RAR_BF16, 2, torch.bfloat16), ("f32", rar.RAR_F32, 4, torch.float32)):
            for P, G in ((8, 4), (16, 4), (32, 4), (64, 4), (128, 4), (64, 8)):
                for lg in range(13, 27):
                    nbytes = 1 << lg
                    n = nbytes // es
                    gen.manual_seed(SWEEP_SEED + lg * 1000 + P * 10 + G)
                    whole = torch.empty(P, n, device="cuda:0", dtype=tdt)
                    for p in range(P):      # row by row: the fp32 draw of a whole 8 GiB point would not be needed at once
                        whole[p] = torch.randn(n, device="cuda:0", generator=gen, dtype=torch.float32).to(tdt)
                    bufs = [whole[p] for p in range(P)]
                    ar = rar.AllReduce(P, G, n, code, rar.RAR_MODE_FUSED)
                    ar.bind(bufs)
                    alg = algorithmic_bytes(P, G, P // G, nbytes)
                    mov = moved_bytes(P, G, P // G, nbytes)
                    reps = max(5, min(500, int(2e-2 / max(alg / 5e12, 5e-6))))
                    _, ev = time_calls(lambda: ar.launch(), max(reps // 5, 2), reps)
                    fused = ev * 1000.0 / reps
                    graph = time_graph(lambda st: ar.launch(st), 20, 1, max(reps // 20, 2)) if nbytes <= (4 << 20) else None
                    packed_graph = None
                    if nbytes <= (1 << 20):
                        try:
                            ar.set_mode(rar.RAR_MODE_FUSED_PACKED)
                            packed_graph = time_graph(lambda st: ar.launch(st), 20, 1, max(reps // 20, 2))
                        except rar.RarError:
                            pass
                    ar.set_mode(rar.RAR_MODE_AUTO)
                    auto = "packed" if ar.effective_mode() == rar.RAR_MODE_FUSED_PACKED else "fused"
                    ar.set_mode(rar.RAR_MODE_STEPWISE)
                    _, ev = time_calls(lambda: ar.launch(), max(reps // 5, 2), reps)
                    stepwise = ev * 1000.0 / reps
                    assert ar.status() == 0
                    B_s, C_s = ar.tuning()
                    ar.close()
                    row = {"dtype": dtype, "P": P, "G": G, "bytes_per_rank": nbytes, "fused_us": fused,
                           "fused_in_graph_us": graph, "packed_in_graph_us": packed_graph, "auto_mode": auto,
                           "stepwise_us": stepwise, "algorithmic_bytes": alg, "moved_bytes": mov,
                           "fused_GBps": mov / (fused * 1e-6) / 1e9, "schedule_GBps": alg / (fused * 1e-6) / 1e9,
                           "B_s": B_s, "C_s": C_s}
                    f.write(json.dumps(row) + "\n")
                    f.flush()
                    rows.append(row)
                    print(f"{dtype:4s} P={P:3d} G={G} {nbytes:9d} B  fused {fused:10.2f} us ({row['fused_GBps']:7.0f} GB/s)"
                          f"  graph {graph if graph is None else round(graph, 2)}  stepwise {stepwise:10.2f} us  B_s={B_s} C_s={C_s}",
                          file=sys.stderr, flush=True)
                    del bufs, whole
                    torch.cuda.empty_cache()
    md = os.path.splitext(path)[0] + ".md"
    with open(md, "w") as f:
        f.write("# Message-size sweep of the all-reduce on one MI355X\n\n"
                "command: `python3 bench.py --sweep <file>.jsonl`; eager launches timed with HIP events; values N(0,1)\n"
                "drawn on the device; GB/s = bytes the fused kernel must move, `P*(2M + 2L*M/G)`, / time, and its fraction of\n"
                "the 8 TB/s HBM peak (small messages live in the caches: the fraction then says nothing about HBM);\n"
                "`schedule GB/s` = the schedule's own count with every partial materialised, `P*(2M + (3L+2)M/G)`, / time;\n"
                "`graph` = the call inside a HIP graph of 20 calls (fused: messages up to 4 MiB; data+flag mode: up to 1 MiB),\n"
                "which takes the host's launch rate out; `auto` = the mode a plan runs in when none is set.\n")
        key = None
        for r in rows:
            if (r["dtype"], r["P"], r["G"]) != key:
                key = (r["dtype"], r["P"], r["G"])
                f.write(f"\n## {r['dtype']}, P={r['P']} (G={r['G']}, N={r['P'] // r['G']})\n\n"
                        "| bytes per rank | fused us | GB/s | frac of 8 TB/s | schedule GB/s | fused in graph us | data+flag in graph us | auto | stepwise us | B_s | C_s |\n"
                        "|---|---|---|---|---|---|---|---|---|---|---|\n")
            g = "-" if r["fused_in_graph_us"] is None else f"{r['fused_in_graph_us']:.2f}"
            pg = "-" if r["packed_in_graph_us"] is None else f"{r['packed_in_graph_us']:.2f}"
            f.write(f"| {r['bytes_per_rank']} | {r['fused_us']:.2f} | {r['fused_GBps']:.0f} | {r['fused_GBps'] / HBM_PEAK_GBPS:.3f} "
                    f"| {r['schedule_GBps']:.0f} | {g} | {pg} | {r['auto_mode']} | {r['stepwise_us']:.2f} | {r['B_s']} | {r['C_s']} |\n")


def sensitivity(path: str) -> None:
    """B_s x C_s sensitivity (the paper's Appendix "Impact of Chunk Size and Block Size", Table 5:
    a 1024 KB message on 16 GPUs), also for the four workloads, as microseconds per all-reduce
    inside HIP graphs of 100 calls, plus what rar_autotune picks.  Writes a markdown report."""
    import torch
    import paper_2511_09557_amd as rar
    cases = [("table5-shape: 1024 KiB, P=16 (G=4, N=4)", 16, 4, 524288)]
    import rar_inputs as ri
    for name in ("c1", "c2", "c3", "c4"):
        w = ri.WORKLOADS[name]
        cases.append((f"{name}: {w.bytes_per_rank >> 10} KiB, P={w.P} (G={w.G}, N={w.N})", w.P, w.G, w.n))
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(SWEEP_SEED + 77)
    lines = ["# B_s / C_s sensitivity of the fused all-reduce on one MI355X (bf16)", "",
             "command: `python3 bench.py --sensitivity <this file>`; microseconds per all-reduce, mean over",
             "10 replays of a HIP graph holding 100 calls; `-` = B_s beyond what the message or the device's",
             "residency allows (the launch clamps it, so the column to the left already shows that case).", ""]
    for title, P, G, n in cases:
        whole = torch.randn(P, n, device="cuda:0", generator=gen).to(torch.bfloat16)
        bufs = [whole[p] for p in range(P)]
        ar = rar.AllReduce(P, G, n, rar.RAR_BF16, rar.RAR_MODE_FUSED)
        ar.bind(bufs)
        lines += [f"## {title}", "", "| C_s \\ B_s | " + " | ".join(str(b) for b in (1, 2, 4, 8, 16, 32, 64)) + " |",
                  "|---|" + "---|" * 7]
        for C_s in (4096, 8192, 16384, 32768):
            row, seen = [], set()
            for B_s in (1, 2, 4, 8, 16, 32, 64):
                ar.set_tuning(B_s, C_s)
                eff = ar.tuning()[0]
                if eff in seen:
                    row.append("-")
                    continue
                seen.add(eff)
                row.append(f"{time_graph(lambda st: ar.launch(st), 100, 1, 10):.2f}")
            lines.append(f"| {C_s} | " + " | ".join(row) + " |")
        ar.set_tuning(0, 0)
        default = ar.tuning()
        d_us = time_graph(lambda st: ar.launch(st), 100, 1, 10)
        best = ar.autotune(bufs, calls=50)
        tuned = ar.tuning()
        t_us = time_graph(lambda st: ar.launch(st), 100, 1, 10)
        lines += ["", f"built-in choice (B_s, C_s) = {default}: {d_us:.2f} us; rar_autotune picks {tuned}: {t_us:.2f} us "
                  f"(its own eager measurement: {best:.2f} us)", ""]
        assert ar.status() == 0
        ar.close()
        print(title, "done", file=sys.stderr, flush=True)
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")


def hierarchy(path: str) -> None:
    """Flat versus hierarchical: the same P ranks and message split as G x N in every way that
    keeps N a power of two.  G = 1 is plain recursive doubling over all ranks (log2 P steps on the
    whole message), G = P is a single node (no inter-node step); the paper's model (Section 4.3)
    has log2 N inter-node steps on |M|/G bytes each.  Writes a markdown report."""
    import torch
    import paper_2511_09557_amd as rar
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(SWEEP_SEED + 99)
    lines = ["# Flat versus hierarchical split of the same ranks, one MI355X (bf16)", "",
             "command: `python3 bench.py --hierarchy <this file>`; fused mode, microseconds per all-reduce inside",
             "HIP graphs of 100 calls; L = log2 N inter-node steps; schedule bytes = P*(2M + (3L+2)M/G) (every partial",
             "materialised, as it would cross a network); the fused kernel moves P*(2M + 2L*M/G).", ""]
    for P, nbytes in ((16, 256 << 10), (16, 2 << 20), (64, 256 << 10), (64, 2 << 20)):
        n = nbytes // 2
        whole = torch.randn(P, n, device="cuda:0", generator=gen).to(torch.bfloat16)
        bufs = [whole[p] for p in range(P)]
        lines += [f"## P = {P}, {nbytes >> 10} KiB per rank", "",
                  "| G | N | L | bytes per step and rank | schedule MB | moved MB | us per all-reduce | moved GB/s |", "|---|---|---|---|---|---|---|---|"]
        G = 1
        while G <= P:
            N = P // G
            ar = rar.AllReduce(P, G, n, rar.RAR_BF16, rar.RAR_MODE_FUSED)
            ar.bind(bufs)
            us = time_graph(lambda st: ar.launch(st), 100, 2, 10)
            assert ar.status() == 0
            ar.close()
            alg = algorithmic_bytes(P, G, N, nbytes)
            mov = moved_bytes(P, G, N, nbytes)
            lines.append(f"| {G} | {N} | {N.bit_length() - 1} | {nbytes // G} | {alg / 1e6:.1f} | {mov / 1e6:.1f} | {us:.2f} | {mov / us / 1e3:.0f} |")
            G *= 2
        lines.append("")
        print(f"P={P} {nbytes} B done", file=sys.stderr, flush=True)
    # node counts that are not powers of two (outside the paper): N = 2^L + r costs the L steps
    # plus a hand-over before and after them on the first 2r nodes
    lines += ["## G = 4, any N (N that is not a power of two is an extension outside the paper)", "",
              "| N | P | L | folded pairs r | us per all-reduce, 256 KiB | us per all-reduce, 2048 KiB |", "|---|---|---|---|---|---|"]
    for N in range(2, 17):
        P, row = 4 * N, []
        for nbytes in (256 << 10, 2 << 20):
            n = nbytes // 2
            whole = torch.randn(P, n, device="cuda:0", generator=gen).to(torch.bfloat16)
            bufs = [whole[p] for p in range(P)]
            ar = rar.AllReduce(P, 4, n, rar.RAR_BF16, rar.RAR_MODE_FUSED)
            ar.bind(bufs)
            row.append(time_graph(lambda st: ar.launch(st), 100, 2, 10))
            assert ar.status() == 0
            ar.close()
            del bufs, whole
        L = N.bit_length() - 1
        lines.append(f"| {N} | {P} | {L} | {N - (1 << L)} | {row[0]:.2f} | {row[1]:.2f} |")
    lines.append("")
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")


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
    t1 = time.perf_counter()
    single_reps = 0
    while single_reps < 3 and (single_reps == 0 or time.perf_counter() - t1 < 5.0):
        oracle.allreduce(x, w.G, threads=1)
        single_reps += 1
    single = (time.perf_counter() - t1) / single_reps
    return {"value": per * 1e6, "unit": "us per all-reduce", "cores": cores, "kind": "oracle",
            "sample": f"{reps} whole all-reduces of workload {name} (P={w.P}, {w.bytes_per_rank} B per rank)",
            "single_thread": {"value": single * 1e6, "unit": "us per all-reduce", "cores": 1,
                              "sample": f"{single_reps} whole all-reduces of the same workload"}}


def tuning_scan(path: str) -> None:
    """Every (B_s, C_s) the planner can launch against its built-in choice, over P = 8..128,
    G = 1..8, 16 KiB .. 16 MiB, bf16 and fp32, inside HIP graphs of 20 calls.  Writes a markdown
    summary (the built-in choice's distance from the best pair of each shape)."""
    import torch
    import paper_2511_09557_amd as rar
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(SWEEP_SEED + 5)
    rows = []
    for dt, code, es, tdt in (("bf16", rar.RAR_BF16, 2, torch.bfloat16), ("f32", rar.RAR_F32, 4, torch.float32)):
        for P, G in ((8, 4), (16, 4), (32, 4), (64, 4), (128, 4), (64, 8), (16, 8), (8, 1), (32, 2)):
            for lg in range(14, 25):
                nbytes = 1 << lg
                n = nbytes // es
                whole = torch.randn(P, n, device="cuda:0", generator=gen).to(tdt)
                ar = rar.AllReduce(P, G, n, code, rar.RAR_MODE_FUSED)
                ar.bind([whole[p] for p in range(P)])
                ar.launch()
                torch.cuda.synchronize()
                default = ar.tuning()
                reps = 10 if nbytes <= (1 << 22) else 3
                res = {}
                for C_s in (4096, 8192, 16384, 32768):
                    for div in (1, 2):
                        ar.set_tuning(0, C_s)
                        B = max(1, ar.tuning()[0] // div)      # the widest grid the planner allows, and half of it
                        ar.set_tuning(B, C_s)
                        t = ar.tuning()
                        if t in res:
                            continue
                        res[t] = time_graph(lambda st: ar.launch(st), 20, 1, reps)
                        assert ar.status() == 0, (t, P, G, nbytes, dt)
                ar.set_tuning(0, 0)
                d = res.get(default) or time_graph(lambda st: ar.launch(st), 20, 1, reps)
                best = min(res, key=res.get)
                rows.append((dt, P, G, nbytes, default, d, best, res[best]))
                print(f"{dt} P={P} G={G} {nbytes} default {default} {d:.2f} best {best} {res[best]:.2f}", file=sys.stderr, flush=True)
                ar.close()
                del whole
    ratios = [r[5] / r[7] for r in rows]
    geo = 1.0
    for r in ratios:
        geo *= r ** (1.0 / len(ratios))
    worst = max(rows, key=lambda r: r[5] / r[7])
    with open(path, "w") as f:
        f.write("# Built-in (B_s, C_s) against the best of the scanned pairs, one MI355X\n\n"
                "command: `python3 bench.py --tuning-scan <this file>`; fused mode (flag exchange), microseconds per all-reduce\n"
                "inside HIP graphs of 20 calls; candidates: C_s in {4, 8, 16, 32} KiB x B_s in {widest grid the planner\n"
                "allows (four workgroups per compute unit at most), half of it}.\n\n"
                f"shapes: {len(rows)}; built-in / best: mean {sum(ratios) / len(ratios):.3f}, geometric mean {geo:.3f}, "
                f"worst {worst[5] / worst[7]:.3f} ({worst[0]} P={worst[1]} G={worst[2]} {worst[3]} B)\n\n"
                "| type | P | G | bytes per rank | built-in (B_s, C_s) | us | best (B_s, C_s) | us | ratio |\n|---|---|---|---|---|---|---|---|---|\n")
        for dt, P, G, nbytes, default, d, best, b in rows:
            f.write(f"| {dt} | {P} | {G} | {nbytes} | {default} | {d:.2f} | {best} | {b:.2f} | {d / b:.3f} |\n")


def cold_loop(workload: str, calls: int) -> None:
    """For a profiler: `calls` x (256 MiB copy, fused all-reduce of the workload) launched eagerly, so
    that a kernel trace shows the all-reduce kernel's own duration on cold caches."""
    import torch
    import paper_2511_09557_amd as rar
    import rar_inputs as ri
    w = ri.WORKLOADS[workload]
    bufs = device_bufs(ri.make_inputs(w))
    ar = rar.AllReduce(w.P, w.G, w.n, rar.RAR_BF16, rar.RAR_MODE_FUSED)
    ar.bind(bufs)
    src = torch.full((COPY_PROBE_BYTES,), 3, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    st = torch.cuda.current_stream().cuda_stream
    for _ in range(calls):
        rar.rar_copy_probe(dst.data_ptr(), src.data_ptr(), COPY_PROBE_BYTES, st)
        ar.launch(st)
    assert ar.status() == 0
    ar.close()


def interleaved_loop(workload: str, calls: int) -> None:
    """For a profiler: `calls` x (every rank's row-parallel product written into its message,
    all-reduce of the workload in automatic mode) launched eagerly, so that a kernel trace shows
    the all-reduce kernel's own duration behind the compute that produces its input."""
    import torch
    import paper_2511_09557_amd as rar
    import rar_inputs as ri
    w = ri.WORKLOADS[workload]
    bufs = device_bufs(ri.make_inputs(w))
    ar = rar.AllReduce(w.P, w.G, w.n, rar.RAR_BF16, rar.RAR_MODE_AUTO)
    ar.bind(bufs)
    hidden = 8192 if w.bytes_per_rank <= (256 << 10) else 16384
    tokens = max(w.n // hidden, 1)
    whole = bufs[0]._base.view(w.P, tokens, hidden)
    a_sh = torch.randn(w.P, tokens, hidden // w.P, device="cuda:0", dtype=torch.bfloat16)
    w_sh = torch.randn(w.P, hidden // w.P, hidden, device="cuda:0", dtype=torch.bfloat16) / hidden ** 0.5
    st = torch.cuda.current_stream().cuda_stream
    for _ in range(calls):
        torch.bmm(a_sh, w_sh, out=whole)
        ar.launch(st)
    assert ar.status() == 0
    ar.close()


def chain_loop(workload: str, launches: int, K: int = 100) -> None:
    """For a profiler: `launches` chained launches of K all-reduces each (rar_allreduce_chain), fused mode."""
    import torch
    import paper_2511_09557_amd as rar
    import rar_inputs as ri
    w = ri.WORKLOADS[workload]
    bufs = device_bufs(ri.make_inputs(w))
    ar = rar.AllReduce(w.P, w.G, w.n, rar.RAR_BF16, rar.RAR_MODE_AUTO)
    ar.bind(bufs)
    st = torch.cuda.current_stream().cuda_stream
    for _ in range(launches):
        ar.launch_chain(K, st)
    assert ar.status() == 0
    ar.close()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4"])
    ap.add_argument("--no-extras", action="store_true", help="only the headline workload, fused mode")
    ap.add_argument("--mode", default="fused", choices=["fused", "stepwise", "packed", "auto"],
                    help="with --no-extras: run the headline workload in this mode (the JSON line says which)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--cold-loop", type=int, metavar="CALLS", help="for a profiler: only CALLS x (cache sweep, fused all-reduce of --workload)")
    ap.add_argument("--interleaved-loop", type=int, metavar="CALLS", help="for a profiler: only CALLS x (row-parallel products, all-reduce of --workload in automatic mode)")
    ap.add_argument("--chain-loop", type=int, metavar="LAUNCHES", help="for a profiler: only LAUNCHES chains of 100 all-reduces of --workload (automatic mode)")
    ap.add_argument("--sensitivity", metavar="OUT.md", help="run the B_s x C_s sensitivity study instead and write it to this file")
    ap.add_argument("--hierarchy", metavar="OUT.md", help="run the flat-versus-hierarchical study instead and write it to this file")
    ap.add_argument("--sweep", metavar="OUT.jsonl", help="run the message-size sweep instead and write it to this file")
    ap.add_argument("--tuning-scan", metavar="OUT.md", help="run the scan of all (B_s, C_s) against the built-in choice instead")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build emulates all P ranks on ONE GPU; --gpus must be 1 "
              "(there is no multi-GPU path: collectives between GPUs are not part of this build)", file=sys.stderr)
        return 2

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    import rar_inputs as ri

    if args.sweep:
        sweep(args.sweep)
        return 0
    if args.sensitivity:
        sensitivity(args.sensitivity)
        return 0
    if args.hierarchy:
        hierarchy(args.hierarchy)
        return 0
    if args.tuning_scan:
        tuning_scan(args.tuning_scan)
        return 0
    if args.cold_loop:
        cold_loop(args.workload, args.cold_loop)
        copy_probe()
        return 0
    if args.interleaved_loop:
        interleaved_loop(args.workload, args.interleaved_loop)
        return 0
    if args.chain_loop:
        chain_loop(args.workload, args.chain_loop)
        return 0

    if args.mode != "fused" and not args.no_extras:
        print("bench.py: --mode needs --no-extras", file=sys.stderr)
        return 2
    # The other workloads first: by the time the headline's W warm-up and K timed steps run, the
    # device has been busy for a while and sits at its running clocks, whatever K and W are.
    # The headline's buffers and scratch are allocated before anything else, as in a process that
    # runs the headline alone: where they land in physical memory moves its time by a few per cent,
    # and blocks that other workloads have used and freed land elsewhere.
    prepared = prepare_workload(args.workload, args.mode)
    others = {}
    if not args.no_extras:
        for other in ("c1", "c2", "c3", "c4"):
            if other != args.workload:
                others[other] = bench_workload(other, args.warmup, args.steps, extras=True, headline=False)
    head = bench_workload(args.workload, args.warmup, args.steps, extras=not args.no_extras, mode=args.mode, prepared=prepared)
    copy_probe()
    w = ri.WORKLOADS[args.workload]
    us = head["fused_us"]
    # The roofline figure: bytes the kernel has to move (moved_bytes) over its launch duration.
    # The schedule's own count (every partial materialised: algorithmic_bytes) is reported beside it
    # as a rate without a fraction: the fused kernel does not move those bytes.
    moved = head["moved_bytes"] if args.mode in ("fused", "auto") else head["algorithmic_bytes"]
    achieved = moved / (us * 1e-6) / 1e9
    traffic = measured_traffic(args.workload) if args.mode == "fused" else None
    roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                "kernel": "fused_kernel" if args.mode == "fused" else args.mode,
                "bytes_per_launch": moved, "bytes_formula": "P*(2M + 2*log2(N)*M/G)" if args.mode in ("fused", "auto") else "P*(2M + (3*log2(N)+2)*M/G)",
                "avg_launch_us": us,
                "schedule_bytes_per_launch": head["algorithmic_bytes"],
                "schedule_GBps": head["algorithmic_bytes"] / (us * 1e-6) / 1e9,
                # L2 <-> fabric bytes per launch from the committed rocprofv3 --pmc summary (the
                # memory-side cache can serve part of them, so this is not HBM traffic proper)
                "traffic_GBps": (traffic / (us * 1e-6) / 1e9) if traffic else None,
                "traffic_frac": (traffic / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS) if traffic else None}
    if not args.no_extras:
        # the kernel's duration with the memory-side cache and the L2s swept before every call
        cold = head["cold_between_events_us"]
        diff = head["cold_us"]
        roofline["cold"] = {"us": cold, "GBps": moved / (cold * 1e-6) / 1e9, "frac": moved / (cold * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                            "traffic_GBps": (traffic / (cold * 1e-6) / 1e9) if traffic else None,
                            "method": "a 256 MiB copy before every all-reduce; median of 35 eager (copy, all-reduce) pairs, HIP "
                                      "events around the all-reduce alone (the kernel's duration plus the gap before it)",
                            # what the pair costs beyond the copy: also charges the all-reduce for what it
                            # leaves the next copy to clean up
                            "graph_difference_us": diff,
                            "graph_difference_frac": moved / (diff * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                            "graph_difference_method": "HIP graphs of 20 x (256 MiB copy, all-reduce) minus graphs of the copies alone",
                            "after_read_only_sweep_us": head["cold_after_read_sweep_us"],
                            "after_read_only_sweep_note": "graph difference with a 512 MiB read-only sweep instead of the copy"}
        # behind the compute that produces its input (automatic mode, as a caller would run it)
        inter, inter_diff = head["interleaved_between_events_us"], head["graph100_interleaved_allreduce_us"]
        roofline["interleaved"] = {"us": inter, "GBps": moved / (inter * 1e-6) / 1e9, "frac": moved / (inter * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                                   "method": "every rank's row-parallel product (bf16, weights of hidden x hidden in total) written into its "
                                             "message before every all-reduce; median of 35 eager pairs, HIP events around the all-reduce alone",
                                   "graph_difference_us": inter_diff,
                                   "graph_difference_frac": moved / (inter_diff * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                                   "graph_difference_method": "HIP graphs of 100 x (products, all-reduce) minus graphs of the products alone"}
        roofline["streaming_ceilings"] = streaming_ceilings()
    line = {
        "metric": "us per all-reduce at 128KB-2MB bf16 (P virtual ranks); achieved HBM GB/s vs peak",
        "value": us,
        "unit": "us",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["fused_wall_us"] / 1000.0,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",             # the additions are binary32; the messages are stored as bf16
        "storage_dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: P={w.P} (G={w.G} x N={w.N}), {w.bytes_per_rank} B bf16 per rank, {args.mode} mode",
                   "tuning": head["tuning"]},
        "roofline": roofline,
    }
    if not args.no_extras:
        detail = {args.workload: head}
        detail.update(others)
        for k, v in detail.items():
            v["achieved_GBps"] = v["moved_bytes"] / (v["fused_us"] * 1e-6) / 1e9
            v["traffic"] = measured_traffic(k)   # L2 <-> fabric bytes per launch from the committed --pmc summaries
        line["detail"] = detail
        line["step_combine"] = bench_step_combine(min(args.warmup, 50), max(args.steps, MIN_CALLS_SHORT))
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
