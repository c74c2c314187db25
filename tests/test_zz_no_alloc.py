"""rar_allreduce_static: the all-reduce for callers that cannot allocate device memory.  It runs on
a scratch array inside the library instead of scratch lent by the caller; its output must be the
output of rar_allreduce (and the oracle's) bit for bit, on calls in a row that share the array,
the later ones with smaller and again larger inputs."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import rar_inputs as ri
from gpu_util import assert_same_bits, to_device, to_host

pytestmark = pytest.mark.gpu

rar = pytest.importorskip("paper_2511_09557_amd") if torch.cuda.is_available() else None


def through_static(x: np.ndarray, G: int, dtype: int) -> np.ndarray:
    """One call of rar_allreduce_static through the C ABI; the plan is given no scratch at all."""
    P, n = x.shape
    plan = rar.rar_plan(P, G, n, dtype)
    assert rar.rar_plan_static_bytes(plan) <= rar.RAR_STATIC_SCRATCH_BYTES
    bufs = to_device(x)
    ptrs = (ctypes.c_void_p * P)(*[b.data_ptr() for b in bufs])
    print(f"[gpu] rar_allreduce_static P={P} G={G} n={n} dtype={dtype}", flush=True)
    rc = rar.lib.rar_allreduce_static(ptrs, plan, torch.cuda.current_stream().cuda_stream)
    assert rc == 0, rar.rar_strerror(rc)
    assert rar.rar_plan_status(plan, torch.cuda.current_stream().cuda_stream) == 0
    out = to_host(bufs, x.dtype)
    rar.rar_plan_free(plan)
    return out


def through_existing(x: np.ndarray, G: int, dtype: int) -> np.ndarray:
    """The existing entry point, rar_allreduce, in the same mode on scratch lent by the caller."""
    P, n = x.shape
    ar = rar.AllReduce(P, G, n, dtype, rar.RAR_MODE_FUSED)
    bufs = to_device(x)
    ar(bufs)
    assert ar.status() == 0
    out = to_host(bufs, x.dtype)
    ar.close()
    return out


def test_static_scratch_calls_in_a_row():
    cases = [("bf16", 16, 4, 131072),     # 256 KiB per rank, P = 16
             ("bf16", 8, 4, 1000),        # a much smaller input right after it: another flag layout on the same array
             ("f32", 12, 4, 4099),        # three nodes, a ragged tail
             ("bf16", 32, 4, 524288)]     # larger again: 1 MiB per rank, P = 32 (32.1 MiB of the array)
    for k, (dtype, P, G, n) in enumerate(cases):
        x = ri.random_inputs(9100 + k, P, n, dtype)
        code = 0 if dtype == "bf16" else 1
        got = through_static(x, G, code)
        assert_same_bits(got, through_existing(x, G, code), f"call {k}: against rar_allreduce")
        assert_same_bits(got, oracle.allreduce(x, G, threads=8), f"call {k}: against the oracle")


def test_static_scratch_inside_a_graph():
    """The callers this entry point is for: captured in a HIP graph (after one eager call on the
    device) and replayed with fresh inputs, with an eager call of another shape between replays,
    which uses the same array."""
    P, G, n = 16, 4, 131072
    x = ri.random_inputs(9200, P, n, "bf16")
    want = oracle.allreduce(x, G, threads=8)
    plan = rar.rar_plan(P, G, n, 0)
    src = to_device(x)
    bufs = [t.clone() for t in src]
    ptrs = (ctypes.c_void_p * P)(*[b.data_ptr() for b in bufs])
    print("[gpu] rar_allreduce_static inside a graph", flush=True)
    assert rar.lib.rar_allreduce_static(ptrs, plan, torch.cuda.current_stream().cuda_stream) == 0   # eager first
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            assert rar.lib.rar_allreduce_static(ptrs, plan, stream.cuda_stream) == 0
    small = ri.random_inputs(9201, 8, 777, "f32")
    for rep in range(3):
        for b, s_ in zip(bufs, src):
            b.copy_(s_)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert rar.rar_plan_status(plan, 0) == 0
        assert_same_bits(to_host(bufs, x.dtype), want, f"replay {rep}")
        assert_same_bits(through_static(small, 4, 1), oracle.allreduce(small, 4), f"eager call between replays {rep}")
    rar.rar_plan_free(plan)


def test_static_scratch_limit():
    w = ri.WORKLOADS["c4"]                 # 160 MiB of partial buffers: beyond the array
    plan = rar.rar_plan(w.P, w.G, w.n, 0)
    assert rar.rar_plan_static_bytes(plan) > rar.RAR_STATIC_SCRATCH_BYTES
    bufs = [torch.zeros(w.n, dtype=torch.bfloat16, device="cuda:0") for _ in range(w.P)]
    ptrs = (ctypes.c_void_p * w.P)(*[b.data_ptr() for b in bufs])
    assert rar.lib.rar_allreduce_static(ptrs, plan, None) == -4
    rar.rar_plan_free(plan)


def test_static_scratch_keeps_a_timeout_until_it_is_reported():
    """The array's status word is shared by every plan on the GPU and no call clears it: a wait
    that gave up (forced here from the host with a wait limit of 0: a wait gives up as soon as it
    has looked once in vain; every kernel still runs to its end) is reported to the plan that caused it and to a plan that ran on the array before
    the report, however many calls were made in between, and the calls after the report are
    exact again."""
    P, G, n = 32, 4, 524288
    x = ri.random_inputs(9300, P, n, "bf16")
    want = oracle.allreduce(x, G, threads=8)
    st = torch.cuda.current_stream().cuda_stream
    a, b = rar.rar_plan(P, G, n, 0), rar.rar_plan(P, G, n, 0)
    rar.rar_plan_set_tuning(a, 2, 4096)                    # many trips, so some wait is all but certain to be pending
    bufs = to_device(x)
    ptrs = (ctypes.c_void_p * P)(*[t.data_ptr() for t in bufs])
    print("[gpu] rar_allreduce_static with a wait limit of 0", flush=True)
    rar.rar_plan_set_wait_limit_us(a, 0)
    for _ in range(3):                                     # no status query in between
        assert rar.lib.rar_allreduce_static(ptrs, a, st) == 0
    rar.rar_plan_set_wait_limit_us(a, 5_000_000)
    torch.cuda.synchronize()
    assert rar.lib.rar_allreduce_static(ptrs, b, st) == 0  # another plan, before anyone has asked
    first = rar.rar_plan_status(b, st)
    second = rar.rar_plan_status(a, st)
    assert first == -8 and second == -8                    # both ran beside the same status word
    for plan in (a, b):                                    # reported once, then clean
        for t, row in zip(bufs, x):
            t.copy_(torch.from_numpy(row.view(np.int16)).view(torch.bfloat16))
        assert rar.lib.rar_allreduce_static(ptrs, plan, st) == 0
        assert rar.rar_plan_status(plan, st) == 0
        assert_same_bits(to_host(bufs, x.dtype), want, "after the report")
    rar.rar_plan_free(a)
    rar.rar_plan_free(b)
