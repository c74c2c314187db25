"""GPU parity of rar_allreduce_chain: K all-reduces in ONE persistent launch, each on the result
of the one before, must give the bits of the CPU oracle applied K times."""
import numpy as np
import pytest
import torch

import oracle
import rar_inputs as ri
from gpu_util import assert_same_bits, to_device, to_host

pytestmark = pytest.mark.gpu

rar = pytest.importorskip("paper_2511_09557_amd") if torch.cuda.is_available() else None

DT = {"bf16": 0, "f32": 1}
MODES = {"fused": 1, "packed": 2, "auto": 3}


def oracle_times(x: np.ndarray, G: int, K: int) -> np.ndarray:
    for _ in range(K):
        x = oracle.allreduce(x, G, threads=8)
    return x


def scaled(x: np.ndarray, by: float) -> np.ndarray:
    """Inputs scaled down (by a power of two, exactly) so that K sums in a row stay finite."""
    if x.dtype == np.uint16:
        return ri.to_bf16_bits(ri.bf16_bits_to_f32(x) * np.float32(by))
    return (x * np.float32(by)).astype(np.float32)


def run_chain(x, G, mode, K, B_s=0, C_s=0, before=0, after=0):
    """`before` plain calls, one chain of K, `after` plain calls on one plan."""
    P, n = x.shape
    dtype = "bf16" if x.dtype == np.uint16 else "f32"
    print(f"[gpu] chain P={P} G={G} n={n} {dtype} mode={mode} K={K} B_s={B_s} C_s={C_s} before={before} after={after}", flush=True)
    ar = rar.AllReduce(P, G, n, DT[dtype], MODES[mode])
    ar.set_tuning(B_s, C_s)
    bufs = to_device(x)
    ar.bind(bufs)
    for _ in range(before):
        ar.launch()
    ar.launch_chain(K)
    for _ in range(after):
        ar.launch()
    assert ar.status() == 0
    out = to_host(bufs, x.dtype)
    ar.close()
    return out


@pytest.mark.parametrize("mode", ["fused", "packed", "auto"])
@pytest.mark.parametrize("name,K", [("c1", 5), ("c2", 4), ("c3", 3)])
def test_chain_matches_oracle_applied_k_times(name, K, mode):
    w = ri.WORKLOADS[name]
    x = scaled(ri.make_inputs(w), 2.0 ** -(K * int(np.log2(w.P)) - 2))
    want = oracle_times(x, w.G, K)
    assert_same_bits(run_chain(x, w.G, mode, K), want, f"{name} {mode} K={K}")


def test_chain_of_one_is_the_plain_call():
    w = ri.WORKLOADS["c2"]
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    for mode in ("fused", "packed"):
        assert_same_bits(run_chain(x, w.G, mode, 1), want, mode)


@pytest.mark.parametrize("mode", ["fused", "packed"])
@pytest.mark.parametrize("B_s,C_s", [(1, 4096), (2, 4096), (3, 8192), (8, 4096), (5, 16384), (0, 32768)])
def test_chain_with_several_trips_per_call(B_s, C_s, mode):
    """Several trips per call and workgroup: the trips of all calls form one sequence."""
    w = ri.WORKLOADS["c2"]
    K = 3
    x = scaled(ri.make_inputs(w), 2.0 ** -10)
    want = oracle_times(x, w.G, K)
    assert_same_bits(run_chain(x, w.G, mode, K, B_s, C_s), want, f"B_s={B_s} C_s={C_s}")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("P,G,n", [(8, 4, 1 << 20), (64, 4, 1 << 20), (16, 2, 700001), (4, 1, 300000)])
def test_chain_on_long_chunks(P, G, n, dtype):
    """Chunks of more than 256 KiB have no second set of buffers: the trips alternate between two
    places inside one partial buffer, and B_s is narrowed so that they fit."""
    K = 3
    x = scaled(ri.random_inputs(7100 + P + n, P, n, dtype), 2.0 ** -(K * int(np.log2(P))))
    want = oracle_times(x, G, K)
    assert_same_bits(run_chain(x, G, "fused", K), want, "built-in tuning")
    assert_same_bits(run_chain(x, G, "fused", K, B_s=256, C_s=4096), want, "widest grid asked for")
    assert_same_bits(run_chain(x, G, "fused", K, B_s=3, C_s=32768), want, "three workgroups per rank")


EDGE = [(1, 1, 1000), (2, 1, 9), (4, 4, 3), (8, 4, 33), (8, 8, 1029), (16, 1, 4097), (32, 8, 12345), (128, 4, 1001),
        # N that is not a power of two (outside the paper): N = 3, 5, 6, 7, 9, 25
        (12, 4, 1000), (3, 1, 9), (20, 4, 65536 + 24), (18, 3, 4099), (7, 1, 513), (36, 4, 262144), (100, 4, 50001),
        (128, 1, 5000), (96, 1, 777)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("P,G,n", EDGE)
def test_chain_edge_shapes(P, G, n, dtype):
    K = 3
    x = scaled(ri.random_inputs(8000 + P * 7 + n, P, n, dtype), 2.0 ** -(K * max(int(np.log2(P)), 1)))
    want = oracle_times(x, G, K)
    assert_same_bits(run_chain(x, G, "fused", K), want, "fused")
    assert_same_bits(run_chain(x, G, "packed", K), want, "packed")
    assert_same_bits(run_chain(x, G, "fused", K, B_s=1, C_s=4096), want, "fused, one workgroup per rank")
    assert_same_bits(run_chain(x, G, "packed", K, B_s=2, C_s=4096), want, "packed, two workgroups per rank")


@pytest.mark.parametrize("mode", ["fused", "packed"])
def test_chain_between_plain_calls(mode):
    """Plain calls before and after a chain on one plan: counters and sequence numbers of both
    sets of buffers stay the same on all ranks whatever the history."""
    w = ri.WORKLOADS["c1"]
    x = scaled(ri.make_inputs(w), 2.0 ** -20)
    want = oracle_times(x, w.G, 2 + 3 + 2)
    assert_same_bits(run_chain(x, w.G, mode, 3, before=2, after=2), want, mode)
    assert_same_bits(run_chain(x, w.G, mode, 3, B_s=2, C_s=4096, before=2, after=2), want, f"{mode}, several trips")


@pytest.mark.parametrize("mode", ["fused", "packed"])
def test_chain_counters_wrap(mode):
    """Counters (flag exchange) and sequence numbers (data+flag exchange) preset just below 2^32,
    the same on all ranks as any history of calls leaves them: chains across the wrap."""
    w = ri.WORKLOADS["c2"]
    K = 4
    x = scaled(ri.make_inputs(w), 2.0 ** -16)
    want = oracle_times(x, w.G, K)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, MODES[mode])
    ar.set_tuning(2, 4096)                       # 8 trips per call and workgroup: a chain of 4 moves the counters by 32
    bufs = to_device(x)
    ar.bind(bufs)
    ar.launch_chain(2)                           # first launch: clears flags and words, uses both sets
    assert ar.status() == 0
    f_off, f_bytes, p_off, p_bytes = rar.rar_plan_scratch_layout(ar.plan)
    base = ar.scratch_base
    if mode == "fused":
        ar.scratch[base + f_off: base + f_off + f_bytes].view(torch.int32).fill_(-20)
    else:
        assert p_bytes > 0
        # every word behind the first data+flag buffer: both sets (the partial buffers between them are rewritten before use)
        ar.scratch[base + p_off: base + p_off + p_bytes].view(torch.int64).fill_(-2 << 32)
    torch.cuda.synchronize()
    for k in range(3):
        print(f"[gpu] chain wrap {mode} launch {k}", flush=True)
        bufs = to_device(x)
        ar.bind(bufs)
        ar.launch_chain(K)
        assert ar.status() == 0
        assert_same_bits(to_host(bufs, x.dtype), want, f"{mode} launch {k} across the wrap")
    ar.close()


@pytest.mark.parametrize("mode", ["fused", "packed"])
def test_chain_in_a_graph(mode):
    """A chain captured in a HIP graph and replayed, with eager chains and plain calls in between."""
    w = ri.WORKLOADS["c2"]
    K = 3
    x = scaled(ri.make_inputs(w), 2.0 ** -12)
    want = oracle_times(x, w.G, K)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, MODES[mode])
    src = to_device(x)
    bufs = [t.clone() for t in src]
    ar.bind(bufs)
    ar.launch_chain(2)                           # eager first: set-up stays out of the graph
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            ar.launch_chain(K, stream)
    for rep in range(4):
        for b, s in zip(bufs, src):
            b.copy_(s)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_same_bits(to_host(bufs, x.dtype), want, f"graph replay {rep}")
        ar.launch() if rep % 2 else ar.launch_chain(rep + 1)
        torch.cuda.synchronize()
    assert ar.status() == 0
    ar.close()


def test_chain_under_replay():
    """2000 chains of changing length and launch shape on fresh inputs, flag exchange and data+flag
    exchange, each compared with the same number of stepwise calls (kernel boundaries only)."""
    P, G, n = 32, 4, 64 * 1024
    a = rar.AllReduce(P, G, n, 0, 1)
    b = rar.AllReduce(P, G, n, 0, 0)
    c = rar.AllReduce(P, G, n, 0, 2)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(987)
    src = torch.empty(P, n, device="cuda:0", dtype=torch.bfloat16)
    wa, wb, wc = torch.empty_like(src), torch.empty_like(src), torch.empty_like(src)
    a.bind([wa[p] for p in range(P)])
    b.bind([wb[p] for p in range(P)])
    c.bind([wc[p] for p in range(P)])
    print("[gpu] chain replay stress", flush=True)
    shapes = [(0, 0), (4, 4096), (3, 4096), (1, 8192), (2, 16384), (8, 4096)]
    for it in range(2000):
        if it % 10 == 0:
            src.copy_(torch.randn(P, n, device="cuda:0", generator=gen))
            src.mul_(2.0 ** -20)
        else:
            src.mul_(0.5)
        K = 1 + it % 4
        wa.copy_(src), wb.copy_(src), wc.copy_(src)
        a.set_tuning(*shapes[(it // 3) % len(shapes)])
        c.set_tuning(*shapes[(it // 7) % len(shapes)])
        a.launch_chain(K), c.launch_chain(K)
        for _ in range(K):
            b.launch()
        assert torch.equal(wa.view(torch.int16), wb.view(torch.int16)), ("fused", it, K)
        assert torch.equal(wc.view(torch.int16), wb.view(torch.int16)), ("packed", it, K)
    assert a.status() == 0 and c.status() == 0
    a.close(), b.close(), c.close()


def test_chain_rejects_bad_arguments():
    w = ri.WORKLOADS["c1"]
    ar = rar.AllReduce(w.P, w.G, w.n, 0, 1)
    bufs = to_device(ri.make_inputs(w))
    ar.bind(bufs)
    for K in (0, -1, (1 << 16) + 1):
        with pytest.raises(rar.RarError) as e:
            ar.launch_chain(K)
        assert e.value.status == -1
    ar.set_mode(0)
    with pytest.raises(rar.RarError) as e:
        ar.launch_chain(2)                       # the stepwise mode has no chain
    assert e.value.status == -1
    ar.close()
