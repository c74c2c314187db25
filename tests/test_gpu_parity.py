"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import rar_inputs as ri
from gpu_util import assert_same_bits, to_device, to_host

pytestmark = pytest.mark.gpu

rar = pytest.importorskip("paper_2511_09557_amd") if torch.cuda.is_available() else None

DT = {"bf16": 0, "f32": 1}
NP = {"bf16": np.uint16, "f32": np.float32}
MODES = {"stepwise": 0, "fused": 1, "packed": 2, "auto": 3}


def run_gpu(x: np.ndarray, G: int, mode: str, B_s: int = 0, C_s: int = 0, calls: int = 1) -> np.ndarray:
    P, n = x.shape
    dtype = "bf16" if x.dtype == np.uint16 else "f32"
    print(f"[gpu] allreduce P={P} G={G} n={n} {dtype} mode={mode} B_s={B_s} C_s={C_s} calls={calls}", flush=True)
    ar = rar.AllReduce(P, G, n, DT[dtype], MODES[mode])
    ar.set_tuning(B_s, C_s)
    bufs = to_device(x)
    for _ in range(calls):
        ar(bufs)
    assert ar.status() == 0
    out = to_host(bufs, x.dtype)
    ar.close()
    return out


# ---- one exchange-and-sum step ----------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("n,chunk", [(8, 0), (1000, 3), (4096, 1), (65536 + 8, 2), (1 << 20, 0), (5, 0), (1027, 0)])
def test_step_combine(dtype, n, chunk):
    print(f"[gpu] step_combine {dtype} n={n} chunk={chunk}", flush=True)
    total = (chunk + 2) * n
    x = ri.random_inputs(900 + n, 2, total, dtype)
    dst, src = x[0].copy(), x[1].copy()
    oracle.step_combine(dst, src, chunk, n)
    d, s = to_device(x)
    rar.rar_step_combine(d.data_ptr(), s.data_ptr(), chunk, n, DT[dtype], torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert_same_bits(to_host([d], x.dtype)[0], dst, "step_combine")
    assert_same_bits(to_host([s], x.dtype)[0], x[1], "src untouched")


def test_step_combine_rejects_bad_arguments():
    a = torch.zeros(64, dtype=torch.bfloat16, device="cuda:0")
    b = torch.zeros(64, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(rar.RarError):
        rar.rar_step_combine(a.data_ptr() + 2, b.data_ptr(), 0, 8, 0)     # misaligned
    with pytest.raises(rar.RarError):
        rar.rar_step_combine(a.data_ptr(), b.data_ptr(), 1, 3, 0)         # offset 6 bytes
    with pytest.raises(rar.RarError):
        rar.rar_step_combine(a.data_ptr(), a.data_ptr(), 0, 8, 0)         # overlap
    with pytest.raises(rar.RarError):
        rar.rar_step_combine(a.data_ptr(), b.data_ptr(), 0, 8, 7)         # dtype
    with pytest.raises(rar.RarError):
        rar.rar_step_combine(0, b.data_ptr(), 0, 8, 0)                    # NULL
    rar.rar_step_combine(a.data_ptr(), b.data_ptr(), 0, 0, 0)             # n = 0 is a no-op
    torch.cuda.synchronize()


# ---- the five workloads -------------------------------------------------------------------------

@pytest.mark.parametrize("mode", ["stepwise", "fused", "packed", "auto"])
@pytest.mark.parametrize("name", ["c1", "c1_int", "c2", "c3", "c4"])
def test_workloads_bit_exact(name, mode):
    w = ri.WORKLOADS[name]
    if mode == "packed" and name == "c4":
        # a 512 KiB chunk is beyond the packed mode's limit: the planner must say so
        plan = rar.rar_plan(w.P, w.G, w.n, 0)
        with pytest.raises(rar.RarError) as e:
            rar.rar_plan_set_mode(plan, 2)
        assert e.value.status == -4
        rar.rar_plan_free(plan)
        return
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    got = run_gpu(x, w.G, mode)
    assert_same_bits(got, want, f"{name}/{mode}")
    if name == "c1_int":
        exact = ri.bf16_bits_to_f32(x).astype(np.int64).sum(axis=0).astype(np.float32)
        assert np.array_equal(ri.bf16_bits_to_f32(got), np.broadcast_to(exact, got.shape))
    # within the stated distance of the plain fp64 sum, away from cancellation
    ref, mag = oracle.naive_sum_f64(x)
    away = np.abs(ref) >= mag / 2
    rel = np.abs(ri.bf16_bits_to_f32(got[0]).astype(np.float64)[away] - ref[away]) / np.abs(ref[away])
    assert rel.max() <= 2.0 ** -7 * np.log2(w.P)


@pytest.mark.parametrize("name", ["c3", "c4"])
def test_workloads_in_the_benchmark_layout(name):
    """bench.py keeps the P messages as rows of one allocation and binds them once; same here,
    with the tuning the library picks by itself, two launches, against the oracle applied twice."""
    w = ri.WORKLOADS[name]
    x = ri.to_bf16_bits(ri.bf16_bits_to_f32(ri.make_inputs(w)) / 64.0)
    want = oracle.allreduce(oracle.allreduce(x, w.G, threads=8), w.G, threads=8)
    whole = torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).to("cuda:0")
    bufs = [whole[p] for p in range(w.P)]
    ar = rar.AllReduce(w.P, w.G, w.n, 0, 1)
    ar.bind(bufs)
    print(f"[gpu] benchmark layout {name} tuning={ar.tuning()}", flush=True)
    ar.launch()
    ar.launch()
    assert ar.status() == 0
    assert_same_bits(whole.cpu().view(torch.int16).numpy().view(np.uint16), want, name)
    ar.close()


SWEEP = [(8, 4), (16, 4), (32, 4), (64, 4), (128, 4), (64, 8)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("P,G", SWEEP)
def test_sweep_small_sizes_bit_exact(P, G, dtype):
    for nbytes in (8 << 10, 64 << 10, 512 << 10):
        w = ri.sweep_workload(P, G, nbytes, dtype)
        x = ri.make_inputs(w)
        want = oracle.allreduce(x, G, threads=8)
        assert_same_bits(run_gpu(x, G, "fused"), want, w.name)
        assert_same_bits(run_gpu(x, G, "packed"), want, w.name + "/packed")
        if nbytes == 64 << 10:
            assert_same_bits(run_gpu(x, G, "stepwise"), want, w.name + "/stepwise")
            ref, mag = oracle.naive_sum_f64(x)
            if dtype == "f32":
                sel = np.abs(ref) >= mag / 4
                assert (np.abs(want[0].astype(np.float64)[sel] - ref[sel]) / np.abs(ref[sel])).max() <= 2.0 ** -20


def test_sweep_large_size_sampled():
    """64 MiB per rank at P = 8: the oracle checks a strided sample of columns (every element
    is reduced independently, so the oracle on a column subset is the oracle's value there)."""
    P, G, dtype = 8, 4, "bf16"
    n = (64 << 20) // 2
    rng = np.random.default_rng(ri.SEED_BASE + 499)
    base = ri.to_bf16_bits(rng.standard_normal((P, 1 << 20), dtype=np.float32))
    reps = n // base.shape[1]
    bufs = []
    for p in range(P):
        row = torch.from_numpy(np.roll(base[p], 977 * p).view(np.int16).copy()).view(torch.bfloat16)
        # tile the seeded block, each repeat scaled by an exact power of two so that columns differ
        dev = row.to("cuda:0").repeat(reps).view(reps, -1)
        scale = torch.tensor([2.0 ** ((r % 7) - 3) for r in range(reps)], dtype=torch.bfloat16, device="cuda:0")
        bufs.append((dev * scale[:, None]).reshape(-1).contiguous())
    cols = np.unique(np.concatenate([np.arange(0, n, 4099), np.arange(n - 4096, n), np.arange(0, 4096),
                                     np.arange(n // 4 - 64, n // 4 + 64)]))
    ci = torch.from_numpy(cols).to("cuda:0")
    x_s = np.stack([b[ci].cpu().view(torch.int16).numpy().view(np.uint16) for b in bufs])
    want = oracle.allreduce(x_s, G, threads=8)     # element-wise independent: chunking is irrelevant
    for mode in ("fused", "stepwise"):
        work = [b.clone() for b in bufs]
        print(f"[gpu] large sampled P={P} n={n} mode={mode}", flush=True)
        ar = rar.AllReduce(P, G, n, 0, MODES[mode])
        ar(work)
        assert ar.status() == 0
        got = np.stack([b[ci].cpu().view(torch.int16).numpy().view(np.uint16) for b in work])
        assert_same_bits(got, want, f"large/{mode}")
        for p in range(1, P):
            assert torch.equal(work[p].view(torch.int16), work[0].view(torch.int16))
        ar.close()


@pytest.mark.parametrize("P,G,nbytes,dtype", [(128, 4, 4 << 20, "bf16"), (64, 8, 16 << 20, "f32"), (32, 4, 32 << 20, "bf16"),
                                               (16, 4, 8 << 20, "f32")])
def test_sweep_large_points_sampled(P, G, nbytes, dtype):
    """Large sweep points (several trips per workgroup, partial buffers reused): inputs drawn on
    the device from a seeded torch generator, the oracle checks a strided sample of columns plus
    both ends and the chunk borders."""
    tdt, es = (torch.bfloat16, 2) if dtype == "bf16" else (torch.float32, 4)
    n = nbytes // es
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(ri.SEED_BASE + 450 + P + G)
    whole = torch.empty(P, n, device="cuda:0", dtype=tdt)
    for p in range(P):
        whole[p] = torch.randn(n, device="cuda:0", generator=gen).to(tdt)
    q = n // G
    cols = np.unique(np.concatenate([np.arange(0, n, 8191), np.arange(0, 2048), np.arange(n - 2048, n)] +
                                    [np.arange(c * q - 256, c * q + 256) for c in range(1, G)]))
    ci = torch.from_numpy(cols).to("cuda:0")

    def sample(t):
        h = t[:, ci].cpu()
        return h.view(torch.int16).numpy().view(np.uint16) if dtype == "bf16" else h.numpy()

    want = oracle.allreduce(np.ascontiguousarray(sample(whole)), G, threads=8)
    for mode in ("fused", "stepwise"):
        work = whole.clone()
        bufs = [work[p] for p in range(P)]
        ar = rar.AllReduce(P, G, n, DT[dtype], MODES[mode])
        print(f"[gpu] large point P={P} G={G} {nbytes} B {dtype} {mode} tuning={ar.tuning()}", flush=True)
        ar(bufs)
        assert ar.status() == 0
        assert_same_bits(np.ascontiguousarray(sample(work)), want, f"{mode}")
        first = work[0].view(torch.int16 if dtype == "bf16" else torch.int32)
        nan = torch.isnan(work[0])
        for p in range(1, P):
            other = work[p].view(first.dtype)
            assert torch.equal(other[~nan], first[~nan])
        ar.close()
        del work, bufs


# ---- edge cases -------------------------------------------------------------------------------------

EDGE = [(1, 1, 1), (1, 1, 1000), (2, 1, 9), (2, 2, 9), (4, 4, 3), (4, 2, 17), (8, 4, 1), (8, 4, 7),
        (8, 4, 31), (8, 4, 33), (8, 4, 4 * 8 * 256 + 5), (8, 8, 1029), (16, 1, 4097), (16, 4, 65536 + 24),
        (32, 8, 12345), (128, 4, 1001), (128, 8, 40000), (6, 3, 1000), (12, 3, 77), (5, 5, 64),
        # N that is not a power of two (outside the paper): N = 3, 5, 6, 7, 9, 11, 25, 31
        (12, 4, 1000), (3, 1, 9), (20, 4, 65536 + 24), (18, 3, 4099), (7, 1, 513), (36, 4, 262144),
        (88, 8, 30000), (100, 4, 50001), (124, 4, 8 * 4096),
        # the most steps the library allows: N = 128 (L = 7), and N = 96, 127 (L = 6, r = 32, 63)
        (128, 1, 5000), (64, 1, 60000), (128, 2, 70001), (96, 1, 777), (127, 1, 30000)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("P,G,n", EDGE)
def test_edge_shapes(P, G, n, dtype):
    x = ri.random_inputs(5000 + P * 7 + n, P, n, dtype)
    want = oracle.allreduce(x, G)
    assert_same_bits(run_gpu(x, G, "fused"), want, "fused")
    assert_same_bits(run_gpu(x, G, "stepwise"), want, "stepwise")
    assert_same_bits(run_gpu(x, G, "auto"), want, "auto")
    N = P // G
    if N & (N - 1):
        # several trips per workgroup (three or more make a workgroup reuse its two places in
        # every partial buffer) with the hand-over before and after the steps
        assert_same_bits(run_gpu(x, G, "fused", B_s=1, C_s=4096, calls=1), want, "fused, one workgroup per rank")
    assert_same_bits(run_gpu(x, G, "packed"), want, "packed")
    assert_same_bits(run_gpu(x, G, "packed", B_s=1, C_s=4096), want, "packed, one workgroup per rank")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_special_values(dtype):
    P, G, n = 16, 4, 8192 + 3
    rng = np.random.default_rng(42)
    if dtype == "bf16":
        pool = np.concatenate([ri.to_bf16_bits(np.array([0.0, -0.0, 2.0 ** -133, -2.0 ** -133, 2.0 ** -126, 3.0e38,
                                                         -3.0e38, 1.0, 256.0, 257.0, 0.5], dtype=np.float32)),
                               np.array([0x7F80, 0xFF80, 0x0001, 0x8001, 0x007F], dtype=np.uint16)])
        x = pool[rng.integers(0, pool.size, size=(P, n))]
        x[:, : n // 2] = rng.integers(0, 1 << 16, size=(P, n // 2), dtype=np.uint16)   # any bit pattern, NaN included
    else:
        pool = np.array([0.0, -0.0, 1e-45, -1e-45, 1e-40, 3e38, -3e38, np.inf, -np.inf, 2.0 ** 24, 1.0, 0.5, 1 / 3],
                        dtype=np.float32)
        x = pool[rng.integers(0, pool.size, size=(P, n))]
        x[:, : n // 2] = rng.integers(0, 1 << 32, size=(P, n // 2), dtype=np.uint32).view(np.float32)
    want = oracle.allreduce(x, G)
    assert_same_bits(run_gpu(x, G, "fused"), want, "fused")
    assert_same_bits(run_gpu(x, G, "stepwise"), want, "stepwise")
    assert_same_bits(run_gpu(x, G, "packed"), want, "packed")


@pytest.mark.parametrize("B_s,C_s", [(1, 4096), (2, 8192), (3, 4096), (8, 16384), (16, 32768), (256, 4096), (5, 0), (0, 8192)])
def test_tuning_never_changes_bits(B_s, C_s):
    w = ri.WORKLOADS["c2"]
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    assert_same_bits(run_gpu(x, w.G, "fused", B_s=B_s, C_s=C_s), want, f"B_s={B_s} C_s={C_s}")
    assert_same_bits(run_gpu(x, w.G, "packed", B_s=B_s, C_s=C_s), want, f"packed B_s={B_s} C_s={C_s}")


@pytest.mark.parametrize("mode", ["fused", "packed"])
def test_autotune_keeps_bits(mode):
    w = ri.WORKLOADS["c2"]
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, MODES[mode])
    print(f"[gpu] autotune {mode}", flush=True)
    best = ar.autotune(to_device(x), calls=5)
    B_s, C_s = ar.tuning()
    assert best > 0 and B_s >= 1 and C_s in (4096, 8192, 16384, 32768)
    bufs = to_device(x)
    ar(bufs)
    assert ar.status() == 0
    assert_same_bits(to_host(bufs, x.dtype), want, f"after autotune ({B_s}, {C_s})")
    ar.set_mode(0)
    with pytest.raises(rar.RarError):
        ar.autotune(bufs, calls=1)
    ar.close()


def test_repeated_calls_in_place():
    """Three chained in-place calls; flags are counters that are never cleared in between."""
    w = ri.WORKLOADS["c1"]
    x = ri.make_inputs(w)
    x = ri.to_bf16_bits(ri.bf16_bits_to_f32(x) / 64.0)
    want = x
    for _ in range(3):
        want = oracle.allreduce(want, w.G)
    assert_same_bits(run_gpu(x, w.G, "fused", calls=3), want, "fused x3")
    assert_same_bits(run_gpu(x, w.G, "fused", B_s=2, C_s=4096, calls=3), want, "fused x3, several trips")
    assert_same_bits(run_gpu(x, w.G, "stepwise", calls=3), want, "stepwise x3")
    assert_same_bits(run_gpu(x, w.G, "packed", calls=3), want, "packed x3")
    assert_same_bits(run_gpu(x, w.G, "packed", B_s=2, C_s=4096, calls=3), want, "packed x3, several trips")
    assert_same_bits(run_gpu(x, w.G, "auto", calls=3), want, "auto x3")


@pytest.mark.parametrize("mode", ["fused", "packed"])
def test_sequence_numbers_wrap(mode):
    """The step-barrier counters (flag exchange) and the sequence numbers in the exchanged words
    (data+flag exchange) are 32-bit and only ever grow: preset them just below 2^32, the same on all
    ranks as any history of calls leaves them, and run calls across the wrap."""
    w = ri.WORKLOADS["c2"]
    x = ri.to_bf16_bits(ri.bf16_bits_to_f32(ri.make_inputs(w)) / 64.0)
    want = oracle.allreduce(x, w.G, threads=8)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, MODES[mode])
    ar.set_tuning(2, 4096)                       # 8 trips per workgroup: the counters move 8 per call
    bufs = to_device(x)
    ar(bufs)                                     # first call: clears flags and words
    assert ar.status() == 0
    f_off, f_bytes, p_off, p_bytes = rar.rar_plan_scratch_layout(ar.plan)
    base = ar.scratch_base
    if mode == "fused":
        flags = ar.scratch[base + f_off: base + f_off + f_bytes].view(torch.int32)
        flags.fill_(-20)                         # 0xFFFFFFEC: wraps during the third call
    else:
        assert p_bytes > 0
        words = ar.scratch[base + p_off: base + p_off + p_bytes].view(torch.int64)
        words.fill_(-3 << 32)                    # sequence number 0xFFFFFFFD in every word: next calls use ..FE, ..FF, then 1
    torch.cuda.synchronize()
    for k in range(6):
        print(f"[gpu] wrap {mode} call {k}", flush=True)
        bufs = to_device(x)
        ar(bufs)
        assert ar.status() == 0
        assert_same_bits(to_host(bufs, x.dtype), want, f"{mode} call {k} across the wrap")
    if mode == "packed":
        seq = (words[0].item() >> 32) & 0xFFFFFFFF
        assert seq == 4, seq                     # ..FE, ..FF, (0 skipped) 1, 2, 3, 4
    ar.close()


def test_packed_mode_alternating_with_flag_mode():
    """One plan switched between the data+flag exchange and the flag exchange with changing launch
    shapes: a word position's sequence number advances only in the calls that write it, and by
    the same amount on every rank."""
    w = ri.WORKLOADS["c2"]
    x = ri.to_bf16_bits(ri.bf16_bits_to_f32(ri.make_inputs(w)) / 64.0)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, 2)
    order = [(2, 0, 0), (1, 0, 0), (2, 3, 4096), (2, 1, 8192), (1, 2, 4096), (2, 16, 4096), (3, 0, 0), (2, 5, 16384),
             (0, 0, 0), (2, 2, 32768), (2, 0, 0)]
    want = oracle.allreduce(x, w.G, threads=8)
    for k, (mode, B_s, C_s) in enumerate(order):
        print(f"[gpu] alternating call {k}: mode {mode} B_s={B_s} C_s={C_s}", flush=True)
        ar.set_mode(mode)
        ar.set_tuning(B_s, C_s)
        bufs = to_device(x)
        ar(bufs)
        assert ar.status() == 0
        assert_same_bits(to_host(bufs, x.dtype), want, f"call {k}")
    ar.close()


def test_odd_node_count_under_replay():
    """N = 6 nodes (outside the paper): 300 calls of the flag exchange and of the data+flag exchange
    with fresh inputs and changing launch shapes against the stepwise path; the hand-over before
    and after the steps uses the same flags and sequence numbers as the steps."""
    P, G, n = 24, 4, 96 * 1024
    a = rar.AllReduce(P, G, n, 0, 1)
    b = rar.AllReduce(P, G, n, 0, 0)
    c = rar.AllReduce(P, G, n, 0, 2)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(4321)
    src = torch.empty(P, n, device="cuda:0", dtype=torch.bfloat16)
    wa, wb, wc = torch.empty_like(src), torch.empty_like(src), torch.empty_like(src)
    a.bind([wa[p] for p in range(P)])
    b.bind([wb[p] for p in range(P)])
    c.bind([wc[p] for p in range(P)])
    print("[gpu] replay stress, N = 6", flush=True)
    shapes = [(0, 0), (2, 4096), (3, 4096), (1, 8192), (5, 16384), (1, 32768)]
    for it in range(300):
        if it % 10 == 0:
            src.copy_(torch.randn(P, n, device="cuda:0", generator=gen))
        else:
            src.mul_(0.5)
        wa.copy_(src), wb.copy_(src), wc.copy_(src)
        a.set_tuning(*shapes[(it // 3) % len(shapes)])
        c.set_tuning(*shapes[(it // 7) % len(shapes)])
        a.launch(), b.launch(), c.launch()
        assert torch.equal(wa.view(torch.int16), wb.view(torch.int16)), ("fused", it)
        assert torch.equal(wc.view(torch.int16), wb.view(torch.int16)), ("packed", it)
        assert torch.equal(wb[P - 1].view(torch.int16), wb[0].view(torch.int16)), ("ranks differ", it)
    assert a.status() == 0 and c.status() == 0
    c.close()
    x = src.cpu().view(torch.int16).numpy().view(np.uint16)
    assert_same_bits(wb.cpu().view(torch.int16).numpy().view(np.uint16), oracle.allreduce(x, G, threads=8), "stepwise, last input")
    a.close(), b.close()


def test_fused_equals_stepwise_under_replay():
    """Stress of the flag protocol: 10,000 fused and packed calls with fresh inputs and changing
    launch shapes (odd B_s puts the exchanging workgroups on different XCDs), each compared with
    the stepwise path, which synchronises by kernel boundaries only."""
    P, G, n = 32, 4, 256 * 1024
    a = rar.AllReduce(P, G, n, 0, 1)
    b = rar.AllReduce(P, G, n, 0, 0)
    c = rar.AllReduce(P, G, n, 0, 2)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(1234)
    src = torch.empty(P, n, device="cuda:0", dtype=torch.bfloat16)
    wa, wb, wc = torch.empty_like(src), torch.empty_like(src), torch.empty_like(src)
    a.bind([wa[p] for p in range(P)])
    b.bind([wb[p] for p in range(P)])
    c.bind([wc[p] for p in range(P)])
    print("[gpu] replay stress", flush=True)
    shapes = [(0, 0), (4, 8192), (3, 4096), (5, 16384), (1, 32768), (16, 4096)]
    for it in range(10000):
        if it % 10 == 0:
            src.copy_(torch.randn(P, n, device="cuda:0", generator=gen))
        else:
            src.mul_(0.5)
        wa.copy_(src), wb.copy_(src), wc.copy_(src)
        a.set_tuning(*shapes[(it // 3) % len(shapes)])
        c.set_tuning(*shapes[(it // 7) % len(shapes)])
        a.launch(), b.launch(), c.launch()
        assert torch.equal(wa.view(torch.int16), wb.view(torch.int16)), ("fused", it)
        assert torch.equal(wc.view(torch.int16), wb.view(torch.int16)), ("packed", it)
        assert torch.equal(wb[P - 1].view(torch.int16), wb[0].view(torch.int16)), ("ranks differ", it)
        if it % 1000 == 999:
            print(f"[gpu] replay stress: {it + 1} calls", flush=True)
    assert a.status() == 0 and c.status() == 0
    a.close(), b.close(), c.close()


@pytest.mark.parametrize("mode", ["fused", "packed", "auto"])
def test_graph_replay(mode):
    """The fused call inside a HIP graph, replayed with eager work in between."""
    w = ri.WORKLOADS["c2"]
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, MODES[mode])
    src = to_device(x)
    bufs = [t.clone() for t in src]
    ar(bufs)                                   # eager warm-up: clears the flags once
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        for b, s in zip(bufs, src):
            b.copy_(s)
        with torch.cuda.graph(graph, stream=stream):
            ar(bufs, stream)
    for rep in range(4):
        for b, s in zip(bufs, src):
            b.copy_(s)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_same_bits(to_host(bufs, x.dtype), want, f"graph replay {rep}")
        ar(bufs)                               # eager call between replays advances the counters too
        torch.cuda.synchronize()
    assert ar.status() == 0
    ar.close()


def force_timeout(ar, bufs, calls=20):
    """Launch with a wait limit of 0 (a wait gives up as soon as it has looked once without finding
    its flag or word) until a wait has given up.  Every kernel still runs to its end.  Returns
    whether a time-out was reported; the plan is re-armed."""
    rar.rar_plan_set_wait_limit_us(ar.plan, 0)
    seen = False
    try:
        for _ in range(calls):
            try:
                ar(bufs)
            except rar.RarError as e:             # the launch itself refuses: the plan is poisoned
                assert e.status == -8
                assert ar.status() == -8          # the report re-arms the plan
                seen = True
                break
            if ar.status() == -8:
                seen = True
                break
    finally:
        rar.rar_plan_set_wait_limit_us(ar.plan, 5_000_000)
    return seen


@pytest.mark.parametrize("mode", ["fused", "packed"])
def test_wait_limit_ends_every_workgroup(mode):
    """A wait limit of 0 makes waits give up instead of spinning: the kernel must still
    finish, report the time-out, and the plan must work again afterwards."""
    w = ri.WORKLOADS["c3"]
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, MODES[mode])
    ar.set_tuning(2, 4096)                     # many trips, so some wait is certain to be pending
    bufs = to_device(x)
    print("[gpu] wait-limit run", flush=True)
    assert force_timeout(ar, bufs), "thousands of waits, and not one had to look twice?"
    assert ar.status() == 0                    # reported once, then clean
    bufs = to_device(x)
    ar(bufs)
    assert ar.status() == 0
    assert_same_bits(to_host(bufs, x.dtype), want, "after a time-out")
    ar.close()


def test_a_timed_out_plan_refuses_to_launch():
    """After a wait has given up, the plan's flags cannot be trusted: every launch returns
    RAR_ERR_TIMEOUT and enqueues nothing until rar_plan_status has been asked."""
    w = ri.WORKLOADS["c3"]
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, 1)
    ar.set_tuning(2, 4096)
    bufs = to_device(x)
    ar.bind(bufs)
    rar.rar_plan_set_wait_limit_us(ar.plan, 0)   # a wait gives up as soon as it has looked once in vain
    print("[gpu] poisoned plan", flush=True)
    refused = False
    for _ in range(30):
        try:
            ar.launch()
        except rar.RarError as e:
            assert e.status == -8
            refused = True
            break
        torch.cuda.synchronize()               # the kernel has ended: its report, if any, is in host memory
    rar.rar_plan_set_wait_limit_us(ar.plan, 5_000_000)
    assert refused, "thousands of waits, and not one had to look twice?"
    before = [b.clone() for b in bufs]
    for call in (ar.launch, lambda: ar.launch_chain(2), ar.barrier_only):
        with pytest.raises(rar.RarError) as e:
            call()
        assert e.value.status == -8
    torch.cuda.synchronize()
    for b, old in zip(bufs, before):           # nothing was enqueued
        assert torch.equal(b.view(torch.int16), old.view(torch.int16))
    assert ar.status() == -8
    assert ar.status() == 0
    bufs = to_device(x)
    ar(bufs)
    assert ar.status() == 0
    assert_same_bits(to_host(bufs, x.dtype), want, "after the report")
    ar.close()


@pytest.mark.parametrize("limit_us", [0, 1])
def test_autotune_discards_candidates_that_time_out(limit_us):
    """rar_autotune under a wait limit that waits cannot keep: candidates during which a wait gave
    up do not count.  With a limit of 0 (give up after the first look) none survives and the call
    says RAR_ERR_TIMEOUT; with 1 us (the clock is looked at every 32 polls) some candidate may
    survive, and the plan must then be clean and exact with the chosen pair.  The plan works
    afterwards either way."""
    w = ri.WORKLOADS["c3"]
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, 1)
    rar.rar_plan_set_wait_limit_us(ar.plan, limit_us)
    print(f"[gpu] autotune under a wait limit of {limit_us} us", flush=True)
    try:
        ar.autotune(to_device(x), calls=5)
        outcome = "a candidate survived"
    except rar.RarError as e:
        assert e.status == -8
        outcome = "no candidate survived"
    assert limit_us != 0 or outcome == "no candidate survived"
    rar.rar_plan_set_wait_limit_us(ar.plan, 5_000_000)
    assert ar.status() == 0                    # autotune leaves no time-out pending
    bufs = to_device(x)
    ar(bufs)
    assert ar.status() == 0
    assert_same_bits(to_host(bufs, x.dtype), want, outcome)
    print(f"[gpu] autotune under a wait limit of {limit_us} us: {outcome}", flush=True)
    ar.close()


def test_first_call_inside_capture_is_refused():
    """A plan's first launch sets up flags and host memory and cannot be part of a graph."""
    w = ri.WORKLOADS["c1"]
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, 1)
    bufs = to_device(x)
    ar.bind(bufs)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    print("[gpu] first call inside capture", flush=True)
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            with pytest.raises(rar.RarError) as e:
                ar.launch(stream)
            assert e.value.status == -10
    torch.cuda.synchronize()
    ar.launch()                                # eager: fine, and later captures are too
    assert ar.status() == 0
    assert_same_bits(to_host(bufs, x.dtype), want, "eager after the refused capture")
    ar.close()


@pytest.mark.parametrize("mode", ["fused", "auto"])
@pytest.mark.parametrize("name", ["c2", "c4"])
def test_two_plans_on_two_streams(name, mode):
    """Two independent all-reduces (two plans, two sets of buffers) enqueued on two streams so that
    their kernels overlap, each plan told that it shares the device with one other (so that the
    two grids together stay resident): both must give the oracle's bits."""
    w = ri.WORKLOADS[name]
    xa = ri.make_inputs(w)
    xb = np.ascontiguousarray(xa[::-1])           # the same rows in another rank order: another result
    want_a, want_b = oracle.allreduce(xa, w.G, threads=8), oracle.allreduce(xb, w.G, threads=8)
    a = rar.AllReduce(w.P, w.G, w.n, 0, MODES[mode])
    b = rar.AllReduce(w.P, w.G, w.n, 0, MODES[mode])
    for p in (a, b):
        rar.rar_plan_set_wait_limit_us(p.plan, 2_000_000)
        rar.rar_plan_set_concurrency(p.plan, 2)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        ba, bb = to_device(xa), to_device(xb)
        a.bind(ba), b.bind(bb)
        torch.cuda.synchronize()
        print(f"[gpu] two plans {name} {mode} rep {rep}", flush=True)
        for _ in range(1):
            a.launch(s1)
            b.launch(s2)
        assert a.status(s1) == 0 and b.status(s2) == 0
        assert_same_bits(to_host(ba, xa.dtype), want_a, "chain a")
        assert_same_bits(to_host(bb, xb.dtype), want_b, "chain b")
    a.close(), b.close()


@pytest.mark.parametrize("mode", ["fused", "packed"])
def test_compute_on_another_stream_at_the_same_time(mode):
    """Matrix products on a second stream compete for the compute units while the all-reduce runs,
    so its workgroups are not all resident at once.  The step waits must still end: every call that
    reports no time-out has the oracle's bits, and a call that does report one is followed by a
    clean call on the same plan; it never hangs."""
    w = ri.WORKLOADS["c3"]
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, MODES[mode])
    rar.rar_plan_set_wait_limit_us(ar.plan, 500_000)
    a = torch.randn(8192, 8192, device="cuda:0", dtype=torch.bfloat16)
    b = torch.randn(8192, 8192, device="cuda:0", dtype=torch.bfloat16)
    side = torch.cuda.Stream()
    ok = 0
    for rep in range(5):
        bufs = to_device(x)
        torch.cuda.synchronize()
        print(f"[gpu] concurrent compute {mode} rep {rep}", flush=True)
        with torch.cuda.stream(side):
            for _ in range(4):
                torch.matmul(a, b)
        ar(bufs)                                   # on the current stream, while the products run
        status = ar.status()
        side.synchronize()
        assert status in (0, -8)
        if status == 0:
            assert_same_bits(to_host(bufs, x.dtype), want, f"{mode} rep {rep}")
            ok += 1
        else:                                      # the device is idle now: the plan must recover at once
            bufs = to_device(x)
            ar(bufs)
            assert ar.status() == 0
            assert_same_bits(to_host(bufs, x.dtype), want, f"{mode} rep {rep}, call after the time-out")
    print(f"[gpu] concurrent compute {mode}: {ok} of 5 calls completed", flush=True)
    assert ok >= 1
    ar.close()


def test_allreduce_rejects_bad_arguments():
    P, G, n = 8, 4, 1024
    plan = rar.rar_plan(P, G, n, 0)
    bufs = [torch.zeros(n, dtype=torch.bfloat16, device="cuda:0") for _ in range(P)]
    ptrs = [b.data_ptr() for b in bufs]
    with pytest.raises(rar.RarError) as e:
        rar.rar_allreduce(ptrs, plan)           # no scratch
    assert e.value.status == -5
    scratch = torch.empty(rar.rar_plan_scratch_bytes(plan) + 256, dtype=torch.uint8, device="cuda:0")
    base = (scratch.data_ptr() + 255) // 256 * 256
    with pytest.raises(rar.RarError):
        rar.rar_plan_set_scratch(plan, base, 100)          # too small
    with pytest.raises(rar.RarError):
        rar.rar_plan_set_scratch(plan, base + 16, rar.rar_plan_scratch_bytes(plan))   # misaligned
    rar.rar_plan_set_scratch(plan, base, rar.rar_plan_scratch_bytes(plan))
    with pytest.raises(rar.RarError) as e:
        rar.rar_allreduce([ptrs[0] + 2] + ptrs[1:], plan)
    assert e.value.status == -6
    with pytest.raises(rar.RarError):
        rar.rar_allreduce([0] + ptrs[1:], plan)
    rar.rar_allreduce(ptrs, plan)
    torch.cuda.synchronize()
    rar.rar_plan_free(plan)


@pytest.mark.parametrize("mode", ["fused", "auto"])
@pytest.mark.parametrize("name", ["c2", "c4"])
def test_two_default_plans_on_two_streams(name, mode):
    """Two plans that were told nothing about each other, launched back to back on two streams: the
    library orders the second fused kernel after the first (an event between the streams), so both
    complete with the oracle's bits and no wait times out."""
    w = ri.WORKLOADS[name]
    xa = ri.make_inputs(w)
    xb = np.ascontiguousarray(xa[::-1])
    want_a, want_b = oracle.allreduce(xa, w.G, threads=8), oracle.allreduce(xb, w.G, threads=8)
    a = rar.AllReduce(w.P, w.G, w.n, 0, MODES[mode])
    b = rar.AllReduce(w.P, w.G, w.n, 0, MODES[mode])
    for p in (a, b):
        rar.rar_plan_set_wait_limit_us(p.plan, 2_000_000)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        ba, bb = to_device(xa), to_device(xb)
        a.bind(ba), b.bind(bb)
        torch.cuda.synchronize()
        print(f"[gpu] two default plans {name} {mode} rep {rep}", flush=True)
        for _ in range(1 + 9 * (rep == 2)):        # the last repetition: ten alternating pairs in a row
            a.launch(s1)
            b.launch(s2)
        torch.cuda.synchronize()
        assert a.status(s1) == 0 and b.status(s2) == 0
        if rep < 2:
            assert_same_bits(to_host(ba, xa.dtype), want_a, "plan a")
            assert_same_bits(to_host(bb, xb.dtype), want_b, "plan b")
    a.close(), b.close()


def test_two_default_plans_in_one_graph():
    """Two plans with the default concurrency on two streams of ONE capture (the second stream forked
    from the first): the library's ordering becomes edges of the graph, the two chains run one
    kernel at a time, and every replay gives the oracle's bits."""
    w = ri.WORKLOADS["c2"]
    xa = ri.to_bf16_bits(ri.bf16_bits_to_f32(ri.make_inputs(w)) / 64.0)
    xb = np.ascontiguousarray(xa[::-1])
    want_a, want_b = xa, xb
    for _ in range(3):
        want_a, want_b = oracle.allreduce(want_a, w.G, threads=8), oracle.allreduce(want_b, w.G, threads=8)
    a = rar.AllReduce(w.P, w.G, w.n, 0, 1)
    b = rar.AllReduce(w.P, w.G, w.n, 0, 1)
    sa, sb = to_device(xa), to_device(xb)
    ba, bb = [t.clone() for t in sa], [t.clone() for t in sb]
    a.bind(ba), b.bind(bb)
    a.launch(), b.launch()                       # eager first: set-up stays out of the graph
    torch.cuda.synchronize()
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    print("[gpu] two default plans in one graph", flush=True)
    with torch.cuda.stream(main):
        with torch.cuda.graph(graph, stream=main):
            side.wait_stream(main)
            for _ in range(3):
                a.launch(main)
                b.launch(side)
            main.wait_stream(side)
    for rep in range(3):
        for t, s_ in zip(ba + bb, sa + sb):
            t.copy_(s_)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert a.status() == 0 and b.status() == 0
        assert_same_bits(to_host(ba, xa.dtype), want_a, f"plan a, replay {rep}")
        assert_same_bits(to_host(bb, xb.dtype), want_b, f"plan b, replay {rep}")
    a.close(), b.close()


def test_two_host_threads_with_their_own_plans():
    """Two host threads, each with its own plan, buffers and stream, launching at the same time:
    the library's bookkeeping of fused launches per device is shared between them (a lock, an
    event); every call of both threads must give the oracle's bits and no wait may time out."""
    import threading
    w = ri.WORKLOADS["c2"]
    xs = [ri.make_inputs(w), np.ascontiguousarray(ri.make_inputs(w)[::-1])]
    wants = [oracle.allreduce(x, w.G, threads=8) for x in xs]
    errors = []

    def worker(k):
        try:
            ar = rar.AllReduce(w.P, w.G, w.n, 0, MODES["auto" if k else "fused"])
            rar.rar_plan_set_wait_limit_us(ar.plan, 2_000_000)
            stream = torch.cuda.Stream()
            src = to_device(xs[k])
            bufs = [t.clone() for t in src]
            ar.bind(bufs)
            for it in range(100):
                with torch.cuda.stream(stream):
                    for b, s_ in zip(bufs, src):
                        b.copy_(s_, non_blocking=True)
                    ar.launch(stream)
                if it % 10 == 9:
                    assert ar.status(stream) == 0
                    assert_same_bits(to_host(bufs, xs[k].dtype), wants[k], f"thread {k}, call {it}")
            assert ar.status(stream) == 0
            ar.close()
        except Exception as e:                     # a thread's assertion must reach pytest
            errors.append((k, repr(e)))

    print("[gpu] two host threads", flush=True)
    threads = [threading.Thread(target=worker, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not any(t.is_alive() for t in threads), "a thread did not finish"
    assert not errors, errors


def test_plans_that_share_the_device_next_to_one_that_does_not():
    """A plan with the default concurrency between two plans that were told they share the device
    with one other: the exclusive launch waits for both sharing streams and the later sharing
    launches wait for it; all three keep giving the oracle's bits."""
    w = ri.WORKLOADS["c2"]
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    plans = [rar.AllReduce(w.P, w.G, w.n, 0, 1) for _ in range(3)]
    rar.rar_plan_set_concurrency(plans[0].plan, 2)
    rar.rar_plan_set_concurrency(plans[2].plan, 2)
    streams = [torch.cuda.Stream() for _ in range(3)]
    print("[gpu] sharing and exclusive plans", flush=True)
    for rep in range(5):
        bufs = [to_device(x) for _ in range(3)]
        for p, b in zip(plans, bufs):
            p.bind(b)
        torch.cuda.synchronize()
        order = (0, 2, 1) if rep % 2 else (1, 0, 2)
        for k in order:
            plans[k].launch(streams[k])
        torch.cuda.synchronize()
        for k in range(3):
            assert plans[k].status(streams[k]) == 0
            assert_same_bits(to_host(bufs[k], x.dtype), want, f"rep {rep}, plan {k}")
    for p in plans:
        p.close()


def test_measurement_aids():
    """rar_launch_floor, rar_barrier_only, rar_copy_probe and rar_read_probe do what the header says
    and leave the plan usable: the barrier-only kernel moves the flag counters like a real call."""
    w = ri.WORKLOADS["c2"]
    x = ri.make_inputs(w)
    want = oracle.allreduce(x, w.G, threads=8)
    ar = rar.AllReduce(w.P, w.G, w.n, 0, 1)
    bufs = to_device(x)
    ar.bind(bufs)
    print("[gpu] measurement aids", flush=True)
    ar.launch_floor()
    for B_s, C_s in ((0, 0), (3, 4096), (16, 8192)):
        ar.set_tuning(B_s, C_s)
        ar.barrier_only()
        ar.launch_floor()
    assert ar.status() == 0
    assert_same_bits(to_host(bufs, x.dtype), x, "the aids move no data")
    ar.set_tuning(0, 0)
    ar.launch()
    assert ar.status() == 0
    assert_same_bits(to_host(bufs, x.dtype), want, "a real call after barrier-only calls")
    ar.close()
    src = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros_like(src)
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    rar.rar_copy_probe(dst.data_ptr(), src.data_ptr(), src.numel(), st)
    rar.rar_read_probe(sink.data_ptr(), src.data_ptr(), src.numel(), st)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    with pytest.raises(rar.RarError):
        rar.rar_copy_probe(dst.data_ptr() + 8, src.data_ptr(), 1024, st)
    with pytest.raises(rar.RarError):
        rar.rar_read_probe(sink.data_ptr(), src.data_ptr(), 1000, st)
    rar.rar_read_probe(sink.data_ptr(), src.data_ptr(), 0, st)
    torch.cuda.synchronize()
