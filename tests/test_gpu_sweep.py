"""GPU parity on every point of the message-size sweep: 14 sizes (8 KiB .. 64 MiB per rank) x 6
(P, G) x 2 types = 168 points, N(0,1) values, each compared bit for bit with the CPU oracle.

Up to 4 MiB per rank the whole result is compared (flag exchange; data+flag exchange where the
planner offers it; the mode a plan picks by itself is checked to be one of the two).  Above that
the oracle checks a sample of columns: a stride through the message, both ends, and the
neighbourhood of every chunk border (each element is reduced independently of the others, so the
oracle on a subset of columns is the oracle's value there); all ranks must also hold the same
bits.  One size per (P, G, type) also runs the stepwise path.
"""
import numpy as np
import pytest
import torch

import oracle
import rar_inputs as ri
from gpu_util import assert_same_bits

pytestmark = pytest.mark.gpu

rar = pytest.importorskip("paper_2511_09557_amd") if torch.cuda.is_available() else None

DT = {"bf16": 0, "f32": 1}
SWEEP = [(8, 4), (16, 4), (32, 4), (64, 4), (128, 4), (64, 8)]
SIZES = [1 << lg for lg in range(13, 27)]
FULL_LIMIT = 4 << 20
STEPWISE_SIZE = 64 << 10


def host_bits(t: torch.Tensor, dtype: str) -> np.ndarray:
    h = t.cpu()
    return h.view(torch.int16).numpy().view(np.uint16) if dtype == "bf16" else h.numpy()


def run_mode(whole_src: torch.Tensor, P: int, G: int, n: int, dtype: str, mode: int):
    work = whole_src.clone()
    ar = rar.AllReduce(P, G, n, DT[dtype], mode)
    ar.bind([work[p] for p in range(P)])
    ar.launch()
    assert ar.status() == 0
    tuning = ar.tuning()
    ar.close()
    return work, tuning


@pytest.mark.parametrize("nbytes", SIZES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("P,G", SWEEP)
def test_sweep_point(P, G, dtype, nbytes):
    tdt, es = (torch.bfloat16, 2) if dtype == "bf16" else (torch.float32, 4)
    n = nbytes // es
    print(f"[gpu] sweep point P={P} G={G} {dtype} {nbytes} B", flush=True)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(ri.SEED_BASE + 400 + (nbytes.bit_length() - 1) * 1000 + P * 10 + G + (0 if dtype == "bf16" else 5))
    whole = torch.empty(P, n, device="cuda:0", dtype=tdt)
    for p in range(P):
        whole[p] = torch.randn(n, device="cuda:0", generator=gen).to(tdt)

    plan = rar.rar_plan(P, G, n, DT[dtype])
    try:
        rar.rar_plan_set_mode(plan, rar.RAR_MODE_FUSED_PACKED)
        packed_offered = True
    except rar.RarError as e:
        assert e.status == -4
        packed_offered = False
    rar.rar_plan_set_mode(plan, rar.RAR_MODE_AUTO)
    auto = rar.rar_plan_effective_mode(plan)
    rar.rar_plan_free(plan)
    assert auto == rar.RAR_MODE_FUSED or (auto == rar.RAR_MODE_FUSED_PACKED and packed_offered)

    modes = [("fused", rar.RAR_MODE_FUSED)]
    if packed_offered:
        modes.append(("packed", rar.RAR_MODE_FUSED_PACKED))
    if nbytes == STEPWISE_SIZE:
        modes.append(("stepwise", rar.RAR_MODE_STEPWISE))

    if nbytes <= FULL_LIMIT:
        want = oracle.allreduce(np.ascontiguousarray(host_bits(whole, dtype)), G, threads=8)
        for name, mode in modes:
            work, tuning = run_mode(whole, P, G, n, dtype, mode)
            assert_same_bits(np.ascontiguousarray(host_bits(work, dtype)), want, f"{name} {tuning}")
            del work
        return

    q = n // G
    cols = np.unique(np.concatenate([np.arange(0, n, 8191), np.arange(0, 2048), np.arange(n - 2048, n)] +
                                    [np.arange(c * q - 256, c * q + 256) for c in range(1, G)]))
    ci = torch.from_numpy(cols).to("cuda:0")
    want = oracle.allreduce(np.ascontiguousarray(host_bits(whole[:, ci], dtype)), G, threads=8)
    # in place on the inputs (they were sampled above): the largest point holds 8 GiB of messages
    ar = rar.AllReduce(P, G, n, DT[dtype], rar.RAR_MODE_FUSED)
    ar.bind([whole[p] for p in range(P)])
    ar.launch()
    assert ar.status() == 0
    tuning = ar.tuning()
    ar.close()
    assert_same_bits(np.ascontiguousarray(host_bits(whole[:, ci], dtype)), want, f"fused {tuning}")
    first = whole[0].view(torch.int16 if dtype == "bf16" else torch.int32)
    keep = ~torch.isnan(whole[0])
    for p in range(1, P):
        assert torch.equal(whole[p].view(first.dtype)[keep], first[keep]), f"rank {p} differs from rank 0"
    del whole
    torch.cuda.empty_cache()
