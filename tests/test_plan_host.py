"""Host-only checks: the library loads, exports every symbol the header declares, and the
planner's integer logic follows Algorithm 1 (peer rule, step count, chunk partition)."""
import os
import re

import pytest

import paper_2511_09557_amd as rar
from paper_2511_09557_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "rar.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(rar_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(binding.lib, name), f"{name} declared in rar.h but not exported"
    assert declared == set(binding.EXPORTS)


def test_version_and_strerror():
    assert rar.rar_version() >= 100
    for code in range(0, -11, -1):
        assert rar.rar_strerror(code) != "unknown status"
    assert rar.rar_strerror(-99) == "unknown status"


@pytest.mark.parametrize("P,G,status", [(0, 1, -1), (8, 0, -1), (10, 4, -2), (20, 8, -2), (256, 4, -4), (8, 16, -2)])
def test_plan_rejects(P, G, status):
    with pytest.raises(rar.RarError) as e:
        rar.rar_plan(P, G, 1024, 0)
    assert e.value.status == status


def test_plan_rejects_other():
    with pytest.raises(rar.RarError) as e:
        rar.rar_plan(8, 4, 0, 0)
    assert e.value.status == -1
    with pytest.raises(rar.RarError) as e:
        rar.rar_plan(8, 4, 16, 5)
    assert e.value.status == -3
    with pytest.raises(rar.RarError) as e:
        rar.rar_plan(8, 4, 1 << 40, 0)
    assert e.value.status == -4


def test_peer_rule_exhaustive():
    for G in (1, 2, 3, 4, 8):
        for N in (1, 2, 4, 8, 16, 32, 64, 128):
            P = G * N
            if P > 128:
                continue
            plan = rar.rar_plan(P, G, 4096, 0)
            L = rar.rar_plan_steps(plan)
            assert (1 << L) == N and rar.rar_plan_nodes(plan) == N and rar.rar_plan_ranks(plan) == P
            for p in range(P):
                r_n, r_g = divmod(p, G)
                reached = {r_n}
                for l in range(L):
                    q = rar.rar_plan_peer(plan, p, l)
                    assert q == (r_n ^ (1 << l)) * G + r_g
                    assert q % G == r_g                       # same local id across nodes
                    assert rar.rar_plan_peer(plan, q, l) == p  # the exchange is mutual
                    reached |= {m ^ (1 << l) for m in reached}
                assert reached == set(range(N))               # after L steps every node contributed
                with pytest.raises(rar.RarError):
                    rar.rar_plan_peer(plan, p, L)
            with pytest.raises(rar.RarError):
                rar.rar_plan_peer(plan, P, 0)
            rar.rar_plan_free(plan)


def test_peer_rule_any_node_count():
    """N = 2^L + r (outside the paper): r even nodes hand over and sit out, the rest run the XOR
    rule on their renumbering, and every node's contribution reaches every node that takes part."""
    for G in (1, 3, 4):
        for N in range(1, 33):
            P = G * N
            if P > 128:
                continue
            plan = rar.rar_plan(P, G, 4096, 0)
            L = rar.rar_plan_steps(plan)
            r = N - (1 << L)
            assert 0 <= r < (1 << L) and rar.rar_plan_nodes(plan) == N
            idle = {m for m in range(2 * r) if m % 2 == 0}
            for g in range(G):
                holds = {m: {m} for m in range(N)}        # node -> nodes whose data it has summed
                for m in range(N):
                    q = rar.rar_plan_fold_partner(plan, m * G + g)
                    assert q % G == g and rar.rar_plan_fold_partner(plan, q) == m * G + g
                    if m in idle:
                        assert q == (m + 1) * G + g
                        holds[m + 1] = holds[m + 1] | {m}
                    elif m < 2 * r:
                        assert q == (m - 1) * G + g
                    else:
                        assert q == m * G + g
                for l in range(L):
                    nxt = dict(holds)
                    for m in range(N):
                        q = rar.rar_plan_peer(plan, m * G + g, l)
                        if m in idle:
                            assert q == m * G + g
                            continue
                        assert q % G == g and q // G not in idle and q // G != m
                        assert rar.rar_plan_peer(plan, q, l) == m * G + g
                        assert not (holds[m] & holds[q // G])   # nothing is counted twice
                        nxt[m] = holds[m] | holds[q // G]
                    holds = nxt
                for m in range(N):
                    if m not in idle:
                        assert holds[m] == set(range(N))
            rar.rar_plan_set_mode(plan, 2)                 # the data+flag mode covers any N
            rar.rar_plan_free(plan)


@pytest.mark.parametrize("dtype,per_vec", [(0, 8), (1, 4)])
def test_chunk_partition(dtype, per_vec):
    for G in (1, 2, 3, 4, 8):
        for n in (1, 2, 7, 8, 9, 31, 32, 33, 1000, 4096, 65536, 65537, 1048576):
            plan = rar.rar_plan(G, G, n, dtype)
            pos = 0
            for c in range(G):
                off, length = rar.rar_plan_chunk(plan, c)
                assert off == pos and off % per_vec == 0 or length == 0
                pos = off + length
            assert pos == n
            full = rar.rar_plan_chunk(plan, 0)[1]
            assert full == min(n, -(-(-(-n // G)) // per_vec) * per_vec)
            with pytest.raises(rar.RarError):
                rar.rar_plan_chunk(plan, G)
            rar.rar_plan_free(plan)


def test_scratch_size_and_tuning():
    plan = rar.rar_plan(64, 4, 1048576, 0)
    # S_0..S_L for 64 ranks of 512 KiB each, plus flags and header
    assert rar.rar_plan_scratch_bytes(plan) >= 5 * 64 * 512 * 1024
    assert rar.rar_plan_scratch_bytes(plan) <= 5 * 64 * 512 * 1024 + (1 << 20)
    rar.rar_plan_set_tuning(plan, 8, 16384)
    assert rar.rar_plan_get_tuning(plan) == (8, 16384)
    rar.rar_plan_set_tuning(plan, 0, 0)
    for bad in [(-1, 0), (257, 0), (4, 1000), (4, 65536)]:
        with pytest.raises(rar.RarError) as e:
            rar.rar_plan_set_tuning(plan, *bad)
        assert e.value.status == -9
    rar.rar_plan_set_mode(plan, 0)
    assert rar.rar_plan_get_mode(plan) == 0
    with pytest.raises(rar.RarError):
        rar.rar_plan_set_mode(plan, 4)
    rar.rar_plan_set_mode(plan, 3)                  # automatic choice: 512 KiB chunks run the flag exchange
    assert rar.rar_plan_get_mode(plan) == 3 and rar.rar_plan_effective_mode(plan) == 1
    with pytest.raises(rar.RarError) as e:          # 512 KiB chunks: too large for the packed mode
        rar.rar_plan_set_mode(plan, 2)
    assert e.value.status == -4
    small = rar.rar_plan(32, 4, 524288, 0)
    rar.rar_plan_set_mode(small, 2)
    # S_0..S_3 (4 x 32 x 256 KiB) + data+flag buffers (3 x 32 x 512 KiB) + flags + header
    assert rar.rar_plan_scratch_bytes(small) >= (4 + 6) * 32 * 256 * 1024
    rar.rar_plan_free(small)
    with pytest.raises(rar.RarError):
        rar.rar_plan_set_scratch(plan, 0, 1 << 30)
    rar.rar_plan_free(plan)


def test_concurrency_halves_the_grid():
    plan = rar.rar_plan(64, 4, 1 << 24, 0)            # a long message: the built-in grid is 4 workgroups per compute unit
    full = rar.rar_plan_get_tuning(plan)
    rar.rar_plan_set_concurrency(plan, 2)
    half = rar.rar_plan_get_tuning(plan)
    assert half[0] * 2 == full[0] and half[1] == full[1]
    for bad in (0, 9, -1):
        with pytest.raises(rar.RarError):
            rar.rar_plan_set_concurrency(plan, bad)
    rar.rar_plan_free(plan)


def test_scratch_layout():
    plan = rar.rar_plan(16, 4, 131072, 0)
    f_off, f_bytes, p_off, p_bytes = rar.rar_plan_scratch_layout(plan)
    total = rar.rar_plan_scratch_bytes(plan)
    L = rar.rar_plan_steps(plan)
    assert f_off == 256 and f_bytes >= (L + 1) * 16 * 256 * 4
    assert p_off >= f_off + f_bytes + (L + 1) * 16 * 65536 and p_off + p_bytes == total
    assert p_bytes >= L * 16 * 2 * 65536            # twice a chunk per (step, rank)
    rar.rar_plan_free(plan)
    big = rar.rar_plan(64, 4, 1048576, 0)           # 512 KiB chunks: no data+flag buffers
    assert rar.rar_plan_scratch_layout(big)[2:] == (0, 0)
    rar.rar_plan_free(big)


def test_automatic_mode():
    """A new plan is in the automatic mode: the data+flag exchange while all ranks together
    exchange at most 1 MiB per step (and there is a step at all), the flag exchange otherwise."""
    for P, G, nbytes, want in ((8, 4, 128 << 10, 2), (16, 4, 256 << 10, 2), (32, 4, 1 << 20, 1), (64, 4, 2 << 20, 1),
                               (64, 4, 64 << 10, 2), (64, 4, 128 << 10, 1), (12, 4, 64 << 10, 2), (4, 4, 64 << 10, 1),
                               (20, 4, 1 << 20, 1),
                               (64, 8, 128 << 10, 2), (8, 1, 128 << 10, 2), (8, 1, 256 << 10, 1)):
        plan = rar.rar_plan(P, G, nbytes // 2, 0)
        assert rar.rar_plan_get_mode(plan) == 3
        assert rar.rar_plan_effective_mode(plan) == want, (P, G, nbytes)
        rar.rar_plan_set_mode(plan, 0)
        assert rar.rar_plan_effective_mode(plan) == 0
        rar.rar_plan_free(plan)


def test_no_device_gives_an_error_not_a_crash():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    plan = rar.rar_plan(8, 4, 1024, 0)
    rar.rar_plan_set_scratch(plan, 0x1000, 1 << 30)   # never dereferenced on the host
    with pytest.raises(rar.RarError) as e:
        rar.rar_allreduce([0x100000 + 4096 * i for i in range(8)], plan)
    assert e.value.status == -7
    rar.rar_plan_free(plan)


def test_new_entry_points_without_a_device():
    """The chained, static-scratch and probe entry points check their arguments on the host and then
    fail with RAR_ERR_HIP where there is no device; nothing crashes."""
    import ctypes
    import torch
    plan = rar.rar_plan(8, 4, 1024, 0)
    ptrs = [0x100000 + 4096 * i for i in range(8)]
    arr = (ctypes.c_void_p * 8)(*ptrs)
    rar.rar_plan_set_scratch(plan, 0x1000, 1 << 30)
    for K in (0, -3, (1 << 16) + 1):
        assert binding.lib.rar_allreduce_chain(arr, plan, K, None) == -1
    assert binding.lib.rar_allreduce_chain(None, plan, 2, None) == -1
    assert binding.lib.rar_allreduce_static(None, plan, None) == -1
    assert binding.lib.rar_read_probe(None, 0x1000, 1024, None) == -1
    assert binding.lib.rar_read_probe(0x1000, 0x2000, 1000, None) == -6
    big = rar.rar_plan(64, 4, 1048576, 0)
    assert rar.rar_plan_static_bytes(big) > rar.RAR_STATIC_SCRATCH_BYTES
    assert binding.lib.rar_allreduce_static((ctypes.c_void_p * 64)(*[0x100000 + 0x1000 * i for i in range(64)]), big, None) == -4
    rar.rar_plan_free(big)
    assert rar.rar_plan_static_bytes(plan) <= rar.rar_plan_scratch_bytes(plan)
    if not torch.cuda.is_available():
        assert binding.lib.rar_allreduce_chain(arr, plan, 2, None) == -7
        assert binding.lib.rar_allreduce_static(arr, plan, None) == -7
        assert binding.lib.rar_launch_floor(plan, None) == -7
    rar.rar_plan_free(plan)


def test_no_grid_beyond_four_workgroups_per_compute_unit():
    """Whatever B_s is asked for, P * B_s stays within four workgroups per compute unit (256 compute
    units until a device has been seen), also for the tuning of a chained launch's plan."""
    for P, G, n in ((8, 4, 1 << 22), (16, 4, 1 << 22), (64, 4, 1 << 20), (128, 4, 1 << 21), (64, 8, 1 << 22), (128, 1, 1 << 20)):
        plan = rar.rar_plan(P, G, n, 0)
        for C_s in (4096, 8192, 16384, 32768, 0):
            for B_s in (0, 1, 7, 64, 256):
                rar.rar_plan_set_tuning(plan, B_s, C_s)
                got_B, got_C = rar.rar_plan_get_tuning(plan)
                assert P * got_B <= 4 * 256 or got_B == 1, (P, G, n, B_s, C_s, got_B)
                assert C_s == 0 or got_C == C_s
        rar.rar_plan_free(plan)


def test_second_buffer_set_for_chained_calls():
    """Plans with chunks of at most 256 KiB carry a second set of partial and data+flag buffers (the
    odd calls of a chain); longer chunks do not."""
    small = rar.rar_plan(16, 4, 131072, 0)          # 64 KiB chunks
    L = rar.rar_plan_steps(small)
    chunk = 65536
    first_set = 256 + (L + 1) * 16 * 1024 + (L + 1) * 16 * chunk
    assert rar.rar_plan_static_bytes(small) == first_set
    assert rar.rar_plan_scratch_bytes(small) >= 2 * (L + 1) * 16 * chunk + 2 * L * 16 * 2 * chunk
    rar.rar_plan_free(small)
    big = rar.rar_plan(64, 4, 1048576, 0)
    assert rar.rar_plan_scratch_bytes(big) == rar.rar_plan_static_bytes(big)
    rar.rar_plan_free(big)
