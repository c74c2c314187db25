"""The step-barrier protocol of the fused kernel on a CPU model (tests/protocol_model.py): buffer
reuse is hazard-free under random interleavings, for plain launches, chains of calls and node
counts that are not powers of two; planted mistakes are caught; and what residency and dispatch
order mean for the waits."""
import pytest

from protocol_model import Launch, run

SHAPES = [(2, 1), (2, 3), (4, 2), (4, 5), (8, 7), (16, 3), (3, 4), (5, 5), (6, 3), (7, 2), (12, 3)]


@pytest.mark.parametrize("N,iters", SHAPES)
def test_plain_launch_reads_what_was_written_for_the_trip(N, iters):
    for seed in range(20):
        res = run(Launch(N, slots=3, iters=iters), seed=seed, stragglers=0.3 * (seed % 2))
        assert res.finished and not res.stale_reads, (seed, res.stale_reads[:3])


@pytest.mark.parametrize("calls", [2, 3, 5])
@pytest.mark.parametrize("N,iters", SHAPES)
def test_chain_reads_what_was_written_for_the_trip(N, iters, calls):
    """Chained calls: two sets of buffers when a call is a single trip, else two places in one."""
    for seed in range(10):
        res = run(Launch(N, slots=2, iters=iters, calls=calls), seed=seed, stragglers=0.3 * (seed % 2))
        assert res.finished and not res.stale_reads, (seed, res.stale_reads[:3])
    res = run(Launch(N, slots=2, iters=iters, calls=calls, places="sets"), seed=99)   # the sets also serve longer calls
    assert res.finished and not res.stale_reads


def test_a_single_place_is_caught():
    """The planted mistake: reusing ONE place trip after trip.  Some interleaving must overwrite a
    slice before its reader has read it, and the model must see that."""
    caught = 0
    for seed in range(40):
        res = run(Launch(4, slots=1, iters=4, places="one"), seed=seed, stragglers=0.3)
        caught += bool(res.stale_reads)
    assert caught > 0
    for N in (2, 4, 8, 6):      # a chain of single-trip calls on one set of buffers
        caught = 0
        for seed in range(40):
            res = run(Launch(N, slots=1, iters=1, calls=4, places="unique"), seed=seed, stragglers=0.3)
            caught += bool(res.stale_reads)
        assert caught > 0, N


def test_reuse_distance_of_two_trips_is_what_matters():
    """A place of its own per trip of a call is reused `iters` trips later in a chain: safe from two
    trips per call on (it is then the alternation between two places), unsafe with one."""
    for iters in (2, 3):
        for seed in range(30):
            assert not run(Launch(8, slots=1, iters=iters, calls=3, places="unique"), seed=seed, stragglers=0.3).stale_reads
    assert any(run(Launch(8, slots=1, iters=1, calls=4, places="unique"), seed=seed, stragglers=0.3).stale_reads
               for seed in range(40))


@pytest.mark.parametrize("base", [0, 7, 0xFFFFFFF0, 0x7FFFFFFA])
def test_counters_wrap(base):
    """The counters only grow and are compared as signed differences: any starting value works."""
    for seed in range(5):
        res = run(Launch(8, slots=2, iters=5, calls=4), seed=seed, base=base)
        assert res.finished and not res.stale_reads


@pytest.mark.parametrize("N,iters", [(2, 1), (4, 5), (16, 5), (32, 2), (6, 3)])
def test_in_order_dispatch_needs_no_full_residency(N, iters):
    """Workgroups dealt to the XCDs round-robin and started in index order on each: the waits end
    with any number of resident workgroups per XCD that holds one group's share (N / 8 of them),
    because the lowest unfinished group always has all its members at the head of the queues."""
    least = -(-N // 8)
    for capacity in (least, least + 1, least + 2, 7 * least):
        for seed in range(5):
            res = run(Launch(N, slots=9, iters=iters), capacity=capacity, dispatch="fifo", seed=seed)
            assert res.finished and not res.stale_reads, (capacity, seed)


def test_arbitrary_dispatch_order_can_block_without_full_residency():
    """With no promise about dispatch order, a grid that is not resident at once can block: resident
    workgroups wait for peers that cannot start.  (That is why the library sizes every fused grid
    to be resident at once, with a margin, and bounds every wait.)  Fully resident, any order is fine."""
    blocked = 0
    for seed in range(30):
        res = run(Launch(16, slots=9, iters=2), capacity=3, dispatch="any", seed=seed)
        blocked += not res.finished
        assert not res.stale_reads
    assert blocked > 0
    for seed in range(10):
        assert run(Launch(16, slots=9, iters=2), capacity=None, dispatch="any", seed=seed).finished
