"""A CPU model of the fused kernel's step-barrier protocol (flags as trip counters, partial buffers
reused two trips later, chained calls, the hand-over for node counts that are not powers of two).

It models what the HIP kernel does per workgroup as a list of atomic operations and runs many
workgroups under a random scheduler with a residency limit and a dispatch policy, so that the
claims the design rests on can be checked on the CPU under interleavings the GPU would rarely show:

* every read of a partial buffer sees the value its writer produced for that very trip (a buffer
  place is never overwritten before its reader is done with it);
* with workgroups dispatched in index order per XCD, the waits end even if the grid is not
  resident at once; with an arbitrary dispatch order they need not.

It shares no code with the kernels (it cannot: it is Python) and is test infrastructure only.
"""
from __future__ import annotations

import random
from dataclasses import dataclass, field


def floor_log2(v: int) -> int:
    l = 0
    while (2 << l) <= v:
        l += 1
    return l


@dataclass
class Launch:
    N: int                 # nodes
    slots: int             # groups of N workgroups that exchange with each other (chunks x B_s)
    iters: int             # trips per workgroup and call
    calls: int = 1         # all-reduces in the launch (a chain if > 1)
    places: str = "auto"   # "unique" | "ring" | "sets" | "one" (a planted mistake: a single place) | "auto"

    def __post_init__(self):
        self.L = floor_log2(self.N)
        self.fold = self.N - (1 << self.L)
        if self.places == "auto":
            if self.calls > 1:
                self.places = "ring" if self.iters >= 2 else "sets"
            else:
                self.places = "ring" if self.iters >= 3 else "unique"

    def sits_out(self, r: int) -> bool:
        return r < 2 * self.fold and r % 2 == 0

    def folds_in(self, r: int) -> bool:
        return r < 2 * self.fold and r % 2 == 1

    def peer(self, r: int, l: int) -> int:
        number = r // 2 if r < 2 * self.fold else r - self.fold
        v = number ^ (1 << l)
        return 2 * v + 1 if v < self.fold else v + self.fold

    def place(self, call: int, it: int, T: int):
        """(buffer set, place inside the buffer) of the slice of trip T."""
        if self.places == "unique":
            return 0, it
        if self.places == "ring":
            return 0, T & 1
        if self.places == "sets":
            return call & 1, it
        if self.places == "one":
            return 0, 0
        raise ValueError(self.places)

    def program(self, r: int):
        """The operations of the workgroup of node r in one slot, in program order."""
        ops, T = [], 0
        idle, takes_in = self.sits_out(r), self.folds_in(r)
        for call in range(self.calls):
            for it in range(self.iters):
                where = self.place(call, it, T)
                t = T + 1
                if self.L:
                    if takes_in:
                        ops += [("wait", 0, r - 1, t), ("read", 0, r - 1, where, T)]
                    ops += [("write", 0, r, where, T), ("publish", 0, r, t)]
                if idle:
                    ops += [("wait", self.L, r + 1, t), ("read", self.L, r + 1, where, T)]
                else:
                    for l in range(self.L):
                        q = self.peer(r, l)
                        ops += [("wait", l, q, t), ("read", l, q, where, T)]
                        if l + 1 < self.L or takes_in:
                            ops += [("write", l + 1, r, where, T), ("publish", l + 1, r, t)]
                T += 1
        return ops


@dataclass
class Result:
    finished: bool
    stale_reads: list = field(default_factory=list)
    steps: int = 0


def run(launch: Launch, capacity: int | None = None, dispatch: str = "fifo", xcds: int = 8, seed: int = 0,
        base: int = 0, stragglers: float = 0.0, max_steps: int = 2_000_000) -> Result:
    """Run all workgroups of the launch.  capacity = workgroups resident at once on each XCD (None =
    all); dispatch = "fifo" (each XCD takes its workgroups in index order; workgroup i belongs to XCD
    i mod xcds) or "any" (a free place takes any waiting workgroup).  `base` = the counters' value
    before the launch (they are compared as signed 32-bit differences); `stragglers` = the share of
    workgroups that the scheduler picks a hundred times less often than the others."""
    rng = random.Random(seed)
    N = launch.N
    blocks = [(slot, r) for slot in range(launch.slots) for r in range(N)]     # index = slot * N + r, as in the kernel
    programs = [launch.program(r) for r in range(N)]
    pc = [0] * len(blocks)
    weight = [0.01 if rng.random() < stragglers else 1.0 for _ in blocks]
    flags, cells = {}, {}
    stale = []
    queues = [[i for i in range(len(blocks)) if i % xcds == x] for x in range(xcds)]
    if dispatch == "any":
        for q in queues:
            rng.shuffle(q)
    resident = [[] for _ in range(xcds)]
    cap = capacity if capacity is not None else len(blocks)

    def refill():
        for x in range(xcds):
            while queues[x] and len(resident[x]) < cap:
                resident[x].append(queues[x].pop(0))

    def signed(v):
        v &= 0xFFFFFFFF
        return v - (1 << 32) if v & 0x80000000 else v

    refill()
    steps = 0
    while steps < max_steps:
        ready = []
        for x in range(xcds):
            for i in resident[x]:
                slot, r = blocks[i]
                op = programs[r][pc[i]]
                if op[0] == "wait":
                    _, level, who, t = op
                    if signed(flags.get((slot, level, who), base) - (base + t)) < 0:
                        continue
                ready.append((x, i))
        if not ready:
            done = not any(resident) and not any(queues)
            return Result(done, stale, steps)
        x, i = rng.choices(ready, weights=[weight[j] for _, j in ready])[0] if stragglers else ready[rng.randrange(len(ready))]
        slot, r = blocks[i]
        op = programs[r][pc[i]]
        if op[0] == "publish":
            _, level, who, t = op
            flags[(slot, level, who)] = (base + t) & 0xFFFFFFFF
        elif op[0] == "write":
            _, level, who, where, T = op
            cells[(slot, level, who, where)] = T
        elif op[0] == "read":
            _, level, who, where, T = op
            got = cells.get((slot, level, who, where))
            if got != T:
                stale.append((slot, r, level, who, where, T, got))
        pc[i] += 1
        steps += 1
        if pc[i] == len(programs[r]):
            resident[x].remove(i)
            refill()
    return Result(False, stale, steps)
