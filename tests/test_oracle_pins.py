"""Pins for the CPU oracle: what the paper and the arithmetic fix, none of it taken from the
oracle itself.  A plausible mistake in oracle/ (a skipped rank, a wrong peer, a chain instead
of a tree, narrowing too early or too late, a wrong tie rule) fails at least one test here.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import exact_rational as ex
import oracle
import rar_inputs as ri
from oracle.tree import narrow as tree_narrow, widen as tree_widen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.txt")

SHAPES = [(1, 1), (2, 1), (2, 2), (4, 1), (4, 2), (4, 4), (8, 1), (8, 2), (8, 4), (8, 8),
          (16, 1), (16, 2), (16, 4), (32, 4), (64, 4), (64, 8), (128, 4),
          # N not a power of two (outside the paper, pairwise fold of the first 2r nodes)
          (3, 1), (6, 2), (12, 4), (5, 1), (20, 4), (7, 1), (28, 4), (24, 2), (44, 4), (100, 4)]


def bf16(values) -> np.ndarray:
    return ri.to_bf16_bits(np.asarray(values, dtype=np.float32))


def as_f32(a: np.ndarray) -> np.ndarray:
    return ri.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a


def same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    return a.dtype == b.dtype and a.shape == b.shape and a.tobytes() == b.tobytes()


# ---- worked examples (tests/golden/worked_examples.txt) -------------------------------------

def _golden_cases():
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, dtype, G, N, ins, want = [f.strip() for f in line.split("|")]
        yield pytest.param(dtype, int(G), int(N), [float(v) for v in ins.split()], float(want), id=name)


@pytest.mark.parametrize("dtype,G,N,ins,want", list(_golden_cases()))
def test_worked_examples(dtype, G, N, ins, want):
    assert len(ins) == G * N
    col = np.asarray(ins, dtype=np.float32).reshape(G * N, 1)
    x = bf16(col) if dtype == "bf16" else col
    w = bf16([want]) if dtype == "bf16" else np.asarray([want], dtype=np.float32)
    for out in (oracle.allreduce(x, G), oracle.tree_allreduce(x, G), ex.allreduce(x, G)):
        for p in range(G * N):
            assert same_bits(out[p], w), (p, out[p], w)


# ---- identity, closed forms ---------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_identity_single_rank(dtype):
    x = ri.random_inputs(1, 1, 1003, dtype)
    # include specials: zeros, subnormals, infinities
    if dtype == "bf16":
        x[0, :6] = [0x0000, 0x8000, 0x0001, 0x8001, 0x7F80, 0xFF80]
    else:
        x[0, :6] = np.array([0.0, -0.0, 1e-45, -1e-45, np.inf, -np.inf], dtype=np.float32)
    assert same_bits(oracle.allreduce(x, 1), x)
    assert same_bits(oracle.tree_allreduce(x, 1), x)


@pytest.mark.parametrize("P,G", SHAPES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_closed_forms(P, G, dtype):
    n = 3 * P + 5
    conv = (lambda a: bf16(a)) if dtype == "bf16" else (lambda a: np.asarray(a, dtype=np.float32))
    ones = conv(np.ones((P, n)))
    out = oracle.allreduce(ones, G)
    assert np.all(as_f32(out) == P)                     # P <= 256 is exact in bf16
    if P > 1:
        alt = conv(np.where(np.arange(P)[:, None] % 2 == 0, 1.0, -1.0) * np.ones((P, n)))
        assert np.all(as_f32(oracle.allreduce(alt, G)) == P % 2)   # +1 -1 +1 ... over P ranks
    # rank indicator: element j is 1 on rank j mod P only; every rank must be counted once.
    ind = conv((np.arange(n)[None, :] % P == np.arange(P)[:, None]).astype(np.float32))
    assert np.all(as_f32(oracle.allreduce(ind, G)) == 1)
    # weighted indicator: rank p contributes p+1 to its own elements, so a swapped or
    # double-counted rank shows up as the wrong weight.
    wind = conv((np.arange(n)[None, :] % P == np.arange(P)[:, None]) * (np.arange(P)[:, None] + 1.0))
    want = (np.arange(n) % P + 1).astype(np.float32)
    got = as_f32(oracle.allreduce(wind, G))
    assert np.all(got == want[None, :])


@pytest.mark.parametrize("P,G", SHAPES)
def test_integer_inputs_sum_exactly(P, G):
    n = 4099
    rng = np.random.default_rng(7 + P * 31 + G)
    r = max(1, min(8, 256 // P))                  # keep sum|x| within bf16's exact integers
    ints = rng.integers(-r, r + 1, size=(P, n))
    ok = np.abs(ints).sum(axis=0) <= 256          # every partial sum representable in bf16
    assert ok.mean() > 0.5
    want = ints.sum(axis=0).astype(np.float32)
    out = as_f32(oracle.allreduce(bf16(ints), G))
    assert np.all(out[:, ok] == want[None, ok])
    out32 = oracle.allreduce(ints.astype(np.float32) * 1000.0, G)   # |sum| << 2^24
    assert np.all(out32 == (ints.sum(axis=0) * 1000.0).astype(np.float32)[None, :])


def test_c1_integer_variant_is_exact():
    w = ri.WORKLOADS["c1_int"]
    x = ri.make_inputs(w)
    want = ri.bf16_bits_to_f32(x).astype(np.int64).sum(axis=0)
    assert np.abs(want).max() <= 64
    out = as_f32(oracle.allreduce(x, w.G))
    assert np.all(out == want[None, :].astype(np.float32))


# ---- two ranks reduce to a library routine ---------------------------------------------------

@pytest.mark.parametrize("G", [1, 2])
def test_two_ranks_equal_torch_cpu_sum(G):
    rng = np.random.default_rng(11)
    n = 1 << 16
    bits = rng.integers(0, 1 << 16, size=(2, n), dtype=np.uint16)
    finite = ((bits & 0x7F80) != 0x7F80).all(axis=0)
    bits = bits[:, finite]
    a = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)
    want = (a[0].float() + a[1].float()).to(torch.bfloat16)       # library add + library cast
    out = oracle.allreduce(bits, G)
    got = torch.from_numpy(out.view(np.int16)).view(torch.bfloat16)
    notnan = ~torch.isnan(want)
    assert torch.equal(got[0].view(torch.int16)[notnan], want.view(torch.int16)[notnan])
    assert torch.equal(torch.isnan(got[0]), torch.isnan(want))
    assert same_bits(out[0], out[1])
    x32 = rng.standard_normal((2, n)).astype(np.float32) * np.float32(1e3)
    assert same_bits(oracle.allreduce(x32, G)[1], x32[0] + x32[1])


def test_step_combine_equals_torch_cpu_sum():
    rng = np.random.default_rng(12)
    n, chunk = 1000, 3
    dst = ri.to_bf16_bits(rng.standard_normal(5 * n).astype(np.float32))
    src = ri.to_bf16_bits(rng.standard_normal(5 * n).astype(np.float32))
    keep = dst.copy()
    oracle.step_combine(dst, src, chunk, n)
    td = torch.from_numpy(keep.view(np.int16)).view(torch.bfloat16)
    ts = torch.from_numpy(src.view(np.int16)).view(torch.bfloat16)
    want = (td.float() + ts.float()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    lo, hi = chunk * n, chunk * n + n
    assert same_bits(dst[lo:hi], want[lo:hi])
    assert same_bits(dst[:lo], keep[:lo]) and same_bits(dst[hi:], keep[hi:])
    d32 = rng.standard_normal(5 * n).astype(np.float32)
    s32 = rng.standard_normal(5 * n).astype(np.float32)
    k32 = d32.copy()
    oracle.step_combine(d32, s32, chunk, n)
    assert same_bits(d32[lo:hi], (k32 + s32)[lo:hi]) and same_bits(d32[:lo], k32[:lo])


def test_narrowing_equals_torch_cast_on_all_upper_halves():
    # every bf16 neighbourhood: all 2^16 upper halves x lower halves around the tie point
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x1234, 0xC000], dtype=np.uint32)
    u = (hi[:, None] | lows[None, :]).reshape(-1)
    f = u.view(np.float32)
    want = ri.to_bf16_bits(f)
    got = tree_narrow(f, np.uint16)
    notnan = ~np.isnan(f)
    assert np.array_equal(got[notnan], want[notnan])
    # and the C oracle's narrowing, reached through a sum whose second operand is zero in a
    # lower precision: x = hi part, y = low part as its own float when exactly representable
    rng = np.random.default_rng(5)
    a = rng.integers(0, 1 << 16, size=200000, dtype=np.uint16)
    b = rng.integers(0, 1 << 16, size=200000, dtype=np.uint16)
    fin = ((a & 0x7F80) != 0x7F80) & ((b & 0x7F80) != 0x7F80)
    a, b = a[fin], b[fin]
    with np.errstate(all="ignore"):
        s = tree_widen(a) + tree_widen(b)
    d = a.copy()
    oracle.step_combine(d, b, 0, d.size)
    ok = ~np.isnan(s)
    assert np.array_equal(d[ok], ri.to_bf16_bits(s)[ok])


# ---- brute force with exact rationals -------------------------------------------------------

def _adversarial(rng, P, n, dtype):
    """Mixed magnitudes, half-ulp ties, subnormals, signed zeros."""
    if dtype == "bf16":
        pool = np.concatenate([
            bf16([256, 1, 3, 128, 0.5, 257, 255, -256, -1, 1.5, 2 ** -126, 2 ** -133, -2 ** -133,
                  3.0e38, -3.0e38, 1e-3, 0.0, -0.0, 384, 2, 6, 10, 1 / 3]),
            rng.integers(0, 1 << 16, size=64, dtype=np.uint16)])
        pool = pool[(pool & 0x7F80) != 0x7F80]
        return pool[rng.integers(0, pool.size, size=(P, n))]
    pool = np.concatenate([
        np.array([2 ** 24, 1, 3, 2 ** 23 + 0.5, 0.5, -2 ** 24, 1e-45, -1e-45, 1e-40, 3e38, -3e38,
                  0.0, -0.0, 1 / 3, 2 ** -126, 16777217 * 2.0], dtype=np.float32),
        (rng.standard_normal(32) * 10.0 ** rng.integers(-3, 4, 32)).astype(np.float32)])
    return pool[rng.integers(0, pool.size, size=(P, n))]


@pytest.mark.parametrize("P,G", [(1, 1), (2, 1), (2, 2), (4, 1), (4, 2), (4, 4), (8, 1), (8, 2),
                                 (8, 4), (16, 1), (16, 2), (16, 4), (16, 8),
                                 (3, 1), (6, 2), (5, 1), (6, 1), (7, 1), (12, 4), (9, 1), (11, 1), (13, 1), (24, 2)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_brute_force_exact_rational(P, G, dtype):
    rng = np.random.default_rng(100 * P + G)
    n = 48
    x = _adversarial(rng, P, n, dtype)
    want = ex.allreduce(x, G)
    got = oracle.allreduce(x, G)
    tree = oracle.tree_allreduce(x, G)
    wf, gf, tf = as_f32(want), as_f32(got), as_f32(tree)
    nan = np.isnan(wf)
    assert np.array_equal(np.isnan(gf), nan) and np.array_equal(np.isnan(tf), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(tree[~nan], want[~nan])


# ---- structure ------------------------------------------------------------------------------

@pytest.mark.parametrize("P,G", SHAPES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_two_formulations_agree_and_ranks_identical(P, G, dtype):
    for n in (1, 7, 8 * G, 8 * G + 1, 1021):
        x = ri.random_inputs(1000 + P + n, P, n, dtype)
        a = oracle.allreduce(x, G)
        b = oracle.tree_allreduce(x, G)
        assert same_bits(a, b)
        for p in range(1, P):
            assert same_bits(a[p], a[0])
        assert same_bits(oracle.allreduce(x, G, threads=4), a)


def test_rejects_bad_shapes():
    x = ri.random_inputs(1, 12, 16, "bf16")
    with pytest.raises(ValueError):
        oracle.allreduce(x, 5)          # G does not divide P
    with pytest.raises(TypeError):
        oracle.allreduce(x.astype(np.float64), 4)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_metamorphic(dtype):
    P, G, n = 32, 4, 2048
    N = P // G
    x = ri.random_inputs(77, P, n, dtype)
    base = oracle.allreduce(x, G)
    f = as_f32(x)
    conv = (lambda a: ri.to_bf16_bits(a)) if dtype == "bf16" else (lambda a: a.astype(np.float32))
    # power-of-two scaling and negation commute with every rounding (no over/underflow here)
    for k in (-6, 5):
        scaled = oracle.allreduce(conv(f * np.float32(2.0 ** k)), G)
        assert np.array_equal(as_f32(scaled), as_f32(base) * np.float32(2.0 ** k))
    assert np.array_equal(as_f32(oracle.allreduce(conv(-f), G)), -as_f32(base))
    # relabelling nodes r_n -> r_n XOR m swaps subtrees of the balanced tree: same bits
    xn = x.reshape(N, G, n)
    for m in (1, 2, 5, 7):
        perm = xn[np.arange(N) ^ m].reshape(P, n)
        assert same_bits(oracle.allreduce(perm, G), base)
    # a relabelling that is not of that form regroups the tree and must be able to change bits:
    # this shows the inputs are order-sensitive, i.e. that these tests can see a wrong order.
    rot = xn[(np.arange(N) + 1) % N].reshape(P, n)
    assert not same_bits(oracle.allreduce(rot, G), base)
    # same for the order inside a node when the message is fp32 (binary32 adds round each time);
    # for bf16 messages the in-node accumulation of four values rarely rounds in binary32.
    if dtype == "f32":
        swapped = xn[:, ::-1, :].reshape(P, n)
        assert not same_bits(oracle.allreduce(swapped, G), base)


# ---- distance from the plain sum -------------------------------------------------------------

@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4"])
def test_error_bound_against_naive_fp64(name):
    w = ri.WORKLOADS[name]
    n = min(w.n, 1 << 15)
    x = ri.make_inputs(w, n=n)
    out = as_f32(oracle.allreduce(x, w.G, threads=4))[0].astype(np.float64)
    ref, mag = oracle.naive_sum_f64(x)
    L = int(np.log2(w.N))
    d = 1 + L                      # narrowings on an element's path: one per node sum + one per step
    u = 2.0 ** -8                  # unit roundoff of bf16 (8 significant bits)
    slack = (1 + u) ** d - 1 + w.G * 2.0 ** -24     # + the binary32 accumulation inside a node
    # always: |out - ref| <= slack * sum|x|
    assert np.all(np.abs(out - ref) <= slack * mag + 1e-300)
    # "not near cancellation" = |ref| >= sum|x| / 2.  There the bound above gives a relative
    # error <= 2*slack ~ 2*d*2^-8 = d*2^-7 <= log2(P)*2^-7 (d = 1 + log2 N <= log2 G + log2 N).
    away = np.abs(ref) >= mag / 2
    assert away.any()
    rel = np.abs(out[away] - ref[away]) / np.abs(ref[away])
    assert rel.max() <= 2.0 ** -7 * np.log2(w.P)
    # observed errors are far inside the worst case even at |ref| >= sum|x| / 4
    wider = np.abs(ref) >= mag / 4
    rel4 = np.abs(out[wider] - ref[wider]) / np.abs(ref[wider])
    assert rel4.max() <= 2.0 ** -7 * np.log2(w.P)


@pytest.mark.parametrize("P,G", [(8, 4), (64, 4), (64, 8), (128, 4)])
def test_error_bound_fp32(P, G):
    x = ri.random_inputs(31 + P, P, 1 << 14, "f32")
    out = oracle.allreduce(x, G)[0].astype(np.float64)
    ref, mag = oracle.naive_sum_f64(x)
    d = (G - 1) + int(np.log2(P // G))
    u = 2.0 ** -24
    assert np.all(np.abs(out - ref) <= ((1 + u) ** d - 1) * mag * (1 + 1e-9) + 1e-300)
    # worst case 4*d*2^-24 at |ref| >= sum|x|/4 can exceed 2^-20 for d > 4; observed errors do not
    sel = np.abs(ref) >= mag / 4
    assert sel.any()
    assert (np.abs(out[sel] - ref[sel]) / np.abs(ref[sel])).max() <= 2.0 ** -20
    # no cancellation at all (same-sign inputs): d * 2^-24 <= 2^-20 is guaranteed for d <= 16
    xp = np.abs(x)
    outp = oracle.allreduce(xp, G)[0].astype(np.float64)
    refp, _ = oracle.naive_sum_f64(xp)
    assert (np.abs(outp - refp) / refp).max() <= 2.0 ** -20


def test_subnormal_arithmetic_is_gradual():
    # 2^-133 is a bf16 subnormal: two of them must add to 2^-132, not flush to zero
    t = bf16([2.0 ** -133])
    x = np.repeat(t, 4).reshape(4, 1)
    assert same_bits(oracle.allreduce(x, 2)[0], bf16([2.0 ** -131]))
    assert same_bits(oracle.tree_allreduce(x, 2)[0], bf16([2.0 ** -131]))
    y = np.full((2, 1), 1e-45, dtype=np.float32)
    assert oracle.allreduce(y, 1)[0, 0] == np.float32(2.8e-45)
