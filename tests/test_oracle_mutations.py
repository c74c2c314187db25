"""Do the pins bite?  Each case plants one plausible mistake in a copy of the C oracle (on the
CPU, in a temporary build) and requires that at least one pin catches it: the hand-worked
examples, the exact-rational brute force, the closed forms, or the two-rank library sum."""
import ctypes
import os
import subprocess

import numpy as np
import pytest
import torch

import exact_rational as ex
import rar_inputs as ri
from test_oracle_pins import GOLDEN, _adversarial, bf16

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "nvrar_oracle.c")

MUTATIONS = {
    "peer distance order reversed":
        ("const int peer = node_of_number(step_number(r_n, r) ^ (1 << l), r) * G + r_g;",
         "const int peer = node_of_number(step_number(r_n, r) ^ (1 << (L - 1 - l)), r) * G + r_g;"),
    "peer has another local id":
        ("const int peer = node_of_number(step_number(r_n, r) ^ (1 << l), r) * G + r_g;",
         "const int peer = node_of_number(step_number(r_n, r) ^ (1 << l), r) * G + (G - 1 - r_g);"),
    "steps pair real node numbers although N is not a power of two":
        ("const int peer = node_of_number(step_number(r_n, r) ^ (1 << l), r) * G + r_g;",
         "const int peer = ((r_n ^ (1 << l)) < N ? (r_n ^ (1 << l)) : r_n) * G + r_g;"),
    "fold pairs (2i+1, 2i+2) instead of (2i, 2i+1)":
        ("const void *handed = B_send[0 * P + (r_n - 1) * G + r_g];",
         "const void *handed = B_send[0 * P + ((r_n + 1 < N ? r_n + 1 : r_n - 1)) * G + r_g];"),
    "the folded-in value is dropped":
        ("float sum = load_elem(handed, i, dtype) + load_elem(own, i, dtype);", "float sum = load_elem(own, i, dtype);"),
    "nodes that sat out get a neighbour's input instead of the result":
        ("memcpy(B_send[L * P + p], B_send[L * P + (r_n + 1) * G + r_g], cnt * es);",
         "memcpy(B_send[L * P + p], B_send[0 * P + (r_n + 1) * G + r_g], cnt * es);"),
    "narrowing inside the node sum":
        ("for (int g = 1; g < G; ++g) acc = acc + load_elem(in[r_n * G + g], j, dtype);",
         "for (int g = 1; g < G; ++g) { acc = acc + load_elem(in[r_n * G + g], j, dtype);"
         " if (dtype == ORACLE_BF16) acc = widen_bf16(narrow_bf16(acc)); }"),
    "ties round away from zero":
        ("(dropped == 0x8000u && (kept & 1u))", "(dropped == 0x8000u)"),
    "truncation instead of rounding":
        ("kept += 1u;", "kept += 0u;"),
    "last local rank skipped":
        ("for (int g = 1; g < G; ++g) acc", "for (int g = 1; g < G - (G > 2); ++g) acc"),
    "node sum in descending local rank order":
        ("float acc = load_elem(in[r_n * G + 0], j, dtype);\n            for (int g = 1; g < G; ++g) acc = acc + load_elem(in[r_n * G + g], j, dtype);",
         "float acc = load_elem(in[r_n * G + G - 1], j, dtype);\n            for (int g = G - 2; g >= 0; --g) acc = acc + load_elem(in[r_n * G + g], j, dtype);"),
    "peer's already updated buffer is read (in-place hazard)":
        ("const void *dst = B_send[l * P + peer];", "const void *dst = B_send[(l + (peer < p)) * P + peer];"),
    "difference instead of sum in a step":
        ("float sum = load_elem(dst, i, dtype) + load_elem(src, i, dtype);\n                store_elem(next",
         "float sum = load_elem(dst, i, dtype) - load_elem(src, i, dtype);\n                store_elem(next"),
    "all-gather lands in chunk 0":
        ("memcpy((char *)out[r_n * G + g] + lo * es, Mprime", "memcpy((char *)out[r_n * G + g] + 0 * es, Mprime"),
    "one step too few":
        ("for (int l = 0; l < L; ++l) {\n        #pragma omp", "for (int l = 0; l < L - (L > 1); ++l) {\n        #pragma omp"),
}


def build_mutant(tmp_path, old: str, new: str):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site not found exactly once: {old!r}"
    text = text.replace(old, new)
    if "L - (L > 1)" in new:   # "one step too few": the all-gather must then read the last buffer written
        text = text.replace("const char *Mprime = (const char *)B_send[L * P + p];",
                            "const char *Mprime = (const char *)B_send[(L - (L > 1)) * P + p];")
    c = tmp_path / "mutant.c"
    so = tmp_path / "mutant.so"
    c.write_text(text)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-o", str(so), str(c)],
                   check=True)
    lib = ctypes.CDLL(str(so))
    lib.nvrar_oracle_allreduce.restype = ctypes.c_int
    lib.nvrar_oracle_allreduce.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
                                           ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int]

    def allreduce(x, G):
        x = np.ascontiguousarray(x)
        P, n = x.shape
        out = np.zeros_like(x)
        ins = (ctypes.c_void_p * P)(*[x[p].ctypes.data for p in range(P)])
        outs = (ctypes.c_void_p * P)(*[out[p].ctypes.data for p in range(P)])
        assert lib.nvrar_oracle_allreduce(ins, outs, G, P // G, n, 0 if x.dtype == np.uint16 else 1, 1) == 0
        return out
    return allreduce


def pins_catch(allreduce) -> bool:
    """True as soon as one pin disagrees with the given implementation."""
    # hand-worked examples
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        _, dtype, G, N, ins, want = [f.strip() for f in line.split("|")]
        col = np.asarray([float(v) for v in ins.split()], dtype=np.float32).reshape(-1, 1)
        x = bf16(col) if dtype == "bf16" else col
        w = bf16([float(want)]) if dtype == "bf16" else np.asarray([float(want)], dtype=np.float32)
        out = allreduce(x, int(G))
        if any(out[p].tobytes() != w.tobytes() for p in range(x.shape[0])):
            return True
    # exact-rational brute force
    for P, G in ((4, 2), (8, 2), (8, 4), (16, 4), (16, 1), (3, 1), (6, 2), (5, 1), (7, 1), (12, 4), (11, 1)):
        for dtype in ("bf16", "f32"):
            x = _adversarial(np.random.default_rng(100 * P + G), P, 48, dtype)
            want, got = ex.allreduce(x, G), allreduce(x, G)
            wf = ri.bf16_bits_to_f32(want) if dtype == "bf16" else want
            nan = np.isnan(wf)
            if not np.array_equal(got[~nan], want[~nan]):
                return True
    # closed forms: weighted rank indicator
    for P, G in ((8, 4), (16, 4), (6, 3), (6, 2), (20, 4), (7, 1)):
        n = 3 * P + 5
        wind = bf16((np.arange(n)[None, :] % P == np.arange(P)[:, None]) * (np.arange(P)[:, None] + 1.0))
        got = ri.bf16_bits_to_f32(allreduce(wind, G))
        if not np.all(got == (np.arange(n) % P + 1).astype(np.float32)[None, :]):
            return True
    # two ranks against the library sum
    bits = np.random.default_rng(11).integers(0, 0x7F80, size=(2, 4096), dtype=np.uint16)
    a = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)
    want = (a[0].float() + a[1].float()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for G in (1, 2):
        if not np.array_equal(allreduce(bits, G)[1], want):
            return True
    return False


def test_the_unmodified_oracle_passes_these_pins(tmp_path):
    same = build_mutant(tmp_path, "kept += 1u;", "kept += 1u; ")
    assert not pins_catch(same)


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTATIONS[name]
    mutant = build_mutant(tmp_path, old, new)
    assert pins_catch(mutant), f"no pin noticed: {name}"
