"""Second formulation of the oracle: the inter-node phase as a balanced binary tree.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

In recursive doubling (Algorithm 1, RD_inter; Section 4.1) node r_n and node r_n XOR 2^l
form the same IEEE sum at step l (addition commutes), so after step l every aligned group of
2^(l+1) nodes holds one common value, and the final value is the balanced tree

    T(lo, 1)  = S_0(lo)                      (the node's reduce-scatter result)
    T(lo, 2k) = rnd( T(lo, k) + T(lo + k, k) )
    result    = T(0, N)

over node index in natural order.  This file computes exactly that, with whole-array numpy
float32 operations and no chunking (every element is independent), and narrows to bf16 with
the integer form of round-to-nearest-even rather than the compare form the C oracle uses.
The tests require both formulations to agree bit for bit.

For N that is not a power of two (outside the paper) the first 2r nodes, N = 2^L + r, are summed
pairwise first and the tree runs over the 2^L values that remain, see nvrar_oracle.c.
"""
from __future__ import annotations

import numpy as np


def widen(a: np.ndarray) -> np.ndarray:
    """Message type -> float32 (exact)."""
    if a.dtype == np.float32:
        return a
    return (a.astype(np.uint32) << np.uint32(16)).view(np.float32)


def narrow(f: np.ndarray, dtype) -> np.ndarray:
    """float32 -> message type; bf16 by round-to-nearest, ties to even."""
    if dtype == np.float32:
        return f.astype(np.float32, copy=False)
    u = np.ascontiguousarray(f, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)
    nan = np.isnan(f)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def _tree(S0: np.ndarray, lo: int, cnt: int, dtype) -> np.ndarray:
    if cnt == 1:
        return S0[lo]
    half = cnt // 2
    left = _tree(S0, lo, half, dtype)
    right = _tree(S0, lo + half, half, dtype)
    with np.errstate(all="ignore"):
        return narrow(widen(left) + widen(right), dtype)


def tree_allreduce(x: np.ndarray, G: int) -> np.ndarray:
    """x[P, n] -> out[P, n]; rank p = r_n*G + r_g."""
    P, n = x.shape
    if G < 1 or P % G:
        raise ValueError("G must divide P")
    N = P // G
    dtype = x.dtype
    S0 = []
    for r_n in range(N):
        with np.errstate(all="ignore"):
            acc = widen(x[r_n * G + 0]).copy()
            for g in range(1, G):
                acc = acc + widen(x[r_n * G + g])
        S0.append(narrow(acc, dtype))
    # N = 2^L + r: the first 2r nodes are folded pairwise (even into odd) before the tree, and the
    # tree runs over the 2^L values in the order [folded pairs..., remaining nodes...]
    L = N.bit_length() - 1
    r = N - (1 << L)
    leaves = []
    for v in range(1 << L):
        if v < r:
            with np.errstate(all="ignore"):
                leaves.append(narrow(widen(S0[2 * v]) + widen(S0[2 * v + 1]), dtype))
        else:
            leaves.append(S0[v + r])
    total = _tree(leaves, 0, 1 << L, dtype)
    return np.broadcast_to(total, (P, n)).copy()
