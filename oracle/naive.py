"""Yardstick for the error-bound check: sequential fp64 sum over ranks 0, 1, .., P-1.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  This is NOT what the method computes
(the method's result depends on its order and rounding points); it is the plain definition
of the sum that the method approximates, used to check the stated relative-error bound.
"""
from __future__ import annotations

import numpy as np


def to_f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:  # bf16 bit patterns
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def naive_sum_f64(x: np.ndarray):
    """x[P, n] -> (sum[n], abs_sum[n]) in fp64, ranks added in ascending order."""
    acc = np.zeros(x.shape[1], dtype=np.float64)
    mag = np.zeros(x.shape[1], dtype=np.float64)
    for p in range(x.shape[0]):
        v = to_f64(x[p])
        acc = acc + v
        mag = mag + np.abs(v)
    return acc, mag
