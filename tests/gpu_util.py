"""Helpers for the GPU parity tests: numpy <-> device tensors, one tensor per virtual rank."""
import numpy as np
import torch


def to_device(x: np.ndarray):
    """x[P, n] (uint16 bf16 bits or float32) -> list of P separately allocated CUDA tensors."""
    out = []
    for p in range(x.shape[0]):
        if x.dtype == np.uint16:
            t = torch.from_numpy(x[p].view(np.int16).copy()).view(torch.bfloat16)
        else:
            t = torch.from_numpy(x[p].copy())
        out.append(t.to("cuda:0"))
    return out


def to_host(tensors, np_dtype) -> np.ndarray:
    rows = []
    for t in tensors:
        c = t.detach().cpu()
        if np_dtype == np.uint16:
            rows.append(c.view(torch.int16).numpy().view(np.uint16).copy())
        else:
            rows.append(c.numpy().copy())
    return np.stack(rows)


def assert_same_bits(got: np.ndarray, want: np.ndarray, what: str = ""):
    """Bit-exact, except that NaN positions only have to be NaN on both sides."""
    assert got.shape == want.shape and got.dtype == want.dtype, what
    if got.dtype == np.uint16:
        nan_g = ((got & 0x7F80) == 0x7F80) & ((got & 0x007F) != 0)
        nan_w = ((want & 0x7F80) == 0x7F80) & ((want & 0x007F) != 0)
    else:
        nan_g, nan_w = np.isnan(got), np.isnan(want)
    assert np.array_equal(nan_g, nan_w), f"{what}: NaN positions differ"
    ok = nan_w | (got.view(np.uint16 if got.dtype == np.uint16 else np.uint32) ==
                  want.view(np.uint16 if want.dtype == np.uint16 else np.uint32))
    if not ok.all():
        bad = np.argwhere(~ok)
        first = tuple(bad[0])
        raise AssertionError(f"{what}: {bad.shape[0]} of {ok.size} elements differ; first at {first}: "
                             f"got {got[first]!r} want {want[first]!r}")
