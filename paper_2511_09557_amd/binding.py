"""ctypes binding of librar.so: the same names as include/rar.h, argument marshalling only.

The library is required: importing this module raises if librar.so has not been built
(python -m paper_2511_09557_amd.build, or __graft_entry__.build()).  There is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

RAR_BF16, RAR_F32 = 0, 1
RAR_MODE_STEPWISE, RAR_MODE_FUSED, RAR_MODE_FUSED_PACKED, RAR_MODE_AUTO = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librar.so")


class RarError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = f" [{lib.rar_last_hip_error().decode()}]" if status == -7 else ""
        super().__init__(f"{where}: {rar_strerror(status)} ({status}){detail}")


def _load() -> ctypes.CDLL:
    # PyTorch wheels bundle their own HIP runtime.  A process that uses both must load torch's
    # first: with librar.so (and the system runtime it links) loaded before torch, the library's
    # runtime then finds no device.  torch is optional for the plain rar_* functions.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2511_09557_amd.build` "
            "(hipcc, gfx950). The HIP library is the only implementation; there is no fallback.")
    L = ctypes.CDLL(LIB_PATH)
    vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    sig = {
        "rar_version": (ci, []),
        "rar_strerror": (ctypes.c_char_p, [ci]),
        "rar_last_hip_error": (ctypes.c_char_p, []),
        "rar_plan": (ci, [ci, ci, sz, ci, ctypes.POINTER(vp)]),
        "rar_plan_free": (ci, [vp]),
        "rar_plan_ranks": (ci, [vp]),
        "rar_plan_nodes": (ci, [vp]),
        "rar_plan_steps": (ci, [vp]),
        "rar_plan_peer": (ci, [vp, ci, ci]),
        "rar_plan_fold_partner": (ci, [vp, ci]),
        "rar_plan_chunk": (ci, [vp, ci, ctypes.POINTER(sz), ctypes.POINTER(sz)]),
        "rar_plan_scratch_bytes": (sz, [vp]),
        "rar_plan_scratch_layout": (ci, [vp, ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(sz)]),
        "rar_plan_set_scratch": (ci, [vp, vp, sz]),
        "rar_plan_set_mode": (ci, [vp, ci]),
        "rar_plan_get_mode": (ci, [vp]),
        "rar_plan_effective_mode": (ci, [vp]),
        "rar_plan_set_tuning": (ci, [vp, ci, sz]),
        "rar_plan_get_tuning": (ci, [vp, ctypes.POINTER(ci), ctypes.POINTER(sz)]),
        "rar_plan_set_concurrency": (ci, [vp, ci]),
        "rar_plan_set_wait_limit_us": (ci, [vp, ctypes.c_uint64]),
        "rar_plan_status": (ci, [vp, vp]),
        "rar_step_combine": (ci, [vp, vp, sz, sz, ci, vp]),
        "rar_allreduce": (ci, [ctypes.POINTER(vp), vp, vp]),
        "rar_allreduce_chain": (ci, [ctypes.POINTER(vp), vp, ci, vp]),
        "rar_allreduce_static": (ci, [ctypes.POINTER(vp), vp, vp]),
        "rar_plan_static_bytes": (sz, [vp]),
        "rar_autotune": (ci, [ctypes.POINTER(vp), vp, vp, ci, ctypes.POINTER(ctypes.c_double)]),
        "rar_launch_floor": (ci, [vp, vp]),
        "rar_barrier_only": (ci, [vp, vp]),
        "rar_copy_probe": (ci, [vp, vp, sz, vp]),
        "rar_read_probe": (ci, [vp, vp, sz, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    return L


lib = _load()
EXPORTS = ["rar_version", "rar_strerror", "rar_last_hip_error", "rar_plan", "rar_plan_free", "rar_plan_ranks",
           "rar_plan_nodes", "rar_plan_steps", "rar_plan_peer", "rar_plan_fold_partner", "rar_plan_chunk",
           "rar_plan_scratch_bytes", "rar_plan_scratch_layout", "rar_plan_set_scratch", "rar_plan_set_mode",
           "rar_plan_get_mode", "rar_plan_effective_mode", "rar_plan_set_tuning", "rar_plan_get_tuning",
           "rar_plan_set_concurrency", "rar_plan_set_wait_limit_us", "rar_plan_status", "rar_step_combine", "rar_allreduce",
           "rar_allreduce_chain", "rar_allreduce_static", "rar_plan_static_bytes", "rar_autotune", "rar_launch_floor", "rar_barrier_only", "rar_copy_probe", "rar_read_probe"]


def _check(status: int, where: str) -> int:
    if status < 0:
        raise RarError(status, where)
    return status


def rar_version() -> int:
    return lib.rar_version()


def rar_strerror(status: int) -> str:
    return lib.rar_strerror(status).decode()


def rar_plan(P: int, G: int, n: int, dtype: int) -> int:
    """Returns the plan handle (an address); raises RarError on a bad shape."""
    out = ctypes.c_void_p()
    _check(lib.rar_plan(P, G, n, dtype, ctypes.byref(out)), "rar_plan")
    return out.value


def rar_plan_free(plan: int) -> None:
    _check(lib.rar_plan_free(plan), "rar_plan_free")


def rar_plan_ranks(plan: int) -> int:
    return _check(lib.rar_plan_ranks(plan), "rar_plan_ranks")


def rar_plan_nodes(plan: int) -> int:
    return _check(lib.rar_plan_nodes(plan), "rar_plan_nodes")


def rar_plan_steps(plan: int) -> int:
    return _check(lib.rar_plan_steps(plan), "rar_plan_steps")


def rar_plan_peer(plan: int, rank: int, step: int) -> int:
    return _check(lib.rar_plan_peer(plan, rank, step), "rar_plan_peer")


def rar_plan_fold_partner(plan: int, rank: int) -> int:
    return _check(lib.rar_plan_fold_partner(plan, rank), "rar_plan_fold_partner")


def rar_plan_chunk(plan: int, c: int):
    off, length = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib.rar_plan_chunk(plan, c, ctypes.byref(off), ctypes.byref(length)), "rar_plan_chunk")
    return off.value, length.value


def rar_plan_scratch_bytes(plan: int) -> int:
    return lib.rar_plan_scratch_bytes(plan)


def rar_plan_scratch_layout(plan: int):
    """(flags_offset, flags_bytes, packed_offset, packed_bytes) inside the scratch."""
    v = [ctypes.c_size_t() for _ in range(4)]
    _check(lib.rar_plan_scratch_layout(plan, *[ctypes.byref(x) for x in v]), "rar_plan_scratch_layout")
    return tuple(x.value for x in v)


def rar_plan_set_scratch(plan: int, scratch_ptr: int, nbytes: int) -> None:
    _check(lib.rar_plan_set_scratch(plan, scratch_ptr, nbytes), "rar_plan_set_scratch")


def rar_plan_set_mode(plan: int, mode: int) -> None:
    _check(lib.rar_plan_set_mode(plan, mode), "rar_plan_set_mode")


def rar_plan_get_mode(plan: int) -> int:
    return _check(lib.rar_plan_get_mode(plan), "rar_plan_get_mode")


def rar_plan_effective_mode(plan: int) -> int:
    return _check(lib.rar_plan_effective_mode(plan), "rar_plan_effective_mode")


def rar_plan_set_tuning(plan: int, B_s: int, C_s: int) -> None:
    _check(lib.rar_plan_set_tuning(plan, B_s, C_s), "rar_plan_set_tuning")


def rar_plan_get_tuning(plan: int):
    b, c = ctypes.c_int(), ctypes.c_size_t()
    _check(lib.rar_plan_get_tuning(plan, ctypes.byref(b), ctypes.byref(c)), "rar_plan_get_tuning")
    return b.value, c.value


def rar_plan_set_concurrency(plan: int, k: int) -> None:
    _check(lib.rar_plan_set_concurrency(plan, k), "rar_plan_set_concurrency")


def rar_plan_set_wait_limit_us(plan: int, microseconds: int) -> None:
    _check(lib.rar_plan_set_wait_limit_us(plan, microseconds), "rar_plan_set_wait_limit_us")


def rar_plan_status(plan: int, stream: int = 0) -> int:
    """Returns the raw status (0 or RAR_ERR_TIMEOUT = -8); raises on any other error."""
    rc = lib.rar_plan_status(plan, stream)
    if rc not in (0, -8):
        raise RarError(rc, "rar_plan_status")
    return rc


def rar_step_combine(dst_ptr: int, src_ptr: int, chunk: int, n: int, dtype: int, stream: int = 0) -> None:
    _check(lib.rar_step_combine(dst_ptr, src_ptr, chunk, n, dtype, stream), "rar_step_combine")


def rar_allreduce(buf_ptrs: Sequence[int], plan: int, stream: int = 0) -> None:
    arr = (ctypes.c_void_p * len(buf_ptrs))(*buf_ptrs)
    _check(lib.rar_allreduce(arr, plan, stream), "rar_allreduce")


def rar_allreduce_chain(buf_ptrs: Sequence[int], plan: int, K: int, stream: int = 0) -> None:
    arr = (ctypes.c_void_p * len(buf_ptrs))(*buf_ptrs)
    _check(lib.rar_allreduce_chain(arr, plan, K, stream), "rar_allreduce_chain")


RAR_STATIC_SCRATCH_BYTES = 48 << 20


def rar_allreduce_static(buf_ptrs: Sequence[int], plan: int, stream: int = 0) -> None:
    """rar_allreduce on the library's own scratch array (the plan needs no scratch of its own)."""
    arr = (ctypes.c_void_p * len(buf_ptrs))(*buf_ptrs)
    _check(lib.rar_allreduce_static(arr, plan, stream), "rar_allreduce_static")


def rar_plan_static_bytes(plan: int) -> int:
    return lib.rar_plan_static_bytes(plan)


def rar_autotune(buf_ptrs: Sequence[int], plan: int, stream: int = 0, calls: int = 20) -> float:
    """Returns the winner's mean microseconds per call; the plan keeps the winning B_s, C_s."""
    arr = (ctypes.c_void_p * len(buf_ptrs))(*buf_ptrs)
    best = ctypes.c_double()
    _check(lib.rar_autotune(arr, plan, stream, calls, ctypes.byref(best)), "rar_autotune")
    return best.value


def rar_launch_floor(plan: int, stream: int = 0) -> None:
    _check(lib.rar_launch_floor(plan, stream), "rar_launch_floor")


def rar_barrier_only(plan: int, stream: int = 0) -> None:
    _check(lib.rar_barrier_only(plan, stream), "rar_barrier_only")


def rar_copy_probe(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(lib.rar_copy_probe(dst_ptr, src_ptr, nbytes, stream), "rar_copy_probe")


def rar_read_probe(sink_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(lib.rar_read_probe(sink_ptr, src_ptr, nbytes, stream), "rar_read_probe")


class AllReduce:
    """A plan plus the torch tensor that backs its scratch.  torch supplies device memory and
    the current stream; every step of the all-reduce runs inside librar.so."""

    def __init__(self, P: int, G: int, n: int, dtype: int, mode: int = RAR_MODE_AUTO, device="cuda:0"):
        import torch
        self.P, self.G, self.n, self.dtype = P, G, n, dtype
        self.plan = rar_plan(P, G, n, dtype)
        try:
            nbytes = rar_plan_scratch_bytes(self.plan)
            self.scratch = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
            base = self.scratch.data_ptr()
            aligned = (base + 255) // 256 * 256
            rar_plan_set_scratch(self.plan, aligned, nbytes)
            self.scratch_base = aligned - base      # offset of the plan's scratch inside self.scratch
            rar_plan_set_mode(self.plan, mode)
        except Exception:
            rar_plan_free(self.plan)
            self.plan = None
            raise
        self._bound = None
        self._bound_ptrs = None

    def _stream(self, stream) -> int:
        if isinstance(stream, int):      # a raw hipStream_t handle: nothing to look up
            return stream
        if stream is None:
            import torch
            return torch.cuda.current_stream().cuda_stream
        return stream.cuda_stream

    def bind(self, tensors) -> None:
        """Check P tensors (one per virtual rank, n elements each) and keep their addresses, so
        that later launches marshal nothing per call.  The tensors must stay alive and in place."""
        if len(tensors) != self.P:
            raise ValueError(f"need {self.P} tensors")
        for t in tensors:
            if t.numel() != self.n or not t.is_contiguous() or not t.is_cuda:
                raise ValueError("each rank's tensor must be a contiguous CUDA tensor of n elements")
        self._bound = tensors
        self._bound_ptrs = (ctypes.c_void_p * self.P)(*[t.data_ptr() for t in tensors])

    def launch(self, stream=None) -> None:
        """In-place all-reduce of the bound tensors."""
        _check(lib.rar_allreduce(self._bound_ptrs, self.plan, self._stream(stream)), "rar_allreduce")

    def launch_chain(self, K: int, stream=None) -> None:
        """K in-place all-reduces of the bound tensors, each on the result of the one before, in one launch."""
        _check(lib.rar_allreduce_chain(self._bound_ptrs, self.plan, K, self._stream(stream)), "rar_allreduce_chain")

    def __call__(self, tensors, stream=None) -> None:
        """In-place all-reduce of P tensors of n elements each (one per virtual rank)."""
        if tensors is not self._bound:
            self.bind(tensors)
        self.launch(stream)

    def set_mode(self, mode: int) -> None:
        rar_plan_set_mode(self.plan, mode)

    def effective_mode(self) -> int:
        return rar_plan_effective_mode(self.plan)

    def set_tuning(self, B_s: int = 0, C_s: int = 0) -> None:
        rar_plan_set_tuning(self.plan, B_s, C_s)

    def tuning(self):
        return rar_plan_get_tuning(self.plan)

    def autotune(self, tensors, calls: int = 20, stream=None) -> float:
        """Measure the candidate (B_s, C_s) pairs on `tensors` (overwritten) and keep the fastest."""
        self.bind(tensors)
        best = ctypes.c_double()
        _check(lib.rar_autotune(self._bound_ptrs, self.plan, self._stream(stream), calls, ctypes.byref(best)),
               "rar_autotune")
        return best.value

    def status(self, stream=None) -> int:
        return rar_plan_status(self.plan, self._stream(stream))

    def launch_floor(self, stream=None) -> None:
        rar_launch_floor(self.plan, self._stream(stream))

    def barrier_only(self, stream=None) -> None:
        rar_barrier_only(self.plan, self._stream(stream))

    def close(self) -> None:
        if self.plan is not None:
            rar_plan_free(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
