"""Thin ctypes binding of the libwagma C-ABI (``include/wagma.h``).

Argument marshalling only: every step of the path runs in the HIP kernels of
``libwagma.so``.  PyTorch tensors are used as device allocations (their
``data_ptr()``) and for the current HIP stream; nothing is computed in Python
and there is no CPU fallback — ``load()`` raises if the library is not built.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libwagma.so")

WAGMA_OK, WAGMA_EINVAL, WAGMA_EHIP, WAGMA_ENOMEM = 0, -1, -2, -3
WAGMA_MAX_P = 1024
WAGMA_STATIC_TABLE_BYTES = 45056
WAGMA_GROUPING_DYNAMIC, WAGMA_GROUPING_FIXED = 0, 1
WAGMA_OPT_NONTEMPORAL, WAGMA_OPT_PLACEMENT = 2, 9
# launch-shape switches outside the public header (csrc/wagma_internal.h): tests and measurements only
WAGMA_DEBUG_FORCE_STREAM, WAGMA_DEBUG_STRIPE_LOG2, WAGMA_DEBUG_XCD_CHUNK_LOG2 = 3, 7, 8
WAGMA_DEBUG_PLACED_SHAPE, WAGMA_DEBUG_MAP, WAGMA_DEBUG_PLACED_COOP_SHAPE = 10, 11, 12
WAGMA_DEBUG_TENSOR_TABLES = 13
WAGMA_PLACE_PLAIN, WAGMA_PLACE_ARRAYS, WAGMA_PLACE_CHUNKS, WAGMA_PLACE_AUTO, WAGMA_PLACE_SEARCH = 0, 1, 2, 3, 4

# name -> (restype, argtypes): every symbol include/wagma.h declares
_i32pp = ctypes.POINTER(ctypes.POINTER(ctypes.c_int32))
_u64p = ctypes.POINTER(ctypes.c_uint64)
SYMBOLS = {
    "wagma_create": (ctypes.c_int, [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_int,
                                    ctypes.c_int64, ctypes.c_int]),
    "wagma_destroy": (ctypes.c_int, [ctypes.c_void_p]),
    "wagma_row_stride": (ctypes.c_int64, [ctypes.c_void_p]),
    "wagma_set_row_stride": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64]),
    "wagma_set_grouping": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int]),
    "wagma_schedule_period": (ctypes.c_int, [ctypes.c_void_p]),
    "wagma_group_schedule": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, _i32pp, _i32pp]),
    "wagma_is_global_iteration": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64]),
    "wagma_step": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                  ctypes.c_void_p, _u64p, ctypes.c_float, ctypes.c_float,
                                  ctypes.c_int64, ctypes.c_void_p]),
    "wagma_step_static": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_int64,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         _u64p, ctypes.c_float, ctypes.c_float, ctypes.c_int64, ctypes.c_void_p]),
    "wagma_tensors_create": (ctypes.c_int, [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
                                            ctypes.POINTER(ctypes.c_int64)] + [ctypes.POINTER(ctypes.c_void_p)] * 4),
    "wagma_tensors_destroy": (ctypes.c_int, [ctypes.c_void_p]),
    "wagma_step_tensors": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, _u64p, ctypes.c_float,
                                          ctypes.c_float, ctypes.c_int64, ctypes.c_void_p]),
    "wagma_step_lag": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_void_p, _u64p, _u64p, ctypes.c_float, ctypes.c_float,
                                      ctypes.c_int64, ctypes.c_void_p]),
    "wagma_step_tensors_lag": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, _u64p, _u64p, ctypes.c_float,
                                              ctypes.c_float, ctypes.c_int64, ctypes.c_void_p]),
    "wagma_lag_masks": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int64, ctypes.c_int,
                                       ctypes.c_uint32, _u64p, _u64p]),
    "wagma_stale_mask": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int64,
                                        ctypes.c_uint32, _u64p]),
    "wagma_straggler_mask": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int64, ctypes.c_int, _u64p]),
    "wagma_clock_mask": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int64, ctypes.c_uint32, _u64p,
                                        ctypes.POINTER(ctypes.c_uint32)]),
    "wagma_alloc_buffers": (ctypes.c_int, [ctypes.c_void_p] + [ctypes.POINTER(ctypes.c_void_p)] * 4),
    "wagma_free_buffers": (ctypes.c_int, [ctypes.c_void_p]),
    "wagma_placement_info": (ctypes.c_int, [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int),
                                            ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int),
                                            ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]),
    "wagma_set_option": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64]),
    "wagma_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "wagma_last_hip_error": (ctypes.c_int, []),
}

# exported, but not declared in include/wagma.h (csrc/wagma_internal.h): tests and measurements only
DEBUG_SYMBOLS = {
    "wagma_debug_set_option": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64]),
    "wagma_debug_get_option": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]),
}

_lib = None


class WagmaError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        text = load().wagma_strerror(code).decode()
        hip = load().wagma_last_hip_error() if code == WAGMA_EHIP else 0
        super().__init__("%s: %s (code %d%s)" % (what, text, code, ", hipError %d" % hip if hip else ""))


def load() -> ctypes.CDLL:
    """Load libwagma.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libwagma.so is not built: run `python -m paper_2005_00124_amd.build` "
                "(there is no CPU fallback)")
        # PyTorch ships its own HIP runtime (same soname).  Import it first so that this
        # library binds to the runtime that owns the tensors and streams it is handed.
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        for name, (restype, argtypes) in {**SYMBOLS, **DEBUG_SYMBOLS}.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = restype, argtypes
        _lib = lib
    return _lib


def _check(code: int, what: str) -> None:
    if code != WAGMA_OK:
        raise WagmaError(code, what)


def _ptr(x) -> int:
    return x if isinstance(x, int) else x.data_ptr()


def _current_stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


# ---- the C-ABI, one function per entry point, same names -------------------

def wagma_create(P: int, S: int, n: int, tau: int) -> int:
    out = ctypes.c_void_p()
    _check(load().wagma_create(ctypes.byref(out), P, S, n, tau), "wagma_create")
    return out.value


def wagma_destroy(ctx: int) -> None:
    _check(load().wagma_destroy(ctx), "wagma_destroy")


def wagma_row_stride(ctx: int) -> int:
    ld = load().wagma_row_stride(ctx)
    if ld < 0:
        raise WagmaError(int(ld), "wagma_row_stride")
    return int(ld)


def wagma_set_row_stride(ctx: int, ld: int) -> None:
    _check(load().wagma_set_row_stride(ctx, ld), "wagma_set_row_stride")


def wagma_set_grouping(ctx: int, mode: int) -> None:
    _check(load().wagma_set_grouping(ctx, mode), "wagma_set_grouping")


def wagma_schedule_period(ctx: int) -> int:
    period = load().wagma_schedule_period(ctx)
    if period < 0:
        raise WagmaError(period, "wagma_schedule_period")
    return period


def wagma_is_global_iteration(ctx: int, it: int) -> bool:
    rc = load().wagma_is_global_iteration(ctx, it)
    if rc < 0:
        raise WagmaError(rc, "wagma_is_global_iteration")
    return bool(rc)


def wagma_group_schedule(ctx: int, it: int, P: int):
    """Returns (device pointer as int, host table as a read-only int32 numpy view of P entries)."""
    dev = ctypes.POINTER(ctypes.c_int32)()
    host = ctypes.POINTER(ctypes.c_int32)()
    _check(load().wagma_group_schedule(ctx, it, ctypes.byref(dev), ctypes.byref(host)),
           "wagma_group_schedule")
    table = np.ctypeslib.as_array(host, shape=(P,))
    table.flags.writeable = False
    return ctypes.cast(dev, ctypes.c_void_p).value, table


def wagma_step(ctx: int, w, g, m, pub, stale_mask: Optional[np.ndarray], lr: float, mu: float,
               it: int, stream: Optional[int] = None) -> None:
    """w, g, m, pub: torch CUDA tensors (or raw device addresses).  stale_mask: uint64 words or None."""
    mask = None
    if stale_mask is not None:
        stale_mask = np.ascontiguousarray(stale_mask, dtype=np.uint64)
        mask = stale_mask.ctypes.data_as(_u64p)
    if stream is None:
        stream = _current_stream()
    _check(load().wagma_step(ctx, _ptr(w), _ptr(g), _ptr(m), _ptr(pub), mask, lr, mu, it, stream),
           "wagma_step")


def wagma_step_static(P: int, S: int, n: int, tau: int, ld: int, w, g, m, pub,
                      stale_mask: Optional[np.ndarray], lr: float, mu: float, it: int,
                      stream: Optional[int] = None) -> None:
    """wagma_step without a context and without any allocation (static schedule table)."""
    keep, mask = _mask_arg(stale_mask)
    if stream is None:
        stream = _current_stream()
    _check(load().wagma_step_static(P, S, n, tau, ld, _ptr(w), _ptr(g), _ptr(m), _ptr(pub), mask, lr, mu,
                                    it, stream), "wagma_step_static")


def _mask_arg(mask: Optional[np.ndarray]):
    """(object to keep alive, ctypes pointer or None) for a host mask of uint64 words."""
    if mask is None:
        return None, None
    mask = np.ascontiguousarray(mask, dtype=np.uint64)
    return mask, mask.ctypes.data_as(_u64p)


def wagma_step_lag(ctx: int, w, g, m, pub, late_mask: Optional[np.ndarray], busy_mask: Optional[np.ndarray],
                   lr: float, mu: float, it: int, stream: Optional[int] = None) -> None:
    """wagma_step with a second mask: the processes that are still computing an earlier step."""
    keep_late, late = _mask_arg(late_mask)
    keep_busy, busy = _mask_arg(busy_mask)
    if stream is None:
        stream = _current_stream()
    _check(load().wagma_step_lag(ctx, _ptr(w), _ptr(g), _ptr(m), _ptr(pub), late, busy, lr, mu, it, stream),
           "wagma_step_lag")


def wagma_tensors_create(ctx: int, sizes, w_ptrs, g_ptrs, m_ptrs, pub_ptrs) -> int:
    """sizes: T ints; *_ptrs: P*T device addresses each, entry p*T + k = tensor k of process p."""
    T = len(sizes)
    c_sizes = (ctypes.c_int64 * T)(*sizes)
    tables = [(ctypes.c_void_p * len(ptrs))(*ptrs) for ptrs in (w_ptrs, g_ptrs, m_ptrs, pub_ptrs)]
    out = ctypes.c_void_p()
    _check(load().wagma_tensors_create(ctx, ctypes.byref(out), T, c_sizes, *tables), "wagma_tensors_create")
    return out.value


def wagma_tensors_destroy(plan: int) -> None:
    _check(load().wagma_tensors_destroy(plan), "wagma_tensors_destroy")


def wagma_step_tensors(ctx: int, plan: int, stale_mask: Optional[np.ndarray], lr: float, mu: float,
                       it: int, stream: Optional[int] = None) -> None:
    mask = None
    if stale_mask is not None:
        stale_mask = np.ascontiguousarray(stale_mask, dtype=np.uint64)
        mask = stale_mask.ctypes.data_as(_u64p)
    if stream is None:
        stream = _current_stream()
    _check(load().wagma_step_tensors(ctx, plan, mask, lr, mu, it, stream), "wagma_step_tensors")


def wagma_step_tensors_lag(ctx: int, plan: int, late_mask: Optional[np.ndarray],
                           busy_mask: Optional[np.ndarray], lr: float, mu: float, it: int,
                           stream: Optional[int] = None) -> None:
    keep_late, late = _mask_arg(late_mask)
    keep_busy, busy = _mask_arg(busy_mask)
    if stream is None:
        stream = _current_stream()
    _check(load().wagma_step_tensors_lag(ctx, plan, late, busy, lr, mu, it, stream), "wagma_step_tensors_lag")


def wagma_lag_masks(ctx: int, seed: int, it: int, window: int, tolerance_ms: int, P: int):
    """Returns (late words, busy words) of iteration ``it``."""
    late = np.zeros((P + 63) // 64, dtype=np.uint64)
    busy = np.zeros((P + 63) // 64, dtype=np.uint64)
    _check(load().wagma_lag_masks(ctx, seed, it, window, tolerance_ms, late.ctypes.data_as(_u64p),
                                  busy.ctypes.data_as(_u64p)), "wagma_lag_masks")
    return late, busy


def wagma_stale_mask(ctx: int, seed: int, it: int, threshold: int, P: int) -> np.ndarray:
    words = np.zeros((P + 63) // 64, dtype=np.uint64)
    _check(load().wagma_stale_mask(ctx, seed, it, threshold, words.ctypes.data_as(_u64p)),
           "wagma_stale_mask")
    return words


def wagma_straggler_mask(ctx: int, seed: int, it: int, count: int, P: int) -> np.ndarray:
    words = np.zeros((P + 63) // 64, dtype=np.uint64)
    _check(load().wagma_straggler_mask(ctx, seed, it, count, words.ctypes.data_as(_u64p)),
           "wagma_straggler_mask")
    return words


def wagma_clock_mask(ctx: int, seed: int, it: int, tolerance_ms: int, P: int):
    """Returns (mask words, step times in ms)."""
    words = np.zeros((P + 63) // 64, dtype=np.uint64)
    ms = np.zeros(P, dtype=np.uint32)
    _check(load().wagma_clock_mask(ctx, seed, it, tolerance_ms, words.ctypes.data_as(_u64p),
                                   ms.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32))), "wagma_clock_mask")
    return words, ms


def wagma_alloc_buffers(ctx: int):
    """Returns the device addresses (w, g, m, pub) of arrays placed by the library."""
    ptrs = [ctypes.c_void_p() for _ in range(4)]
    _check(load().wagma_alloc_buffers(ctx, *[ctypes.byref(p) for p in ptrs]), "wagma_alloc_buffers")
    return tuple(p.value for p in ptrs)


def wagma_free_buffers(ctx: int) -> None:
    _check(load().wagma_free_buffers(ctx), "wagma_free_buffers")


def wagma_placement_info(ctx: int) -> dict:
    mode, cand, regions, g_with_w = ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    same, split = ctypes.c_double(), ctypes.c_double()
    _check(load().wagma_placement_info(ctx, ctypes.byref(mode), ctypes.byref(cand), ctypes.byref(regions),
                                       ctypes.byref(g_with_w), ctypes.byref(same), ctypes.byref(split)),
           "wagma_placement_info")
    return {"mode": {0: "plain", 1: "arrays", 2: "chunks", 4: "search"}.get(mode.value, "?"), "candidates": cand.value, "regions": regions.value, "g_with_w": bool(g_with_w.value),
            "probe_same_region_gbs": same.value, "probe_two_regions_gbs": split.value}


class _DeviceArray:
    """A (P, ld) fp32 view of library-owned device memory for torch.as_tensor."""

    def __init__(self, ptr: int, shape):
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": "<f4", "data": (ptr, False),
                                         "version": 2, "strides": None}


def wagma_set_option(ctx: int, option: int, value: int) -> None:
    _check(load().wagma_set_option(ctx, option, value), "wagma_set_option")


def wagma_debug_set_option(ctx: int, option: int, value: int) -> None:
    """Launch-shape switches outside the public header; also takes the public options."""
    _check(load().wagma_debug_set_option(ctx, option, value), "wagma_debug_set_option")


def wagma_debug_get_option(ctx: int, option: int) -> int:
    value = ctypes.c_int64()
    _check(load().wagma_debug_get_option(ctx, option, ctypes.byref(value)), "wagma_debug_get_option")
    return int(value.value)


# ---- convenience wrapper ------------------------------------------------------

class Wagma:
    """Owns one wagma_ctx; checks tensor shapes on the host before a kernel sees them."""

    def __init__(self, P: int, S: int, n: int, tau: int):
        self.P, self.S, self.n, self.tau = P, S, n, tau
        self.ctx = wagma_create(P, S, n, tau)

    @property
    def ld(self) -> int:
        return wagma_row_stride(self.ctx)

    def set_row_stride(self, ld: int) -> None:
        wagma_set_row_stride(self.ctx, ld)

    def set_grouping(self, mode: int) -> None:
        wagma_set_grouping(self.ctx, mode)

    def set_option(self, option: int, value: int) -> None:
        wagma_set_option(self.ctx, option, value)

    def debug_set_option(self, option: int, value: int) -> None:
        wagma_debug_set_option(self.ctx, option, value)

    def debug_get_option(self, option: int) -> int:
        return wagma_debug_get_option(self.ctx, option)

    @property
    def period(self) -> int:
        return wagma_schedule_period(self.ctx)

    def is_global(self, it: int) -> bool:
        return wagma_is_global_iteration(self.ctx, it)

    def group_schedule(self, it: int):
        return wagma_group_schedule(self.ctx, it, self.P)

    def stale_mask(self, seed: int, it: int, threshold: int) -> np.ndarray:
        return wagma_stale_mask(self.ctx, seed, it, threshold, self.P)

    def straggler_mask(self, seed: int, it: int, count: int) -> np.ndarray:
        return wagma_straggler_mask(self.ctx, seed, it, count, self.P)

    def clock_mask(self, seed: int, it: int, tolerance_ms: int):
        return wagma_clock_mask(self.ctx, seed, it, tolerance_ms, self.P)

    def lag_masks(self, seed: int, it: int, tolerance_ms: int, window: int = 64):
        return wagma_lag_masks(self.ctx, seed, it, window, tolerance_ms, self.P)

    def alloc(self, device="cuda"):
        """Four (P, ld) fp32 device buffers w, g, m, pub (uninitialised)."""
        import torch
        return tuple(torch.empty((self.P, self.ld), dtype=torch.float32, device=device)
                     for _ in range(4))

    def alloc_placed(self):
        """w, g, m, pub as torch views of arrays that the library allocated with w, m and pub in
        different HBM regions (see wagma_alloc_buffers).  The library owns the memory: it lives
        until free_placed() or destroy(), and the tensors must not be used after that."""
        import torch
        ptrs = wagma_alloc_buffers(self.ctx)
        dev = torch.device("cuda", torch.cuda.current_device())
        return tuple(torch.as_tensor(_DeviceArray(p, (self.P, self.ld)), device=dev) for p in ptrs)

    def free_placed(self) -> None:
        wagma_free_buffers(self.ctx)

    def placement_info(self) -> dict:
        return wagma_placement_info(self.ctx)

    def _validate(self, *tensors) -> None:
        import torch
        ld = self.ld
        for t in tensors:
            if not isinstance(t, torch.Tensor):
                raise TypeError("expected torch tensors")
            if (t.dtype != torch.float32 or not t.is_cuda or t.dim() != 2
                    or t.shape[0] != self.P or t.shape[1] != ld or not t.is_contiguous()):
                raise ValueError("buffers must be contiguous CUDA fp32 tensors of shape (P, ld) = (%d, %d)"
                                 % (self.P, ld))

    def step(self, w, g, m, pub, stale_mask, lr: float, mu: float, it: int,
             stream: Optional[int] = None, busy_mask=None) -> None:
        """busy_mask given: wagma_step_lag (processes still computing an earlier step)."""
        self._validate(w, g, m, pub)
        for mask in (stale_mask, busy_mask):
            if mask is not None and len(mask) != (self.P + 63) // 64:
                raise ValueError("a mask must hold ceil(P/64) words")
        if busy_mask is None:
            wagma_step(self.ctx, w, g, m, pub, stale_mask, lr, mu, it, stream)
        else:
            wagma_step_lag(self.ctx, w, g, m, pub, stale_mask, busy_mask, lr, mu, it, stream)

    def tensor_plan(self, w, g, m, pub) -> "TensorPlan":
        """w, g, m, pub: for every process a list of T one-dimensional fp32 CUDA tensors
        (the same sizes in every process and every array)."""
        return TensorPlan(self, w, g, m, pub)

    def destroy(self) -> None:
        if self.ctx:
            wagma_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()


class TensorPlan:
    """Owns one wagma_tensors plan; keeps the tensors alive while the plan exists."""

    def __init__(self, owner: Wagma, w, g, m, pub):
        import torch
        self.owner = owner
        self.keep = (w, g, m, pub)
        sizes = [int(t.numel()) for t in w[0]]
        tables = []
        for arr in (w, g, m, pub):
            if len(arr) != owner.P:
                raise ValueError("one tensor list per process expected")
            flat = []
            for tensors in arr:
                if [int(t.numel()) for t in tensors] != sizes:
                    raise ValueError("every process and array must hold tensors of the same sizes")
                for t in tensors:
                    if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
                        raise ValueError("tensors must be contiguous CUDA fp32")
                    flat.append(t.data_ptr())
            tables.append(flat)
        self.plan = wagma_tensors_create(owner.ctx, sizes, *tables)

    def step(self, stale_mask, lr: float, mu: float, it: int, stream: Optional[int] = None,
             busy_mask=None) -> None:
        for mask in (stale_mask, busy_mask):
            if mask is not None and len(mask) != (self.owner.P + 63) // 64:
                raise ValueError("a mask must hold ceil(P/64) words")
        if busy_mask is None:
            wagma_step_tensors(self.owner.ctx, self.plan, stale_mask, lr, mu, it, stream)
        else:
            wagma_step_tensors_lag(self.owner.ctx, self.plan, stale_mask, busy_mask, lr, mu, it, stream)

    def destroy(self) -> None:
        if self.plan:
            wagma_tensors_destroy(self.plan)
            self.plan = None
            self.keep = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()
