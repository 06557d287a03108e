"""ctypes front end of the plain-C CPU oracle (``wagma_oracle.c``).

TEST INFRASTRUCTURE ONLY: used by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  Nothing in the product package imports it,
and it imports nothing from the product package.

Arrays are numpy, row-major ``(P, ld)`` with ``n <= ld`` used columns, updated
in place exactly as Algorithm 2 (lines 6-17) of the paper updates W, the
momentum state and the send buffer.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "wagma_oracle.c")
_LIB = os.path.join(_HERE, "libwagma_oracle.so")

# No contraction, no fast-math: the oracle is IEEE fp32 with explicit fmaf.
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c99", "-Wall",
          "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (always when ``force``), return the path."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def bind(lib: ctypes.CDLL) -> ctypes.CDLL:
    """Attach the C signatures to a loaded oracle library."""
    i32p = ctypes.POINTER(ctypes.c_int32)
    u64p = ctypes.POINTER(ctypes.c_uint64)
    f32p = ctypes.POINTER(ctypes.c_float)
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.oracle_grouping_unionfind.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, i32p]
    lib.oracle_member_table.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, i32p]
    lib.oracle_is_global_iteration.argtypes = [ctypes.c_int, ctypes.c_int64]
    lib.oracle_step_f32.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                    ctypes.c_int, ctypes.c_int64, f32p, f32p, f32p, f32p, u64p,
                                    ctypes.c_float, ctypes.c_float, ctypes.c_int]
    lib.oracle_step_f64.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                    ctypes.c_int, ctypes.c_int64, f64p, f64p, f64p, f64p, u64p,
                                    ctypes.c_double, ctypes.c_double, ctypes.c_int]
    lib.oracle_step_lag_f32.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_int, ctypes.c_int64, f32p, f32p, f32p, f32p, u64p, u64p,
                                        ctypes.c_float, ctypes.c_float, ctypes.c_int]
    lib.oracle_step_lag_f64.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_int, ctypes.c_int64, f64p, f64p, f64p, f64p, u64p, u64p,
                                        ctypes.c_double, ctypes.c_double, ctypes.c_int]
    lib.oracle_lag_states.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_uint32),
                                      ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint8)]
    lib.oracle_lag_masks.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_int, ctypes.c_uint32, u64p, u64p]
    for f in (lib.oracle_step_lag_f32, lib.oracle_step_lag_f64, lib.oracle_lag_states,
              lib.oracle_lag_masks):
        f.restype = ctypes.c_int
    lib.oracle_stale_mask.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int,
                                      ctypes.c_uint32, u64p]
    lib.oracle_straggler_mask.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int, ctypes.c_int, u64p]
    lib.oracle_clock_mask.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32, u64p,
                                      ctypes.POINTER(ctypes.c_uint32)]
    lib.oracle_straggler_mask.restype = lib.oracle_clock_mask.restype = ctypes.c_int
    for f in (lib.oracle_grouping_unionfind, lib.oracle_member_table,
              lib.oracle_is_global_iteration, lib.oracle_step_f32,
              lib.oracle_step_f64, lib.oracle_stale_mask):
        f.restype = ctypes.c_int
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = bind(ctypes.CDLL(build()))
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError("%s failed with oracle error %d" % (what, rc))


def grouping_unionfind(P: int, S: int, t: int) -> np.ndarray:
    """Algorithm 1 run literally; entry p = smallest member of p's group."""
    rep = np.empty(P, dtype=np.int32)
    _check(_load().oracle_grouping_unionfind(
        P, S, t, rep.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))), "grouping_unionfind")
    return rep


def member_table(P: int, S: int, t: int) -> np.ndarray:
    """(P/S, S) table: ordered members of every group of iteration t."""
    table = np.empty(P, dtype=np.int32)
    _check(_load().oracle_member_table(
        P, S, t, table.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))), "member_table")
    return table.reshape(P // S, S)


def is_global_iteration(tau: int, t: int) -> bool:
    return bool(_load().oracle_is_global_iteration(tau, t))


def mask_words(stale) -> np.ndarray | None:
    """Pack an iterable of late ranks / a bool vector / uint64 words into words."""
    if stale is None:
        return None
    a = np.asarray(stale)
    if a.dtype == np.uint64:
        return np.ascontiguousarray(a)
    if a.dtype == np.bool_:
        ranks = np.nonzero(a)[0]
        P = a.size
    else:
        raise TypeError("stale must be None, a bool vector of length P or uint64 words")
    words = np.zeros((P + 63) // 64, dtype=np.uint64)
    for p in ranks:
        words[p >> 6] |= np.uint64(1) << np.uint64(p & 63)
    return words


def _step(fn, ctype, dtype, P, S, tau, t, w, g, m, pub, stale, lr, mu, n=None, fixed_groups=False,
          busy=None):
    for name, a in (("w", w), ("g", g), ("m", m), ("pub", pub)):
        if a.dtype != dtype or a.ndim != 2 or a.shape[0] != P or not a.flags.c_contiguous:
            raise ValueError("%s must be a C-contiguous (P, ld) %s array" % (name, dtype))
        if a.shape != w.shape:
            raise ValueError("w, g, m, pub must share one shape")
    ld = w.shape[1]
    n = ld if n is None else n
    words = mask_words(stale)
    busy_words = mask_words(busy)
    for a in (words, busy_words):
        if a is not None and a.size != (P + 63) // 64:
            raise ValueError("a mask must hold ceil(P/64) words")
    ptr = ctypes.POINTER(ctype)
    u64p = ctypes.POINTER(ctypes.c_uint64)
    _check(fn(P, S, n, ld, tau, t,
              w.ctypes.data_as(ptr), g.ctypes.data_as(ptr), m.ctypes.data_as(ptr),
              pub.ctypes.data_as(ptr),
              None if words is None else words.ctypes.data_as(u64p),
              None if busy_words is None else busy_words.ctypes.data_as(u64p),
              lr, mu, 1 if fixed_groups else 0), "step")


def _plain(fn):
    """Adapts oracle_step_f32/_f64 (no busy mask) to the argument list _step passes."""
    def call(P, S, n, ld, tau, t, w, g, m, pub, words, busy_words, lr, mu, fixed):
        assert busy_words is None
        return fn(P, S, n, ld, tau, t, w, g, m, pub, words, lr, mu, fixed)
    return call


def step_f32(P, S, tau, t, w, g, m, pub, stale, lr, mu, n=None, fixed_groups=False) -> None:
    """One iteration of Algorithm 2 (lines 6-17) in fp32, in place.
    fixed_groups: the groups of iteration 0 every time (Section 6.2, second ablation)."""
    _step(_plain(_load().oracle_step_f32), ctypes.c_float, np.float32,
          P, S, tau, t, w, g, m, pub, stale, lr, mu, n, fixed_groups)


def step_f64(P, S, tau, t, w, g, m, pub, stale, lr, mu, n=None, fixed_groups=False) -> None:
    """The same iteration carried in fp64 (rounding shadow)."""
    _step(_plain(_load().oracle_step_f64), ctypes.c_double, np.float64,
          P, S, tau, t, w, g, m, pub, stale, lr, mu, n, fixed_groups)


def step_lag_f32(P, S, tau, t, w, g, m, pub, stale, busy, lr, mu, n=None, fixed_groups=False) -> None:
    """The iteration when the processes of ``busy`` are still computing an earlier step:
    they contribute their send buffer again and nothing of them changes."""
    _step(_load().oracle_step_lag_f32, ctypes.c_float, np.float32,
          P, S, tau, t, w, g, m, pub, stale, lr, mu, n, fixed_groups, busy)


def step_lag_f64(P, S, tau, t, w, g, m, pub, stale, busy, lr, mu, n=None, fixed_groups=False) -> None:
    _step(_load().oracle_step_lag_f64, ctypes.c_double, np.float64,
          P, S, tau, t, w, g, m, pub, stale, lr, mu, n, fixed_groups, busy)


def stale_mask(seed: int, t: int, P: int, threshold: int) -> np.ndarray:
    """uint64 words, bit p set = process p late in iteration t."""
    words = np.zeros((P + 63) // 64, dtype=np.uint64)
    _check(_load().oracle_stale_mask(
        seed, t, P, threshold, words.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64))),
        "stale_mask")
    return words


def straggler_mask(seed: int, t: int, P: int, count: int) -> np.ndarray:
    """Exactly ``count`` randomly selected late processes (Section 6.2 selects two per step)."""
    words = np.zeros((P + 63) // 64, dtype=np.uint64)
    _check(_load().oracle_straggler_mask(
        seed, t, P, count, words.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64))), "straggler_mask")
    return words


def clock_mask(seed: int, t: int, P: int, tolerance_ms: int):
    """(mask words, step times in ms): late = more than tolerance_ms behind the fastest process."""
    words = np.zeros((P + 63) // 64, dtype=np.uint64)
    ms = np.zeros(P, dtype=np.uint32)
    _check(_load().oracle_clock_mask(
        seed, t, P, tolerance_ms, words.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
        ms.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32))), "clock_mask")
    return words, ms


FRESH, LATE, BUSY = 0, 1, 2


def lag_states(step_ms: np.ndarray, tolerance_ms: int) -> np.ndarray:
    """(K, P) states of K iterations after a global one, from (K+1, P) step times in ms:
    FRESH, LATE (finishes before the next group allreduce reads its send buffer) or BUSY."""
    step_ms = np.ascontiguousarray(step_ms, dtype=np.uint32)
    K, P = step_ms.shape[0] - 1, step_ms.shape[1]
    states = np.zeros((K, P), dtype=np.uint8)
    _check(_load().oracle_lag_states(
        P, K, step_ms.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), tolerance_ms,
        states.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))), "lag_states")
    return states


def lag_masks(seed: int, t: int, P: int, tau: int, window: int, tolerance_ms: int):
    """(late words, busy words) of iteration t when steps run back to back between global
    iterations (every ``window`` iterations when tau == 0) with clock_mask's step times."""
    late = np.zeros((P + 63) // 64, dtype=np.uint64)
    busy = np.zeros((P + 63) // 64, dtype=np.uint64)
    u64p = ctypes.POINTER(ctypes.c_uint64)
    _check(_load().oracle_lag_masks(seed, t, P, tau, window, tolerance_ms,
                                    late.ctypes.data_as(u64p), busy.ctypes.data_as(u64p)), "lag_masks")
    return late, busy
