"""ctypes binding of the parallelism-selector table (include/earl_selector.h): argument
marshalling only, same names as the C functions without the `earl_` prefix."""
from __future__ import annotations

import ctypes as C
from typing import List, Sequence, Tuple

import numpy as np

from . import binding as _b

EXPORTED = ("earl_speedup_percent", "earl_selector_build", "earl_selector_n_ranges",
            "earl_selector_get_ranges", "earl_selector_best_at", "earl_selector_observe",
            "earl_selector_current_range", "earl_selector_destroy")
EARL_NO_FEASIBLE_CONFIG = 5

_ready = False


def _lib() -> C.CDLL:
    global _ready
    lib = _b.load_library()
    if not _ready:
        vp, i32, f64 = C.c_void_p, C.c_int32, C.c_double
        lib.earl_speedup_percent.argtypes = [f64, f64]
        lib.earl_speedup_percent.restype = f64
        lib.earl_selector_build.argtypes = [vp, i32, i32, vp, f64, i32, C.POINTER(vp)]
        lib.earl_selector_n_ranges.argtypes = [vp, C.POINTER(i32)]
        lib.earl_selector_get_ranges.argtypes = [vp, vp, vp]
        lib.earl_selector_best_at.argtypes = [vp, i32, C.POINTER(i32)]
        lib.earl_selector_observe.argtypes = [vp, f64, C.POINTER(i32), C.POINTER(i32)]
        lib.earl_selector_current_range.argtypes = [vp, C.POINTER(i32)]
        lib.earl_selector_destroy.argtypes = [vp]
        for name in EXPORTED[1:]:
            getattr(lib, name).restype = i32
        _ready = True
    return lib


def _check(status: int) -> None:
    if status != _b.EARL_OK:
        raise _b.EarlError(status, _lib().earl_status_string(status).decode())


def speedup_percent(tgs_a: float, tgs_b: float) -> float:
    return float(_lib().earl_speedup_percent(tgs_a, tgs_b))


class Selector:
    def __init__(self, handle: int, n_lengths: int):
        self.handle = handle
        self.n_lengths = n_lengths


def selector_build(context_lengths: Sequence[int], tgs, hysteresis: float = 0.0,
                   initial_config: int = -1) -> Selector:
    lengths = np.ascontiguousarray(context_lengths, dtype=np.int64)
    table = np.ascontiguousarray(tgs, dtype=np.float64)
    if table.ndim != 2 or table.shape[0] != lengths.shape[0]:
        raise ValueError("tgs must have one row per context length")
    out = C.c_void_p()
    _check(_lib().earl_selector_build(lengths.ctypes.data, lengths.shape[0], table.shape[1],
                                      table.ctypes.data, hysteresis, initial_config, C.byref(out)))
    return Selector(out.value, int(lengths.shape[0]))


def selector_n_ranges(sel: Selector) -> int:
    n = C.c_int32()
    _check(_lib().earl_selector_n_ranges(sel.handle, C.byref(n)))
    return n.value


def selector_get_ranges(sel: Selector) -> Tuple[List[int], List[int]]:
    n = selector_n_ranges(sel)
    hi = np.zeros((n,), dtype=np.int64)
    cfg = np.zeros((n,), dtype=np.int32)
    _check(_lib().earl_selector_get_ranges(sel.handle, hi.ctypes.data, cfg.ctypes.data))
    return hi.tolist(), cfg.tolist()


def selector_best_at(sel: Selector, j: int) -> int:
    k = C.c_int32()
    _check(_lib().earl_selector_best_at(sel.handle, j, C.byref(k)))
    return k.value


def selector_observe(sel: Selector, avg_context_length: float) -> Tuple[int, bool]:
    """Returns (configuration, switched); raises EarlError with EARL_NO_FEASIBLE_CONFIG if every
    configuration failed in the range the length falls into."""
    k, sw = C.c_int32(), C.c_int32()
    _check(_lib().earl_selector_observe(sel.handle, avg_context_length, C.byref(k), C.byref(sw)))
    return k.value, bool(sw.value)


def selector_current_range(sel: Selector) -> int:
    t = C.c_int32()
    _check(_lib().earl_selector_current_range(sel.handle, C.byref(t)))
    return t.value


def selector_destroy(sel: Selector) -> None:
    if sel.handle:
        _check(_lib().earl_selector_destroy(sel.handle))
        sel.handle = None
