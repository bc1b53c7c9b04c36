"""Benchmark-only binding of the per-kernel timing calls of liblss_attn.so (csrc/lss_timing.h).

Not part of the product interface: bench.py uses it to bracket kernels with HIP events on their
launch stream.
"""
from __future__ import annotations

import ctypes

from . import lss

_ready = False


def _lib():
    global _ready
    lib = lss.load()
    if not _ready:
        ci, i64 = ctypes.c_int, ctypes.c_int64
        lib.lss_timing_enable.argtypes = [ci]
        lib.lss_timing_select.argtypes = [ctypes.c_uint64]
        lib.lss_timing_read.argtypes = [ci, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        lib.lss_timing_kernel_name.argtypes = [ci]
        lib.lss_timing_kernel_name.restype = ctypes.c_char_p
        for name in ("lss_timing_enable", "lss_timing_select", "lss_timing_reset", "lss_timing_read"):
            getattr(lib, name).restype = ci
        _ready = True
    return lib


def enable(on: bool) -> None:
    lss._check(_lib().lss_timing_enable(int(bool(on))))


def select(kernel_ids) -> None:
    """Record only the kernels whose ids are listed (an empty list records nothing)."""
    mask = 0
    for k in kernel_ids:
        mask |= 1 << int(k)
    lss._check(_lib().lss_timing_select(mask))


def reset() -> None:
    lss._check(_lib().lss_timing_reset())


def kernel_name(kernel_id: int):
    name = _lib().lss_timing_kernel_name(kernel_id)
    return name.decode() if name else None


def kernel_names() -> dict:
    """{id: name} of every kernel the library can time."""
    out, kid = {}, 0
    while (name := kernel_name(kid)) is not None:
        out[kid] = name
        kid += 1
    return out


def read(kernel_id: int):
    """(total milliseconds, launches) of kernel `kernel_id` since the last reset."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
    lss._check(_lib().lss_timing_read(kernel_id, ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value
