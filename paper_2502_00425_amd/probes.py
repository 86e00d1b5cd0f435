"""ctypes binding of libmquant_probes.so: the benchmark's measurement probes (an MFMA-only
loop, a read-only stream, an empty kernel).  They are instruments, not part of the method and
not part of the product's ABI; only bench.py and their own test load this module."""
from __future__ import annotations

import ctypes
import os

import torch  # noqa: F401  (before the HIP library, as in binding.py)

from . import binding as _b

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libmquant_probes.so")
EXPORTS = ("mqprobe_mfma_i8_ops", "mqprobe_mfma_i8", "mqprobe_hbm_read", "mqprobe_empty")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2502_00425_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    i32, i64, p = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
    lib.mqprobe_mfma_i8_ops.restype = i64
    lib.mqprobe_mfma_i8_ops.argtypes = [i32]
    lib.mqprobe_mfma_i8.argtypes = [i32, p, i64, p, p]
    lib.mqprobe_hbm_read.argtypes = [p, i64, p, p]
    lib.mqprobe_empty.argtypes = [i32, i32, p]
    return lib


lib = _load()


def mfma_i8(iters: int, data, sink) -> int:
    """Launches the MFMA-only loop; returns the int8 operations it performs."""
    _b._check(lib.mqprobe_mfma_i8(iters, data.data_ptr(), data.numel() * data.element_size(),
                                  sink.data_ptr(), _b._stream()), "mqprobe_mfma_i8")
    return int(lib.mqprobe_mfma_i8_ops(iters))


def hbm_read(data, sink) -> int:
    """Launches the read-only stream; returns the bytes it reads."""
    n = data.numel() * data.element_size()
    _b._check(lib.mqprobe_hbm_read(data.data_ptr(), n, sink.data_ptr(), _b._stream()), "mqprobe_hbm_read")
    return n


def empty(groups: int = 256, threads: int = 256) -> None:
    _b._check(lib.mqprobe_empty(groups, threads, _b._stream()), "mqprobe_empty")
