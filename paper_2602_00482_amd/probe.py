"""ctypes binding for include/dta_probe.h (libdta_probe.so): the two measurement
kernels the benchmark uses.  Not part of the attention library."""
from __future__ import annotations

import ctypes as C
import os

from .binding import _check, _ptr, _stream

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdta_probe.so")
_lib = None

exported_symbols = ["dta_probe_mfma_bf16", "dta_probe_overlap"]


def load_library():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} not found: run `python -m paper_2602_00482_amd.build` first")
        lib = C.CDLL(_LIB_PATH)
        vp = C.c_void_p
        lib.dta_probe_mfma_bf16.argtypes = [C.c_int32, C.c_int32, vp, vp, vp, C.POINTER(C.c_int64),
                                            C.POINTER(C.c_int32)]
        lib.dta_probe_mfma_bf16.restype = C.c_int
        lib.dta_probe_overlap.argtypes = [C.c_int32, C.c_int32, C.c_int32, vp, vp]
        lib.dta_probe_overlap.restype = C.c_int
        _lib = lib
    return _lib


def probe_mfma_bf16(n_blocks: int, iters: int, out, ticks):
    """dta_probe_mfma_bf16: enqueues the matrix-pipe rate probe; out is a device
    fp32 tensor of n_blocks*256 elements, ticks a device int64 tensor of
    2*n_blocks; runs on torch's current stream.  Returns (floating-point operations of the launch,
    rate of the wall-clock counter in kHz)."""
    if out.numel() < n_blocks * 256 or ticks.numel() < 2 * n_blocks or ticks.element_size() != 8:
        raise ValueError("probe buffers too small")
    flop, khz = C.c_int64(), C.c_int32()
    _check(load_library().dta_probe_mfma_bf16(int(n_blocks), int(iters), _ptr(out), _ptr(ticks), _stream(),
                                              C.byref(flop), C.byref(khz)), "dta_probe_mfma_bf16")
    return int(flop.value), int(khz.value)


def probe_overlap(n_blocks: int, mfma_iters: int, valu_iters: int, out):
    """dta_probe_overlap on torch's current stream; out is a device fp32 tensor
    of n_blocks*512 elements."""
    if out.numel() < n_blocks * 512:
        raise ValueError("probe buffer too small")
    _check(load_library().dta_probe_overlap(int(n_blocks), int(mfma_iters), int(valu_iters), _ptr(out), _stream()),
           "dta_probe_overlap")
