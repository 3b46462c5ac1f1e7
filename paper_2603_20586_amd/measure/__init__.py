"""Measurement helpers (not product surface): the reference micro-benchmarks of
include/mka_measure.h in their own library, and the rocprofv3 summariser behind profiles/.
Only bench.py and the people who regenerate profiles/ use this sub-package."""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_int32, c_size_t, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmka_measure.so")
_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with "
                              "`python -m paper_2603_20586_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        L.mka_measure_mfma_loop.restype = c_int32
        L.mka_measure_mfma_loop.argtypes = [c_void_p, c_int32, c_int32,
                                            POINTER(ctypes.c_double), c_void_p]
        L.mka_measure_mfma_loop_data.restype = c_int32
        L.mka_measure_mfma_loop_data.argtypes = [c_void_p, c_void_p, c_int32, c_int32,
                                                 POINTER(ctypes.c_double), c_void_p]
        L.mka_measure_stream_read.restype = c_int32
        L.mka_measure_stream_read.argtypes = [c_void_p, c_size_t, c_void_p, c_void_p]
        _lib = L
    return _lib


def _stream():
    import torch

    return c_void_p(torch.cuda.current_stream().cuda_stream)


def mfma_loop(out, workgroups: int, iters: int) -> float:
    """Enqueue the pure-MFMA loop; returns the flops of the launch."""
    fl = ctypes.c_double(0.0)
    rc = lib().mka_measure_mfma_loop(c_void_p(out.data_ptr()), workgroups, iters,
                                     ctypes.byref(fl), _stream())
    if rc:
        raise RuntimeError(f"mka_measure_mfma_loop: status {rc}")
    return fl.value


FRAG_BYTES = 16 * 512 * 16


def mfma_loop_data(out, frags, workgroups: int, iters: int) -> float:
    """Enqueue the MFMA loop on the operand fragments in `frags` (FRAG_BYTES bytes of bf16 on the
    device); returns the flops of the launch."""
    if frags.numel() * frags.element_size() < FRAG_BYTES:
        raise ValueError("frags is smaller than FRAG_BYTES")
    fl = ctypes.c_double(0.0)
    rc = lib().mka_measure_mfma_loop_data(c_void_p(out.data_ptr()), c_void_p(frags.data_ptr()),
                                          workgroups, iters, ctypes.byref(fl), _stream())
    if rc:
        raise RuntimeError(f"mka_measure_mfma_loop_data: status {rc}")
    return fl.value


def stream_read(src) -> int:
    """Enqueue the streaming read of `src`; returns the bytes it reads."""
    nbytes = src.numel() * src.element_size()
    rc = lib().mka_measure_stream_read(c_void_p(src.data_ptr()), nbytes, None, _stream())
    if rc:
        raise RuntimeError(f"mka_measure_stream_read: status {rc}")
    return (nbytes // 16 // 6 // 1024 * 1024) * 16 * 6
