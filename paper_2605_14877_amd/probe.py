"""ctypes binding of include/heatkv_probe.h (libheatkv_probe.so): measurement aids for bench.py and their tests.

Not part of the product path: nothing in binding.py or libheatkv.so depends on this module."""
from __future__ import annotations

import ctypes as C
import os

from . import binding
from .binding import HeatKVError, _check_tensor, _ptr, _stream

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libheatkv_probe.so")
_lib = None


def library_path():
    return _LIB_PATH


def lib():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is not built; run `python -m paper_2605_14877_amd.build`")
    binding.lib()  # imports torch first, so that both libraries bind to PyTorch's HIP runtime
    L = C.CDLL(_LIB_PATH)
    vp = C.c_void_p
    L.heatkv_probe_last_error.restype = C.c_char_p
    L.heatkv_probe_last_error.argtypes = []
    L.heatkv_probe_mfma_operand_bytes.restype = C.c_size_t
    L.heatkv_probe_mfma_operand_bytes.argtypes = []
    L.heatkv_probe_mfma.restype = C.c_int
    L.heatkv_probe_mfma.argtypes = [vp, vp, C.c_int, C.c_int, vp]
    L.heatkv_probe_tile_step_bytes.restype = C.c_size_t
    L.heatkv_probe_tile_step_bytes.argtypes = []
    L.heatkv_probe_tile_step.restype = C.c_int
    L.heatkv_probe_tile_step.argtypes = [vp, vp, C.c_int, C.c_int, vp]
    L.heatkv_probe_tile_stream_bytes.restype = C.c_size_t
    L.heatkv_probe_tile_stream_bytes.argtypes = [C.c_int, C.c_int]
    L.heatkv_probe_tile_stream.restype = C.c_int
    L.heatkv_probe_tile_stream.argtypes = [vp, C.c_size_t, vp, C.c_int, C.c_int, vp]
    _lib = L
    return L


def _check(rc):
    if rc != 0:
        raise HeatKVError(rc, lib().heatkv_probe_last_error().decode())


def heatkv_probe_mfma_operand_bytes():
    return int(lib().heatkv_probe_mfma_operand_bytes())


def heatkv_probe_mfma(operands, out, workgroups, iters, stream=None):
    """Back-to-back bf16 MFMAs on the caller's operand bits (see include/heatkv_probe.h)."""
    lib()
    _check_tensor(operands, "operands", min_bytes=heatkv_probe_mfma_operand_bytes())
    _check_tensor(out, "out", min_bytes=max(int(workgroups), 0) * 256 * 4)
    _check(lib().heatkv_probe_mfma(_ptr(operands), _ptr(out), int(workgroups), int(iters),
                                   _stream() if stream is None else stream))


def heatkv_probe_tile_step_bytes():
    return int(lib().heatkv_probe_tile_step_bytes())


def heatkv_probe_tile_step(tiles, out, workgroups, iters, stream=None):
    """A model of the bf16 attention kernel's tile step (see include/heatkv_probe.h)."""
    lib()
    _check_tensor(tiles, "tiles", min_bytes=heatkv_probe_tile_step_bytes())
    _check_tensor(out, "out", min_bytes=max(int(workgroups), 0) * 256 * 4)
    _check(lib().heatkv_probe_tile_step(_ptr(tiles), _ptr(out), int(workgroups), int(iters),
                                        _stream() if stream is None else stream))


def heatkv_probe_tile_stream_bytes(workgroups, steps):
    return int(lib().heatkv_probe_tile_stream_bytes(int(workgroups), int(steps)))


def heatkv_probe_tile_stream(src, out, workgroups, steps, stream=None):
    """The attention kernel's HBM -> LDS tile copies without arithmetic (see include/heatkv_probe.h)."""
    lib()
    _check_tensor(src, "src")
    _check_tensor(out, "out", min_bytes=max(int(workgroups), 0) * 256 * 4)
    src_bytes = 0 if src is None else src.numel() * src.element_size()
    _check(lib().heatkv_probe_tile_stream(_ptr(src), src_bytes, _ptr(out), int(workgroups), int(steps),
                                          _stream() if stream is None else stream))
