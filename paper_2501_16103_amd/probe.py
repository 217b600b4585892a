"""ctypes binding of libmoe_probe (measurement kernels, see include/moe_probe.h): argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_probe.so")
EXPORTS = ["moe_probe_mfma", "moe_probe_pipeline", "moe_probe_wave_placement"]

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2501_16103_amd.build`.")
        L = ctypes.CDLL(LIB_PATH)
        L.moe_probe_mfma.restype = ctypes.c_int
        L.moe_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.moe_probe_pipeline.restype = ctypes.c_int
        L.moe_probe_pipeline.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                         ctypes.c_void_p]
        L.moe_probe_wave_placement.restype = ctypes.c_int
        L.moe_probe_wave_placement.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        _lib = L
    return _lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def moe_probe_mfma(block: int, random_operands: bool, iters: int, sink) -> int:
    """One launch of the pure-MFMA probe; FLOPs = 256 * 8 * iters * 524288.  `sink`: device tensor of >= 4 bytes."""
    return int(lib().moe_probe_mfma(int(block), int(bool(random_operands)), int(iters), _ptr(sink),
                                    _stream() if sink is not None else None))


def moe_probe_pipeline(mode: int, iters: int, src, sink) -> int:
    """One launch of the tile-loop probe (modes 1-12, see the header); `src`: device tensor of >= 1 MiB (modes 4
    and 12: 513 MiB) holding bf16 values."""
    nbytes = 0 if src is None else src.numel() * src.element_size()
    return int(lib().moe_probe_pipeline(int(mode), int(iters), _ptr(src), ctypes.c_size_t(nbytes), _ptr(sink),
                                        _stream() if sink is not None and src is not None else None))


def moe_probe_wave_placement(workgroups: int, out) -> int:
    """out[8 * g + w] = SIMD of wavefront w of workgroup g (512-thread workgroups, one per CU); `out`: int32 device
    tensor of workgroups * 8 elements."""
    if out is not None and (out.dtype != torch.int32 or out.numel() < workgroups * 8):
        raise ValueError("out must be an int32 tensor of workgroups * 8 elements")
    return int(lib().moe_probe_wave_placement(int(workgroups), _ptr(out), _stream() if out is not None else None))
