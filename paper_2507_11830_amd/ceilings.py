"""Binding of libspceilings.so — the benchmark's two reference kernels (a register-resident bf16
MFMA loop and a streaming read), declared in ``include/sp_ceilings.h``.  Measurement aids only:
the attention library neither contains nor uses them, and nothing but the benchmark loads this."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspceilings.so")
EXPORTS = ("spc_ceiling_mfma", "spc_ceiling_stream", "spc_last_error")

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2507_11830_amd.build` first")
        import torch  # noqa: F401  (its HIP runtime must be in the process first)

        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        L.spc_ceiling_mfma.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_double), vp, sz, vp]
        L.spc_ceiling_mfma.restype = ctypes.c_int
        L.spc_ceiling_stream.argtypes = [vp, sz, i32, i32, vp, sz, vp]
        L.spc_ceiling_stream.restype = ctypes.c_int
        L.spc_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != 0:
        raise RuntimeError(f"libspceilings ({rc}): {lib().spc_last_error().decode()}")


def _stream(stream):
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def ceiling_mfma(iters: int, sink, random_operands: bool = False, stream=None) -> float:
    """Enqueues the MFMA-only reference loop; returns the flops it performs.  `sink`: cuda uint8 tensor."""
    flops = ctypes.c_double(0.0)
    _check(lib().spc_ceiling_mfma(int(iters), int(bool(random_operands)), ctypes.byref(flops), sink.data_ptr(),
                                  sink.numel() * sink.element_size(), _stream(stream)))
    return flops.value


def ceiling_stream(buf, sink, blocks_per_cu: int = 8, unroll: int = 4, stream=None) -> int:
    """Enqueues the streaming-read reference kernel over all of `buf`; returns the bytes it reads."""
    nbytes = buf.numel() * buf.element_size()
    _check(lib().spc_ceiling_stream(buf.data_ptr(), nbytes, int(blocks_per_cu), int(unroll), sink.data_ptr(),
                                    sink.numel() * sink.element_size(), _stream(stream)))
    return nbytes
