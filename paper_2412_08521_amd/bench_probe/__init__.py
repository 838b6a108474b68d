"""Thin ctypes binding of libems_probe.so: the benchmark's ceiling measurements (ems_probe.h).
Not part of the product library."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(os.path.dirname(_HERE), "libems_probe.so")
OPERAND_BYTES = 65536
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2412_08521_amd.build`")
        l = C.CDLL(LIB_PATH)
        l.ems_probe_mfma.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        l.ems_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        _lib = l
    return _lib


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def probe_mfma(blocks: int, iters: int, sink, operands=None):
    """Enqueue the MFMA ceiling kernel; returns the flops it performs."""
    if not (sink.is_cuda and sink.dtype == torch.float32 and sink.numel() == blocks * 256):
        raise ValueError("sink must be a device float32 tensor of blocks * 256 elements")
    op = None
    if operands is not None:
        if not (operands.is_cuda and operands.is_contiguous()
                and operands.numel() * operands.element_size() >= OPERAND_BYTES):
            raise ValueError("operands must be a contiguous device tensor of at least 64 KiB")
        op = C.c_void_p(operands.data_ptr())
    rc = lib().ems_probe_mfma(int(blocks), int(iters), op, C.c_void_p(sink.data_ptr()), _stream())
    if rc != 0:
        raise RuntimeError(f"ems_probe_mfma failed ({rc})")
    return blocks * 4 * iters * 32 * 32768


def probe_copy(src, dst):
    """Enqueue the copy ceiling kernel; returns the bytes it moves (read + written)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (src.is_cuda and dst.is_cuda):
        raise ValueError("src and dst must be device tensors of the same size")
    rc = lib().ems_probe_copy(C.c_void_p(src.data_ptr()), C.c_void_p(dst.data_ptr()), nbytes, _stream())
    if rc != 0:
        raise RuntimeError(f"ems_probe_copy failed ({rc})")
    return 2 * nbytes
