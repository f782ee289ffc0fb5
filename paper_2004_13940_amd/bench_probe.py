"""ctypes loader of libfm_bench_probe.so: calibration probes for bench.py (a random-row gather rate and a
plain copy of known size).  Not part of the method; the product library does not contain them."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfm_bench_probe.so")
_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2004_13940_amd.build`")
        import torch  # noqa: F401  (the HIP runtime torch ships must be the one this library binds to)
        _lib = ctypes.CDLL(LIB_PATH)
    return _lib


def _stream(stream):
    import torch
    return ctypes.c_void_p((stream or torch.cuda.current_stream()).cuda_stream)


def gather_rate(buffer_bytes, row_bytes=128, stream=None) -> float:
    """Rows of ``row_bytes`` (64 or 128) read per second from pseudo-random places of a zeroed device buffer of
    ``buffer_bytes`` (1 MiB .. 64 GiB) that the call allocates and frees; waits for the stream."""
    out = ctypes.c_double(0.0)
    rc = load().bench_probe_gather(ctypes.c_int64(int(buffer_bytes)), ctypes.c_int32(int(row_bytes)), ctypes.byref(out),
                                   _stream(stream))
    if rc != 0:
        raise RuntimeError(f"bench_probe_gather failed with status {rc}")
    return out.value


def copy(src, dst, reps=1, stream=None) -> None:
    """``reps`` plain kernel copies of the CUDA tensor ``src`` into ``dst`` (same size, a multiple of 16 bytes)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst differ in size")
    rc = load().bench_probe_copy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), ctypes.c_int64(nbytes),
                                 ctypes.c_int32(int(reps)), _stream(stream))
    if rc != 0:
        raise RuntimeError(f"bench_probe_copy failed with status {rc}")
