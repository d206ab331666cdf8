"""Streams restricted to a subset of the compute units, for callers that share the GPU.

The paper's router runs on the same GPU as the LLM serving instances (Sec. 1, Sec. 4.1.1).
The attention library launches on whatever stream it is given and assumes nothing about how
many compute units that stream may use, so a caller that wants to leave part of the chip to
another tenant passes a stream created with a CU mask.  This module wraps the two HIP runtime
calls needed for that (stream creation with a mask, destruction); it contains no part of the
attention computation.
"""
from __future__ import annotations

import ctypes

_hip = None


def _runtime():
    global _hip
    if _hip is None:
        lib = ctypes.CDLL("libamdhip64.so")
        lib.hipExtStreamCreateWithCUMask.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint32,
                                                     ctypes.POINTER(ctypes.c_uint32)]
        lib.hipExtStreamCreateWithCUMask.restype = ctypes.c_int
        lib.hipStreamDestroy.argtypes = [ctypes.c_void_p]
        lib.hipStreamDestroy.restype = ctypes.c_int
        lib.hipStreamSynchronize.argtypes = [ctypes.c_void_p]
        lib.hipStreamSynchronize.restype = ctypes.c_int
        _hip = lib
    return _hip


class CuMaskedStream:
    """A HIP stream (default priority) whose kernels run only on the compute units whose bit is
    set in `mask_words` (32 units per word, lowest bit first).  `handle` is the raw hipStream_t
    as an integer, which the binding's `stream=` argument accepts.  Use as a context manager, or
    call close(); the stream is synchronised before it is destroyed."""

    def __init__(self, mask_words):
        words = [int(w) & 0xFFFFFFFF for w in mask_words]
        if not words or not any(words):
            raise ValueError("a CU mask needs at least one enabled unit")
        arr = (ctypes.c_uint32 * len(words))(*words)
        s = ctypes.c_void_p()
        rc = _runtime().hipExtStreamCreateWithCUMask(ctypes.byref(s), len(words), arr)
        if rc != 0 or not s.value:
            raise RuntimeError(f"hipExtStreamCreateWithCUMask failed with HIP error {rc}")
        self.handle = int(s.value)

    def synchronize(self):
        rc = _runtime().hipStreamSynchronize(ctypes.c_void_p(self.handle))
        if rc != 0:
            raise RuntimeError(f"hipStreamSynchronize failed with HIP error {rc}")

    def close(self):
        if self.handle:
            self.synchronize()
            _runtime().hipStreamDestroy(ctypes.c_void_p(self.handle))
            self.handle = 0

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
        return False


def first_units(count: int, total: int = 256):
    """Mask words enabling compute units 0 .. count-1 of `total`."""
    if not 0 < count <= total:
        raise ValueError("count must be in 1..total")
    words = []
    for w in range((total + 31) // 32):
        bits = min(max(count - 32 * w, 0), 32)
        words.append((1 << bits) - 1 if bits < 32 else 0xFFFFFFFF)
    return words
