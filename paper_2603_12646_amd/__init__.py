"""Thin ctypes binding over libfa_mi355x.so (the C boundary in include/fa.h).

Argument marshalling only: every step of the attention forward runs in the HIP
kernels.  torch tensors are used as handles to device memory and for the current
stream; raw integer device pointers are accepted as well.  There is no fallback:
if the shared library has not been built, importing the compute entry points
raises.
"""
from __future__ import annotations

import ctypes
import os

__all__ = [
    "fa_fwd", "fa_fwd_bf16", "fa_fwd_ex", "fa_workspace_bytes", "fa_rope_scratch_bytes", "fa_strerror", "fa_version",
    "FA_STATIC_SCRATCH_BYTES",
    "FaParams", "FaError", "load_library", "LIB_PATH",
    "FA_DTYPE_F16", "FA_DTYPE_BF16",
    "FA_TUNE_BM_128", "FA_TUNE_BM_256", "FA_TUNE_BM_32", "FA_TUNE_BM_384", "FA_TUNE_BM_512", "FA_TUNE_BM_MIXED", "FA_TUNE_V_LDS_TRANSPOSE", "FA_TUNE_V_SCALAR",
    "FA_TUNE_MAP_LINEAR", "FA_TUNE_MAP_XCD", "FA_TUNE_WIN_PIPELINED", "FA_TUNE_WIN_TWO_PHASE",
]

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfa_mi355x.so")

FA_DTYPE_F16, FA_DTYPE_BF16 = 0, 1
FA_TUNE_BM_128, FA_TUNE_BM_256, FA_TUNE_BM_32 = 0x1, 0x2, 0x3
FA_TUNE_BM_384, FA_TUNE_BM_512, FA_TUNE_BM_MIXED = 0x4, 0x5, 0x6
FA_TUNE_V_LDS_TRANSPOSE, FA_TUNE_V_SCALAR = 0x10, 0x20
FA_TUNE_MAP_LINEAR, FA_TUNE_MAP_XCD = 0x100, 0x200
FA_TUNE_WIN_PIPELINED, FA_TUNE_WIN_TWO_PHASE = 0x1000, 0x2000


class FaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"fa error {code}: {message}")
        self.code = code


class FaParams(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("dtype", ctypes.c_int32),
        ("q", ctypes.c_void_p),
        ("k", ctypes.c_void_p),
        ("v", ctypes.c_void_p),
        ("o", ctypes.c_void_p),
        ("lse", ctypes.c_void_p),
        ("seq_lens", ctypes.c_void_p),
        ("batch", ctypes.c_int32),
        ("heads", ctypes.c_int32),
        ("max_len", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("window_left", ctypes.c_int32),
        ("window_right", ctypes.c_int32),
        ("q_strides", ctypes.c_int64 * 3),
        ("k_strides", ctypes.c_int64 * 3),
        ("v_strides", ctypes.c_int64 * 3),
        ("o_strides", ctypes.c_int64 * 3),
        ("stream", ctypes.c_void_p),
        ("tuning", ctypes.c_uint32),
        ("key_bias", ctypes.c_void_p),
        ("key_bias_stride", ctypes.c_int64),
        ("rope_cos", ctypes.c_void_p),
        ("rope_sin", ctypes.c_void_p),
        ("rope_stride", ctypes.c_int64),
        ("scratch", ctypes.c_void_p),
        ("scratch_bytes", ctypes.c_size_t),
    ]


_lib = None


def load_library():
    """dlopen the in-tree shared library and declare its prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2603_12646_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    simple = [ctypes.c_void_p] * 4 + [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_int,
                                      ctypes.c_void_p]
    for name in ("fa_fwd", "fa_fwd_bf16"):
        fn = getattr(lib, name)
        fn.argtypes = simple
        fn.restype = ctypes.c_int
    lib.fa_fwd_ex.argtypes = [ctypes.POINTER(FaParams)]
    lib.fa_fwd_ex.restype = ctypes.c_int
    lib.fa_fwd_ex_static_scratch.argtypes = [ctypes.POINTER(FaParams)]
    lib.fa_fwd_ex_static_scratch.restype = ctypes.c_int
    for name in ("fa_workspace_bytes", "fa_rope_scratch_bytes"):
        fn = getattr(lib, name)
        fn.argtypes = [ctypes.c_int] * 4
        fn.restype = ctypes.c_size_t
    lib.fa_strerror.argtypes = [ctypes.c_int]
    lib.fa_strerror.restype = ctypes.c_char_p
    lib.fa_version.argtypes = []
    lib.fa_version.restype = ctypes.c_int
    _lib = lib
    return lib


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()  # torch tensor


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def fa_strerror(code: int) -> str:
    return load_library().fa_strerror(int(code)).decode()


def fa_version() -> int:
    return int(load_library().fa_version())


def fa_workspace_bytes(batch: int, heads: int, max_len: int, head_dim: int) -> int:
    return int(load_library().fa_workspace_bytes(batch, heads, max_len, head_dim))


def fa_rope_scratch_bytes(batch: int, heads: int, max_len: int, head_dim: int) -> int:
    return int(load_library().fa_rope_scratch_bytes(batch, heads, max_len, head_dim))


FA_STATIC_SCRATCH_BYTES = 64 << 20


def _check(rc: int, check: bool) -> int:
    if check and rc != 0:
        raise FaError(rc, fa_strerror(rc))
    return rc


def _call_simple(name, q, k, v, o, lse, batch, heads, seq_lens, max_len, head_dim, scale, window,
                 stream, check):
    lib = load_library()
    rc = getattr(lib, name)(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), batch, heads,
                            _ptr(seq_lens), max_len, head_dim, scale, window, _stream(stream))
    return _check(rc, check)


def fa_fwd(q, k, v, o, lse, batch, heads, seq_lens, max_len, head_dim, scale, window=-1,
           stream=None, check=True):
    """fp16 forward; same argument order as the C function.  Tensors or int pointers."""
    return _call_simple("fa_fwd", q, k, v, o, lse, batch, heads, seq_lens, max_len, head_dim,
                        scale, window, stream, check)


def fa_fwd_bf16(q, k, v, o, lse, batch, heads, seq_lens, max_len, head_dim, scale, window=-1,
                stream=None, check=True):
    """bf16 forward; same argument order as the C function."""
    return _call_simple("fa_fwd_bf16", q, k, v, o, lse, batch, heads, seq_lens, max_len, head_dim,
                        scale, window, stream, check)


def fa_fwd_ex(*, dtype, q, k, v, o, lse=None, seq_lens=None, batch, heads, max_len, head_dim=64,
              scale, window_left=-1, window_right=-1, q_strides=None, k_strides=None,
              v_strides=None, o_strides=None, stream=None, tuning=0, key_bias=None,
              key_bias_stride=0, rope_cos=None, rope_sin=None, rope_stride=0, scratch=None, scratch_bytes=0,
              static_scratch=False, check=True):
    """Fill an fa_params struct and call fa_fwd_ex (static_scratch: fa_fwd_ex_static_scratch)."""
    p = FaParams()
    p.struct_size = ctypes.sizeof(FaParams)
    p.dtype = dtype
    p.q, p.k, p.v, p.o = _ptr(q), _ptr(k), _ptr(v), _ptr(o)
    p.lse, p.seq_lens = _ptr(lse), _ptr(seq_lens)
    p.batch, p.heads, p.max_len, p.head_dim = batch, heads, max_len, head_dim
    p.scale = scale
    p.window_left, p.window_right = window_left, window_right
    for name, val in (("q_strides", q_strides), ("k_strides", k_strides),
                      ("v_strides", v_strides), ("o_strides", o_strides)):
        arr = getattr(p, name)
        for i in range(3):
            arr[i] = 0 if val is None else int(val[i])
    p.stream = _stream(stream)
    p.tuning = tuning
    p.key_bias, p.key_bias_stride = _ptr(key_bias), key_bias_stride
    p.rope_cos, p.rope_sin, p.rope_stride = _ptr(rope_cos), _ptr(rope_sin), rope_stride
    p.scratch, p.scratch_bytes = _ptr(scratch), scratch_bytes
    lib = load_library()
    fn = lib.fa_fwd_ex_static_scratch if static_scratch else lib.fa_fwd_ex
    return _check(fn(ctypes.byref(p)), check)
