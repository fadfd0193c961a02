"""Thin ctypes binding of libsoftmax_tp.so: argument marshalling only.

Every function has the name and argument order of its C-ABI entry point
(include/softmax_tp.h).  Array arguments are torch tensors on the GPU (their
data_ptr is passed) or raw integer device addresses; `stream` is a
torch.cuda.Stream, a raw hipStream_t value, or None for torch's current stream.
A non-zero return code raises SoftmaxTpError.  There is no CPU fallback: if the
library is not built the import of the first function fails loudly.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsoftmax_tp.so")

_i64 = ctypes.c_int64
_vp = ctypes.c_void_p

ENTRY_POINTS = {
    "softmax2p_f32": [_vp, _vp, _i64, _i64, _vp],
    "softmax3p_recompute_f32": [_vp, _vp, _i64, _i64, _vp],
    "softmax3p_reload_f32": [_vp, _vp, _i64, _i64, _vp],
    "softmax2p_bf16io": [_vp, _vp, _i64, _i64, _vp],
    "softmax3p_recompute_bf16io": [_vp, _vp, _i64, _i64, _vp],
    "softmax3p_reload_bf16io": [_vp, _vp, _i64, _i64, _vp],
    "softmax2p_f16io": [_vp, _vp, _i64, _i64, _vp],
    "softmax3p_recompute_f16io": [_vp, _vp, _i64, _i64, _vp],
    "softmax3p_reload_f16io": [_vp, _vp, _i64, _i64, _vp],
    "softmax2p_onchip_f32": [_vp, _vp, _i64, _i64, _vp],
    "softmax2p_onchip_bf16io": [_vp, _vp, _i64, _i64, _vp],
    "softmax2p_onchip_f16io": [_vp, _vp, _i64, _i64, _vp],
    "softmax3p_onchip_f32": [_vp, _vp, _i64, _i64, _vp],
    "softmax3p_onchip_bf16io": [_vp, _vp, _i64, _i64, _vp],
    "softmax3p_onchip_f16io": [_vp, _vp, _i64, _i64, _vp],
    "softmax2p_f32_static": [_vp, _vp, _i64, _i64, _vp],
    "softmax_tp_extexp_f32": [_vp, _vp, _vp, _i64, _vp],
    "softmax_tp_extexp_hw_f32": [_vp, _vp, _vp, _i64, _vp],
    "softmax2p_f32_pass1": [_vp, _vp, _i64, _i64, _vp],
    "softmax2p_f32_pass2": [_vp, _vp, _vp, _i64, _i64, _vp],
    "softmax_tp_stream_read_f32": [_vp, _vp, _i64, _vp],
    "softmax_tp_stream_fill_f32": [_vp, ctypes.c_float, _i64, _vp],
    "softmax_tp_stream_copy_f32": [_vp, _vp, _i64, _vp],
    "softmax_tp_stream_scale_f32": [_vp, _vp, ctypes.c_float, _i64, _vp],
    "softmax_tp_plan": [_i64, _i64, ctypes.c_int32, ctypes.c_int32, _vp],
    "softmax_tp_tune": [ctypes.c_char_p, _i64],
    "softmax_tp_reserve": [_i64, _i64, ctypes.c_int32, _vp],
    "softmax_tp_release": [],
    "softmax_tp_strerror": [ctypes.c_int],
}

TP_ERR_NULL, TP_ERR_NEGATIVE, TP_ERR_TOO_LARGE, TP_ERR_ALIGN, TP_ERR_TUNING = -1, -2, -3, -4, -5
TP_ERR_SCRATCH = -6
TP_STATIC_SCRATCH_BYTES = 256 * 1024


class Shape(ctypes.Structure):
    """Mirror of softmax_tp_shape_t."""

    _fields_ = [("block", ctypes.c_int32), ("unroll", ctypes.c_int32),
                ("chunk_vecs", _i64), ("chunks", _i64)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class Plan(ctypes.Structure):
    """Mirror of softmax_tp_plan_t."""

    _fields_ = [
        ("path", ctypes.c_int32),
        ("vector_elems", ctypes.c_int32),
        ("launches", ctypes.c_int32),
        ("merge_kernel", ctypes.c_int32),
        ("nt_first_load", ctypes.c_int32),
        ("rows", Shape),
        ("rows_recompute", Shape),
        ("rows_reload", Shape),
        ("reduce", Shape),
        ("map", Shape),
        ("mapsum", Shape),
        ("workspace_bytes", _i64),
    ]

    def as_dict(self):
        d = {}
        for k, _ in self._fields_:
            v = getattr(self, k)
            d[k] = v.as_dict() if isinstance(v, Shape) else v
        if self.path == 1:
            for k in ("reduce", "map", "mapsum"):
                d.pop(k)
        else:
            for k in ("rows", "rows_recompute", "rows_reload"):
                d.pop(k)
        return d


TUNE_KEYS = ("path", "block_rows", "unroll_rows", "block_reduce", "unroll_reduce", "target_reduce",
             "block_map", "unroll_map", "tiles_map", "block_mapsum", "unroll_mapsum", "tiles_mapsum",
             "direction", "nt_first", "fold_max", "nt_store", "scalar_io")


class SoftmaxTpError(RuntimeError):
    def __init__(self, fn, code):
        self.code = code
        super().__init__(f"{fn} failed with code {code}: {strerror(code)}")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2001_04438_amd.buildlib` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        for name, argtypes in ENTRY_POINTS.items():
            fn = getattr(L, name)
            fn.argtypes = argtypes
            fn.restype = ctypes.c_char_p if name == "softmax_tp_strerror" else ctypes.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().softmax_tp_strerror(int(code)).decode()


def _addr(a):
    if a is None:
        return None
    if isinstance(a, int):
        return a
    return a.data_ptr()  # torch tensor


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(name, code):
    if code != 0:
        raise SoftmaxTpError(name, code)


def _softmax(name, x, y, rows, n, stream):
    _check(name, getattr(lib(), name)(_addr(x), _addr(y), rows, n, _stream(stream)))


def softmax2p_f32(x, y, rows, n, stream=None):
    _softmax("softmax2p_f32", x, y, rows, n, stream)


def softmax3p_recompute_f32(x, y, rows, n, stream=None):
    _softmax("softmax3p_recompute_f32", x, y, rows, n, stream)


def softmax3p_reload_f32(x, y, rows, n, stream=None):
    _softmax("softmax3p_reload_f32", x, y, rows, n, stream)


def softmax2p_bf16io(x, y, rows, n, stream=None):
    _softmax("softmax2p_bf16io", x, y, rows, n, stream)


def softmax3p_recompute_bf16io(x, y, rows, n, stream=None):
    _softmax("softmax3p_recompute_bf16io", x, y, rows, n, stream)


def softmax3p_reload_bf16io(x, y, rows, n, stream=None):
    _softmax("softmax3p_reload_bf16io", x, y, rows, n, stream)


def softmax2p_f16io(x, y, rows, n, stream=None):
    _softmax("softmax2p_f16io", x, y, rows, n, stream)


def softmax3p_recompute_f16io(x, y, rows, n, stream=None):
    _softmax("softmax3p_recompute_f16io", x, y, rows, n, stream)


def softmax3p_reload_f16io(x, y, rows, n, stream=None):
    _softmax("softmax3p_reload_f16io", x, y, rows, n, stream)


def softmax2p_onchip_f32(x, y, rows, n, stream=None):
    _softmax("softmax2p_onchip_f32", x, y, rows, n, stream)


def softmax2p_onchip_bf16io(x, y, rows, n, stream=None):
    _softmax("softmax2p_onchip_bf16io", x, y, rows, n, stream)


def softmax2p_onchip_f16io(x, y, rows, n, stream=None):
    _softmax("softmax2p_onchip_f16io", x, y, rows, n, stream)


def softmax3p_onchip_f32(x, y, rows, n, stream=None):
    _softmax("softmax3p_onchip_f32", x, y, rows, n, stream)


def softmax3p_onchip_bf16io(x, y, rows, n, stream=None):
    _softmax("softmax3p_onchip_bf16io", x, y, rows, n, stream)


def softmax3p_onchip_f16io(x, y, rows, n, stream=None):
    _softmax("softmax3p_onchip_f16io", x, y, rows, n, stream)


def softmax2p_f32_static(x, y, rows, n, stream=None):
    _softmax("softmax2p_f32_static", x, y, rows, n, stream)


def softmax_tp_extexp_f32(x, m, e, count, stream=None):
    _check("softmax_tp_extexp_f32",
           lib().softmax_tp_extexp_f32(_addr(x), _addr(m), _addr(e), count, _stream(stream)))


def softmax_tp_extexp_hw_f32(x, m, e, count, stream=None):
    _check("softmax_tp_extexp_hw_f32",
           lib().softmax_tp_extexp_hw_f32(_addr(x), _addr(m), _addr(e), count, _stream(stream)))


def softmax2p_f32_pass1(x, pairs, rows, n, stream=None):
    _check("softmax2p_f32_pass1",
           lib().softmax2p_f32_pass1(_addr(x), _addr(pairs), rows, n, _stream(stream)))


def softmax2p_f32_pass2(x, pairs, y, rows, n, stream=None):
    _check("softmax2p_f32_pass2",
           lib().softmax2p_f32_pass2(_addr(x), _addr(pairs), _addr(y), rows, n, _stream(stream)))


def softmax_tp_stream_read_f32(x, sink, count, stream=None):
    _check("softmax_tp_stream_read_f32",
           lib().softmax_tp_stream_read_f32(_addr(x), _addr(sink), count, _stream(stream)))


def softmax_tp_stream_fill_f32(y, value, count, stream=None):
    _check("softmax_tp_stream_fill_f32",
           lib().softmax_tp_stream_fill_f32(_addr(y), float(value), count, _stream(stream)))


def softmax_tp_stream_copy_f32(x, y, count, stream=None):
    _check("softmax_tp_stream_copy_f32",
           lib().softmax_tp_stream_copy_f32(_addr(x), _addr(y), count, _stream(stream)))


def softmax_tp_stream_scale_f32(x, y, a, count, stream=None):
    _check("softmax_tp_stream_scale_f32",
           lib().softmax_tp_stream_scale_f32(_addr(x), _addr(y), float(a), count, _stream(stream)))


def softmax_tp_plan(rows, n, elem_bytes=4, congruent16=True) -> Plan:
    p = Plan()
    _check("softmax_tp_plan",
           lib().softmax_tp_plan(rows, n, elem_bytes, 1 if congruent16 else 0, ctypes.byref(p)))
    return p


def softmax_tp_tune(key: str, value: int):
    _check("softmax_tp_tune", lib().softmax_tp_tune(key.encode(), int(value)))


def softmax_tp_tune_reset():
    """Restores every planner parameter to its default."""
    for key in TUNE_KEYS:
        softmax_tp_tune(key, 0)


def softmax_tp_reserve(rows, n, elem_bytes=4, stream=None):
    _check("softmax_tp_reserve", lib().softmax_tp_reserve(rows, n, elem_bytes, _stream(stream)))


def softmax_tp_release():
    _check("softmax_tp_release", lib().softmax_tp_release())
