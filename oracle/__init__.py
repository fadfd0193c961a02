"""Softmax oracle: TEST INFRASTRUCTURE, not part of the product.

ctypes front end of the plain-C long-double oracle (softmax_oracle.c) and of
the double-precision scalar model of Algorithms 1-3 (twopass_model.c).  Only
tests, the smoke check and the bench's cpu_baseline leg may import this.
Nothing here imports or is imported by the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_SOURCES = ("softmax_oracle.c", "twopass_model.c")

_i64 = ctypes.c_int64
_vp = ctypes.c_void_p


class Cmp(ctypes.Structure):
    """Mirror of oracle_cmp_t."""

    _fields_ = [
        ("max_rel_err", ctypes.c_double),
        ("worst_index", _i64),
        ("worst_expected", ctypes.c_double),
        ("worst_got", ctypes.c_double),
        ("max_sub_abs_err", ctypes.c_double),
        ("max_row_sum_dev", ctypes.c_double),
        ("n_rel_viol", _i64),
        ("n_sub_viol", _i64),
        ("n_nonfinite", _i64),
        ("n_negative", _i64),
        ("n_normal", _i64),
        ("n_total", _i64),
        ("max_bound_ratio", ctypes.c_double),
    ]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}

    def ok(self):
        return (self.n_rel_viol == 0 and self.n_sub_viol == 0 and self.n_nonfinite == 0
                and self.n_negative == 0)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math) into oracle/liboracle.so."""
    srcs = [os.path.join(_HERE, s) for s in _SOURCES]
    if not force and os.path.exists(_LIB_PATH):
        newest = max(os.path.getmtime(s) for s in srcs)
        if os.path.getmtime(_LIB_PATH) >= newest:
            return _LIB_PATH
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", _LIB_PATH, *srcs, "-lm", "-lpthread"]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_PATH)
        L.oracle_threads_available.restype = ctypes.c_int
        for name in ("oracle_stats_f32", "oracle_stats_bf16", "oracle_stats_f16"):
            getattr(L, name).argtypes = [_vp, _i64, _i64, _vp, _vp, ctypes.c_int]
            getattr(L, name).restype = None
        for name in ("oracle_softmax_f32", "oracle_softmax_bf16", "oracle_softmax_f16"):
            getattr(L, name).argtypes = [_vp, _i64, _i64, _vp, ctypes.c_int]
            getattr(L, name).restype = None
        for name in ("oracle_compare_f32", "oracle_compare_bf16", "oracle_compare_f16"):
            getattr(L, name).argtypes = [_vp, _vp, _i64, _i64, ctypes.c_double,
                                         ctypes.POINTER(Cmp), ctypes.c_int]
            getattr(L, name).restype = None
        L.oracle_compare_sloped_f32.argtypes = [_vp, _vp, _i64, _i64, ctypes.c_double, ctypes.c_double,
                                                ctypes.POINTER(Cmp), ctypes.c_int]
        L.oracle_compare_sloped_f32.restype = None
        L.oracle_pair_rel_err_f32.argtypes = [_vp, _vp, _vp, _i64, _vp]
        L.oracle_pair_rel_err_f32.restype = ctypes.c_double
        L.oracle_logsumexp_f32.argtypes = [_vp, _i64, ctypes.c_int]
        L.oracle_logsumexp_f32.restype = ctypes.c_longdouble
        L.model_extexp.argtypes = [ctypes.c_double, ctypes.POINTER(ctypes.c_double),
                                   ctypes.POINTER(ctypes.c_double)]
        L.model_pair_add.argtypes = [ctypes.c_double] * 4 + [ctypes.POINTER(ctypes.c_double)] * 2
        L.model_twopass_pass1.argtypes = [_vp, _i64, ctypes.POINTER(ctypes.c_double),
                                          ctypes.POINTER(ctypes.c_double)]
        for name in ("model_twopass", "model_threepass_recompute", "model_threepass_reload"):
            getattr(L, name).argtypes = [_vp, _vp, _i64]
            getattr(L, name).restype = None
        _lib = L
    return _lib


def threads_available() -> int:
    return int(lib().oracle_threads_available())


def _as2d(x, dtype):
    a = np.ascontiguousarray(x, dtype=dtype)
    if a.ndim == 1:
        a = a.reshape(1, -1)
    assert a.ndim == 2
    return a


def _ptr(a):
    return a.ctypes.data_as(_vp)


def _kind(bf16, f16):
    assert not (bf16 and f16)
    return "bf16" if bf16 else "f16" if f16 else "f32"


def stats(x, bf16: bool = False, threads: int = 0, f16: bool = False):
    """Per-row (mu, S) as numpy longdouble arrays.  x: fp32 values, or bf16 / fp16 bit patterns."""
    a = _as2d(x, np.uint16 if (bf16 or f16) else np.float32)
    rows, n = a.shape
    mu = np.zeros(rows, dtype=np.longdouble)
    S = np.zeros(rows, dtype=np.longdouble)
    fn = getattr(lib(), "oracle_stats_" + _kind(bf16, f16))
    fn(_ptr(a), rows, n, _ptr(mu), _ptr(S), threads)
    return mu, S


def softmax(x, bf16: bool = False, threads: int = 0, f16: bool = False):
    """Row-wise softmax as a numpy longdouble array of x's shape."""
    shape = np.shape(x)
    a = _as2d(x, np.uint16 if (bf16 or f16) else np.float32)
    rows, n = a.shape
    p = np.zeros((rows, n), dtype=np.longdouble)
    fn = getattr(lib(), "oracle_softmax_" + _kind(bf16, f16))
    fn(_ptr(a), rows, n, _ptr(p), threads)
    return p.reshape(shape)


def compare(x, y, tol: float, bf16: bool = False, threads: int = 0, f16: bool = False,
            slope: float = 0.0) -> Cmp:
    """Stream y against the oracle's p for x (same shape); see oracle_cmp_t.  With slope > 0
    (fp32 only) element i is held to tol + slope * |x_i - mu| instead of tol."""
    dt = np.uint16 if (bf16 or f16) else np.float32
    a = _as2d(x, dt)
    b = _as2d(y, dt)
    assert a.shape == b.shape
    rows, n = a.shape
    out = Cmp()
    if slope:
        assert not (bf16 or f16)
        lib().oracle_compare_sloped_f32(_ptr(a), _ptr(b), rows, n, float(tol), float(slope),
                                        ctypes.byref(out), threads)
        return out
    fn = getattr(lib(), "oracle_compare_" + _kind(bf16, f16))
    fn(_ptr(a), _ptr(b), rows, n, float(tol), ctypes.byref(out), threads)
    return out


# The fp32 subtraction x - mu of the Three-Pass algorithms is off by up to half an ulp of the
# difference: 2^-24 |x - mu| relative in the result (see the comparator in softmax_oracle.c).
THREE_PASS_SLOPE = 2.0 ** -24


def pair_rel_err(x, m, n):
    """|m * 2^n / e^x - 1| per element (computed overflow-free) and its maximum."""
    xa = np.ascontiguousarray(x, dtype=np.float32).ravel()
    ma = np.ascontiguousarray(m, dtype=np.float32).ravel()
    na = np.ascontiguousarray(n, dtype=np.float32).ravel()
    rel = np.zeros(xa.size, dtype=np.float64)
    worst = lib().oracle_pair_rel_err_f32(_ptr(xa), _ptr(ma), _ptr(na), xa.size, _ptr(rel))
    return rel, float(worst)


def logsumexp(x, threads: int = 0):
    """mu + ln S of one fp32 vector, as numpy longdouble."""
    a = np.ascontiguousarray(x, dtype=np.float32).ravel()
    return np.longdouble(lib().oracle_logsumexp_f32(_ptr(a), a.size, threads))


# ---- double-precision scalar model of Algorithms 1-3 ------------------------

def model_extexp(x: float):
    m = ctypes.c_double()
    n = ctypes.c_double()
    lib().model_extexp(float(x), ctypes.byref(m), ctypes.byref(n))
    return m.value, n.value


def model_pair_add(a, b):
    m = ctypes.c_double()
    n = ctypes.c_double()
    lib().model_pair_add(float(a[0]), float(a[1]), float(b[0]), float(b[1]),
                         ctypes.byref(m), ctypes.byref(n))
    return m.value, n.value


def model_pass1(x):
    a = np.ascontiguousarray(x, dtype=np.float64).ravel()
    m = ctypes.c_double()
    n = ctypes.c_double()
    lib().model_twopass_pass1(_ptr(a), a.size, ctypes.byref(m), ctypes.byref(n))
    return m.value, n.value


def _model_run(name, x):
    a = np.ascontiguousarray(x, dtype=np.float64).ravel()
    y = np.zeros_like(a)
    getattr(lib(), name)(_ptr(a), _ptr(y), a.size)
    return y


def model_twopass(x):
    return _model_run("model_twopass", x)


def model_threepass_recompute(x):
    return _model_run("model_threepass_recompute", x)


def model_threepass_reload(x):
    return _model_run("model_threepass_reload", x)
