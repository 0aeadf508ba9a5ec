"""CPU oracle (test infrastructure, never part of the product path).

Two independent pieces:

* ``tcr_oracle.c`` -- the plain definition of reduction / inclusive scan and their
  regular segmented forms (Section 3 of the paper), one sequential binary64 loop per
  segment, reached from Python through ``ctypes``.
* ``matrix_form`` -- the paper's own matrix-product algorithms (Sections 4 and 5)
  carried out step by step with explicit 16x16 matrices in binary64 numpy.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tcr_oracle.c")
_LIB = os.path.join(_HERE, "libtcr_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_LIB_OPENMP = os.path.join(_HERE, "libtcr_oracle_omp.so")


def build_openmp(force: bool = False) -> str:
    """The same source compiled with -fopenmp: the regular segmented reduce and scan share their segments among
    threads (every segment is still one sequential binary64 loop, so the results are bit-identical).  Only the
    multi-core timing of bench.py and the test that compares it with the sequential build use it."""
    if force or not os.path.exists(_LIB_OPENMP) or os.path.getmtime(_LIB_OPENMP) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB_OPENMP, _SRC, "-lm"])
    return _LIB_OPENMP


def _bind(path: str):
    lib = ctypes.CDLL(path)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    f64p = ctypes.POINTER(ctypes.c_double)
    u64p = ctypes.POINTER(ctypes.c_uint64)
    u64 = ctypes.c_uint64
    lib.oracle_half_to_double.argtypes = [ctypes.c_uint16]
    lib.oracle_half_to_double.restype = ctypes.c_double
    lib.oracle_double_to_half.argtypes = [ctypes.c_double]
    lib.oracle_double_to_half.restype = ctypes.c_uint16
    lib.oracle_segmented_scan_half_acc.argtypes = [u16p, u16p, u64, u64, ctypes.c_int]
    lib.oracle_segmented_scan_half_acc.restype = ctypes.c_int
    for name, args in (
        ("oracle_segmented_reduce", [u16p, f64p, u64, u64]),
        ("oracle_segmented_scan", [u16p, f64p, u64, u64]),
        ("oracle_segmented_scan_exclusive", [u16p, f64p, u64, u64]),
        ("oracle_segmented_moments", [u16p, f64p, f64p, u64, u64]),
        ("oracle_irregular_reduce", [u16p, u64p, f64p, u64]),
        ("oracle_irregular_scan", [u16p, u64p, f64p, u64]),
        ("oracle_irregular_scan_exclusive", [u16p, u64p, f64p, u64]),
        ("oracle_irregular_moments", [u16p, u64p, f64p, f64p, u64]),
        ("oracle_reduce", [u16p, f64p, u64]),
        ("oracle_scan", [u16p, f64p, u64]),
        ("oracle_segmented_scan_at", [u16p, u64, u64, u64p, u64, f64p]),
    ):
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = ctypes.c_int
    return lib


def _in_ptr(x: np.ndarray):
    if x.dtype != np.float16 or not x.flags.c_contiguous or x.ndim != 1:
        raise TypeError("input must be a contiguous 1-D float16 array")
    return x.view(np.uint16).ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _out_ptr(y: np.ndarray):
    return y.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


class Oracle:
    """The C oracle behind numpy arguments.  ``path`` names the shared object to load; the
    default is the one built from ``tcr_oracle.c`` (tests load deliberately broken builds
    through the same class to show that the pins reject them)."""

    def __init__(self, path: str | None = None):
        self._lib = _bind(path or build())

    def half_to_double(self, bits: int) -> float:
        return self._lib.oracle_half_to_double(int(bits) & 0xFFFF)

    def segmented_reduce(self, x: np.ndarray, seg_len: int) -> np.ndarray:
        n = x.shape[0]
        if seg_len <= 0 or n % seg_len:
            raise ValueError("seg_len must be positive and divide n")
        out = np.empty(n // seg_len, dtype=np.float64)
        if self._lib.oracle_segmented_reduce(_in_ptr(x), _out_ptr(out), n, seg_len):
            raise ValueError("oracle_segmented_reduce rejected its arguments")
        return out

    def segmented_scan(self, x: np.ndarray, seg_len: int) -> np.ndarray:
        n = x.shape[0]
        if seg_len <= 0 or n % seg_len:
            raise ValueError("seg_len must be positive and divide n")
        out = np.empty(n, dtype=np.float64)
        if self._lib.oracle_segmented_scan(_in_ptr(x), _out_ptr(out), n, seg_len):
            raise ValueError("oracle_segmented_scan rejected its arguments")
        return out

    def double_to_half(self, v: float) -> int:
        return int(self._lib.oracle_double_to_half(float(v)))

    def segmented_scan_half_acc(self, x: np.ndarray, seg_len: int, exclusive: bool = False) -> np.ndarray:
        """The scan with every addition rounded to binary16 (left to right); a float16 array."""
        n = x.shape[0]
        if seg_len <= 0 or n % seg_len:
            raise ValueError("seg_len must be positive and divide n")
        out = np.empty(n, dtype=np.uint16)
        if self._lib.oracle_segmented_scan_half_acc(_in_ptr(x), out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), n, seg_len,
                                                    1 if exclusive else 0):
            raise ValueError("oracle_segmented_scan_half_acc rejected its arguments")
        return out.view(np.float16)

    def segmented_scan_exclusive(self, x: np.ndarray, seg_len: int) -> np.ndarray:
        n = x.shape[0]
        if seg_len <= 0 or n % seg_len:
            raise ValueError("seg_len must be positive and divide n")
        out = np.empty(n, dtype=np.float64)
        if self._lib.oracle_segmented_scan_exclusive(_in_ptr(x), _out_ptr(out), n, seg_len):
            raise ValueError("oracle_segmented_scan_exclusive rejected its arguments")
        return out

    def segmented_moments(self, x: np.ndarray, seg_len: int):
        """(sum, sum of squares) of every segment."""
        n = x.shape[0]
        if seg_len <= 0 or n % seg_len:
            raise ValueError("seg_len must be positive and divide n")
        a = np.empty(n // seg_len, dtype=np.float64)
        q = np.empty(n // seg_len, dtype=np.float64)
        if self._lib.oracle_segmented_moments(_in_ptr(x), _out_ptr(a), _out_ptr(q), n, seg_len):
            raise ValueError("oracle_segmented_moments rejected its arguments")
        return a, q

    def irregular_moments(self, x: np.ndarray, offsets):
        """(sum, sum of squares) of every segment [offsets[s], offsets[s+1])."""
        off = np.ascontiguousarray(offsets, dtype=np.uint64)
        if off.ndim != 1 or off.size < 1 or (off.size > 1 and int(off.max()) > x.shape[0]):
            raise ValueError("offsets must hold nseg + 1 indices into x")
        a = np.zeros(off.size - 1, dtype=np.float64)
        q = np.zeros(off.size - 1, dtype=np.float64)
        if self._lib.oracle_irregular_moments(_in_ptr(x), off.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
                                              _out_ptr(a), _out_ptr(q), off.size - 1):
            raise ValueError("oracle_irregular_moments rejected its arguments")
        return a, q

    def irregular_reduce(self, x: np.ndarray, offsets) -> np.ndarray:
        off = np.ascontiguousarray(offsets, dtype=np.uint64)
        if off.ndim != 1 or off.size < 1 or (off.size > 1 and int(off.max()) > x.shape[0]):
            raise ValueError("offsets must hold nseg + 1 indices into x")
        out = np.zeros(off.size - 1, dtype=np.float64)
        if self._lib.oracle_irregular_reduce(_in_ptr(x), off.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
                                             _out_ptr(out), off.size - 1):
            raise ValueError("oracle_irregular_reduce rejected its arguments")
        return out

    def irregular_scan(self, x: np.ndarray, offsets) -> np.ndarray:
        off = np.ascontiguousarray(offsets, dtype=np.uint64)
        if off.ndim != 1 or off.size < 1 or (off.size > 1 and int(off.max()) > x.shape[0]):
            raise ValueError("offsets must hold nseg + 1 indices into x")
        out = np.zeros(x.shape[0], dtype=np.float64)
        if self._lib.oracle_irregular_scan(_in_ptr(x), off.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
                                           _out_ptr(out), off.size - 1):
            raise ValueError("oracle_irregular_scan rejected its arguments")
        return out

    def irregular_scan_exclusive(self, x: np.ndarray, offsets) -> np.ndarray:
        off = np.ascontiguousarray(offsets, dtype=np.uint64)
        if off.ndim != 1 or off.size < 1 or (off.size > 1 and int(off.max()) > x.shape[0]):
            raise ValueError("offsets must hold nseg + 1 indices into x")
        out = np.zeros(x.shape[0], dtype=np.float64)
        if self._lib.oracle_irregular_scan_exclusive(_in_ptr(x), off.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
                                                     _out_ptr(out), off.size - 1):
            raise ValueError("oracle_irregular_scan_exclusive rejected its arguments")
        return out

    def reduce(self, x: np.ndarray) -> float:
        out = np.zeros(1, dtype=np.float64)
        if self._lib.oracle_reduce(_in_ptr(x), _out_ptr(out), x.shape[0]):
            raise ValueError("oracle_reduce rejected its arguments")
        return float(out[0])

    def scan(self, x: np.ndarray) -> np.ndarray:
        out = np.empty(x.shape[0], dtype=np.float64)
        if self._lib.oracle_scan(_in_ptr(x), _out_ptr(out), x.shape[0]):
            raise ValueError("oracle_scan rejected its arguments")
        return out

    def segmented_scan_at(self, x: np.ndarray, seg_len: int, idx) -> np.ndarray:
        idx = np.ascontiguousarray(idx, dtype=np.uint64)
        out = np.empty(idx.shape[0], dtype=np.float64)
        rc = self._lib.oracle_segmented_scan_at(
            _in_ptr(x), x.shape[0], seg_len,
            idx.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)), idx.shape[0], _out_ptr(out))
        if rc:
            raise ValueError("oracle_segmented_scan_at rejected its arguments")
        return out


_default = None


_openmp = None


def openmp() -> "Oracle":
    """The OpenMP build behind the same class."""
    global _openmp
    if _openmp is None:
        _openmp = Oracle(build_openmp())
    return _openmp


def _get() -> Oracle:
    global _default
    if _default is None:
        _default = Oracle()
    return _default


def half_to_double(bits):
    return _get().half_to_double(bits)


def segmented_reduce(x, seg_len):
    return _get().segmented_reduce(x, seg_len)


def segmented_scan(x, seg_len):
    return _get().segmented_scan(x, seg_len)


def segmented_scan_exclusive(x, seg_len):
    return _get().segmented_scan_exclusive(x, seg_len)


def double_to_half(v):
    return _get().double_to_half(v)


def segmented_scan_half_acc(x, seg_len, exclusive=False):
    return _get().segmented_scan_half_acc(x, seg_len, exclusive)


def irregular_reduce(x, offsets):
    return _get().irregular_reduce(x, offsets)


def irregular_scan(x, offsets):
    return _get().irregular_scan(x, offsets)


def irregular_scan_exclusive(x, offsets):
    return _get().irregular_scan_exclusive(x, offsets)


def reduce(x):
    return _get().reduce(x)


def scan(x):
    return _get().scan(x)


def segmented_scan_at(x, seg_len, idx):
    return _get().segmented_scan_at(x, seg_len, idx)


def segmented_moments(x, seg_len):
    return _get().segmented_moments(x, seg_len)


def irregular_moments(x, offsets):
    return _get().irregular_moments(x, offsets)
