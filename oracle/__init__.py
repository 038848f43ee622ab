"""CPU oracle for D := alpha*op(A)*op(B) + beta*op(C)  --  TEST INFRASTRUCTURE ONLY.

Thin ctypes front end of ``contraction_oracle.cpp`` (the loop nest of the paper's
Sec. "Algorithm Structure", written out plainly).  Only tests, the smoke check and the
bench's ``cpu_baseline`` leg may import this package; the GPU library never does and
the two share no code.

Tensors are described by plain Python sequences: ``extents``, ``strides`` (in elements,
from the element whose indices are all zero) and integer ``labels``; data are 1-D numpy
buffers plus an element offset of the all-zero element inside the buffer.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "contraction_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

DT_F32, DT_F64, DT_C64, DT_C128, DT_F16, DT_BF16 = 0, 1, 2, 3, 4, 5
MODE_TRUTH, MODE_TIMED, MODE_LITERAL = 0, 1, 2
OP_IDENTITY, OP_CONJ = 0, 1

V_OK, V_EXTENT_MISMATCH, V_CD_MISMATCH, V_D_ALIASING, V_ISOLATED, V_BAD_ARG = range(6)
V_NAMES = ["ok", "extent_mismatch", "cd_mismatch", "d_aliasing", "isolated_index", "bad_arg"]

_NP_DTYPE = {DT_F32: np.float32, DT_F64: np.float64, DT_C64: np.complex64, DT_C128: np.complex128, DT_F16: np.float16,
             DT_BF16: np.uint16}      # numpy has no bfloat16: buffers of its bit patterns
_DT_OF_NP = {np.dtype(v): k for k, v in _NP_DTYPE.items()}


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (g++ -O2 -fopenmp). Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["g++", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c++17", _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_validate.restype = ctypes.c_int
        _lib.oracle_contract.restype = ctypes.c_int
        _lib.oracle_max_threads.restype = ctypes.c_int
        _lib.oracle_half_from_double.restype = ctypes.c_uint16
        _lib.oracle_half_from_double.argtypes = [ctypes.c_double]
        _lib.oracle_half_to_double.restype = ctypes.c_double
        _lib.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        _lib.oracle_bfloat16_from_double.restype = ctypes.c_uint16
        _lib.oracle_bfloat16_from_double.argtypes = [ctypes.c_double]
        _lib.oracle_bfloat16_to_double.restype = ctypes.c_double
        _lib.oracle_bfloat16_to_double.argtypes = [ctypes.c_uint16]
    return _lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def half_from_double(x: float) -> int:
    """Bits of the 16-bit value nearest to x (ties to even): the oracle's own conversion."""
    return int(_load().oracle_half_from_double(float(x)))


def half_to_double(bits: int) -> float:
    return float(_load().oracle_half_to_double(int(bits)))


def bfloat16_from_double(x: float) -> int:
    return int(_load().oracle_bfloat16_from_double(float(x)))


def bfloat16_to_double(bits: int) -> float:
    return float(_load().oracle_bfloat16_to_double(int(bits)))


def _i64(seq):
    arr = (ctypes.c_int64 * max(1, len(seq)))()
    for i, v in enumerate(seq):
        arr[i] = int(v)
    return arr


def _desc_args(extents, strides, labels):
    n = len(extents)
    assert len(strides) == n and len(labels) == n
    return [ctypes.c_int(n), _i64(extents), _i64(strides), _i64(labels)]


def validate(A, B, C, D) -> int:
    """Each argument is (extents, strides, labels). Returns a V_* class."""
    args = []
    for t in (A, B, C, D):
        args += _desc_args(*t)
    return int(_load().oracle_validate(*args))


def contract(A, B, C, D, ops: Sequence[int], alpha, beta,
             bufA: np.ndarray, bufB: np.ndarray, bufC, bufD: np.ndarray,
             base=(0, 0, 0, 0), mode: int = MODE_TRUTH, want_S: bool = False):
    """Run the loop nest.  A, B, C, D are (extents, strides, labels); ops = (opA, opB, opC).

    bufX are 1-D numpy arrays of one dtype (float32, float64, complex64, complex128, float16, or
    uint16 holding bfloat16 bit patterns); bufD is
    written in place (bufC may be bufD, or None when beta == 0).  base[i] is the element
    offset inside the buffer of the element with all indices zero.  Returns (status, S)
    where S is None or a float64 array shaped like bufD holding sum|a||b| per D element.
    """
    lib = _load()
    dt = _DT_OF_NP[bufD.dtype]
    for b in (bufA, bufB):
        assert b.dtype == bufD.dtype and b.flags.c_contiguous and b.ndim == 1
    assert bufD.flags.c_contiguous and bufD.flags.writeable and bufD.ndim == 1
    item = bufD.dtype.itemsize

    def ptr(buf, off):
        return ctypes.c_void_p(buf.ctypes.data + int(off) * item) if buf is not None else ctypes.c_void_p(0)

    S = np.zeros(bufD.shape[0], dtype=np.float64) if want_S else None
    al = (ctypes.c_double * 2)(complex(alpha).real, complex(alpha).imag)
    be = (ctypes.c_double * 2)(complex(beta).real, complex(beta).imag)
    args = [ctypes.c_int(dt), ctypes.c_int(mode)]
    args += _desc_args(*A) + [ctypes.c_int(ops[0])]
    args += _desc_args(*B) + [ctypes.c_int(ops[1])]
    args += _desc_args(*C) + [ctypes.c_int(ops[2])]
    args += _desc_args(*D)
    args += [al, be, ptr(bufA, base[0]), ptr(bufB, base[1]), ptr(bufC, base[2]), ptr(bufD, base[3])]
    args += [ctypes.c_void_p(S.ctypes.data + int(base[3]) * 8) if want_S else ctypes.c_void_p(0)]
    st = int(lib.oracle_contract(*args))
    return st, S
