"""ctypes binding of libtcx.so: the same entry points as include/tcx.h, argument marshalling only.

Functions keep the C names.  They return the created handle / value and raise
:class:`TcxError` (carrying the integer code and the library's own explanation) when the
library returns a non-zero code.  Nothing here computes anything and there is no fallback:
if the shared library is missing the import raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtcx.so")

# PyTorch-ROCm ships its own HIP runtime.  A process that holds device memory through torch must
# let torch load that runtime first: if libtcx.so pulled in the system's libamdhip64 before it,
# torch would afterwards find no GPU.  Processes that do not use torch are unaffected.
try:
    import torch  # noqa: F401
except ImportError:
    pass

if not os.path.exists(LIB_PATH):
    raise ImportError("libtcx.so is not built: run `python paper_2601_07827_amd/build.py` "
                      "(hipcc --offload-arch=gfx950); there is no CPU fallback")
_lib = ctypes.CDLL(LIB_PATH)

# ---- constants of include/tcx.h ------------------------------------------------------------
TCX_F32, TCX_F64, TCX_C64, TCX_C128, TCX_F16, TCX_BF16 = 0, 1, 2, 3, 4, 5
TCX_OP_IDENTITY, TCX_OP_CONJ = 0, 1
TCX_PREC_DEFAULT, TCX_PREC_F64 = 0, 1
TCX_PATH_GENERIC, TCX_PATH_GETT_MFMA, TCX_PATH_BANDWIDTH = 0, 1, 2
(TCX_SUCCESS, TCX_ERR_NULL_ARG, TCX_ERR_INVALID_HANDLE, TCX_ERR_BAD_DTYPE, TCX_ERR_BAD_NMODE, TCX_ERR_BAD_EXTENT,
 TCX_ERR_EXTENT_MISMATCH, TCX_ERR_CD_MISMATCH, TCX_ERR_D_ALIASING, TCX_ERR_ISOLATED_INDEX, TCX_ERR_DTYPE_MIX,
 TCX_ERR_UNSUPPORTED_OP, TCX_ERR_UNSUPPORTED_PRECISION, TCX_ERR_ALLOC, TCX_ERR_LAUNCH, TCX_ERR_NO_DEVICE,
 TCX_ERR_TOO_LARGE, TCX_ERR_BAD_KEY, TCX_ERR_BUFFER_TOO_SMALL, TCX_ERR_PLAN_REFUSED,
 TCX_ERR_SCRATCH_TOO_SMALL) = range(21)
(TCX_KEY_PATH, TCX_KEY_SIZE_H, TCX_KEY_SIZE_M, TCX_KEY_SIZE_N, TCX_KEY_SIZE_K, TCX_KEY_NMODES_H, TCX_KEY_NMODES_M,
 TCX_KEY_NMODES_N, TCX_KEY_NMODES_K, TCX_KEY_TILE_M, TCX_KEY_TILE_N, TCX_KEY_TILE_K, TCX_KEY_GRID, TCX_KEY_BLOCK,
 TCX_KEY_A_K_FASTEST, TCX_KEY_B_K_FASTEST, TCX_KEY_D_N_FASTEST, TCX_KEY_VARIANT, TCX_KEY_HIP_ERROR, TCX_KEY_MODES_M,
 TCX_KEY_MODES_N, TCX_KEY_MODES_K, TCX_KEY_MODES_H, TCX_KEY_FORCE_PATH, TCX_KEY_SPLIT_K, TCX_KEY_LAUNCHES,
 TCX_KEY_GATHER_WIDTH, TCX_KEY_TABLE_ENTRIES, TCX_KEY_WORKSPACE_BYTES, TCX_KEY_DEVICE, TCX_KEY_NUM_CU,
 TCX_KEY_STREAM, TCX_KEY_PRECISION, TCX_KEY_PACED_LOADS) = range(1, 35)
TCX_MAX_MODES = 32
TCX_SCRATCH_BYTES = 32 * 1024 * 1024
TCX_PROBE_MFMA_F64, TCX_PROBE_MFMA_F32, TCX_PROBE_STORE, TCX_PROBE_COPY = 0, 1, 2, 3
TCX_KEY_USER = 65536

EXPORTS = [
    "tcx_create_handle", "tcx_destroy_handle", "tcx_handle_has_device", "tcx_create_executor", "tcx_destroy_executor",
    "tcx_create_tensor_info", "tcx_destroy_tensor_info", "tcx_tensor_info_get", "tcx_create_product",
    "tcx_destroy_product", "tcx_product_get", "tcx_product_set", "tcx_execute_product", "tcx_execute_product_noalloc",
    "tcx_status_get",
    "tcx_destroy_status", "tcx_check_success", "tcx_explain_error",
    "tcx_create_attr", "tcx_destroy_attr", "tcx_attr_set", "tcx_attr_get", "tcx_attr_clear", "tcx_probe_launch",
    "tcx_create_binary", "tcx_execute_binary", "tcx_create_unary", "tcx_execute_unary",
]

_h = ctypes.c_ssize_t            # intptr_t
_hp = ctypes.POINTER(_h)
_i64p = ctypes.POINTER(ctypes.c_int64)
_vp = ctypes.c_void_p
_szp = ctypes.POINTER(ctypes.c_size_t)

_lib.tcx_create_handle.argtypes = [_hp]
_lib.tcx_destroy_handle.argtypes = [_hp]
_lib.tcx_handle_has_device.argtypes = [_h, ctypes.POINTER(ctypes.c_int32)]
_lib.tcx_create_executor.argtypes = [_h, _vp, _hp]
_lib.tcx_destroy_executor.argtypes = [_hp]
_lib.tcx_create_tensor_info.argtypes = [_h, ctypes.c_int, ctypes.c_int32, _i64p, _i64p, _hp]
_lib.tcx_destroy_tensor_info.argtypes = [_hp]
_lib.tcx_tensor_info_get.argtypes = [_h, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int32), _i64p, _i64p]
_lib.tcx_create_product.argtypes = [_h] + [ctypes.c_int, _h, _i64p] * 4 + [ctypes.c_int, _hp]
_lib.tcx_destroy_product.argtypes = [_hp]
_lib.tcx_product_get.argtypes = [_h, ctypes.c_int32, _vp, _szp]
_lib.tcx_product_set.argtypes = [_h, ctypes.c_int32, _vp, ctypes.c_size_t]
_lib.tcx_execute_product.argtypes = [_h, _h, _hp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.tcx_execute_product_noalloc.argtypes = [_h, _h, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.tcx_create_binary.argtypes = [_h] + [ctypes.c_int, _h, _i64p] * 3 + [ctypes.c_int, _hp]
_lib.tcx_execute_binary.argtypes = [_h, _h, _hp, _vp, _vp, _vp, _vp, _vp]
_lib.tcx_create_unary.argtypes = [_h] + [ctypes.c_int, _h, _i64p] * 2 + [ctypes.c_int, _hp]
_lib.tcx_execute_unary.argtypes = [_h, _h, _hp, _vp, _vp, _vp]
_lib.tcx_status_get.argtypes = [_h, ctypes.c_int32, _vp, _szp]
_lib.tcx_destroy_status.argtypes = [_hp]
_lib.tcx_create_attr.argtypes = [_h, _hp]
_lib.tcx_destroy_attr.argtypes = [_hp]
_lib.tcx_attr_set.argtypes = [_h, ctypes.c_int32, _vp, ctypes.c_size_t]
_lib.tcx_attr_get.argtypes = [_h, ctypes.c_int32, _vp, _szp]
_lib.tcx_attr_clear.argtypes = [_h, ctypes.c_int32]
_lib.tcx_probe_launch.argtypes = [_h, ctypes.c_int32, _vp, ctypes.c_size_t, ctypes.c_int64, ctypes.POINTER(ctypes.c_double)]
_lib.tcx_check_success.argtypes = [ctypes.c_int32]
_lib.tcx_explain_error.argtypes = [ctypes.c_int32, ctypes.c_size_t, ctypes.c_char_p]
_lib.tcx_explain_error.restype = ctypes.c_size_t
for _name in EXPORTS:
    if _name not in ("tcx_explain_error",):
        getattr(_lib, _name).restype = ctypes.c_int32


class TcxError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = int(code)
        super().__init__("%s: error %d: %s" % (where, code, tcx_explain_error(code)))


def _check(code: int, where: str):
    if not _lib.tcx_check_success(code):
        raise TcxError(code, where)


def _arr(seq: Optional[Sequence[int]]):
    if seq is None:
        return None
    return (ctypes.c_int64 * max(1, len(seq)))(*[int(v) for v in seq])


def tcx_check_success(code: int) -> bool:
    return bool(_lib.tcx_check_success(int(code)))


def tcx_explain_error(code: int) -> str:
    need = _lib.tcx_explain_error(int(code), 0, None)
    buf = ctypes.create_string_buffer(need + 1)
    _lib.tcx_explain_error(int(code), need + 1, buf)
    return buf.value.decode()


def tcx_create_handle() -> int:
    h = _h(0)
    _check(_lib.tcx_create_handle(ctypes.byref(h)), "tcx_create_handle")
    return h.value


def tcx_destroy_handle(handle: int) -> int:
    """Returns the handle value after destruction (0), as the C call leaves it."""
    h = _h(handle)
    _check(_lib.tcx_destroy_handle(ctypes.byref(h)), "tcx_destroy_handle")
    return h.value


def tcx_handle_has_device(handle: int) -> bool:
    out = ctypes.c_int32(0)
    _check(_lib.tcx_handle_has_device(handle, ctypes.byref(out)), "tcx_handle_has_device")
    return bool(out.value)


def tcx_create_executor(handle: int, hip_stream: int = 0) -> int:
    e = _h(0)
    _check(_lib.tcx_create_executor(handle, _vp(hip_stream), ctypes.byref(e)), "tcx_create_executor")
    return e.value


def tcx_destroy_executor(executor: int) -> int:
    e = _h(executor)
    _check(_lib.tcx_destroy_executor(ctypes.byref(e)), "tcx_destroy_executor")
    return e.value


def tcx_create_tensor_info(handle: int, dtype: int, extents: Sequence[int], strides: Sequence[int]) -> int:
    t = _h(0)
    assert len(extents) == len(strides)
    _check(_lib.tcx_create_tensor_info(handle, dtype, len(extents), _arr(extents), _arr(strides), ctypes.byref(t)),
           "tcx_create_tensor_info")
    return t.value


def tcx_destroy_tensor_info(info: int) -> int:
    t = _h(info)
    _check(_lib.tcx_destroy_tensor_info(ctypes.byref(t)), "tcx_destroy_tensor_info")
    return t.value


def tcx_tensor_info_get(info: int):
    dt, n = ctypes.c_int(0), ctypes.c_int32(0)
    _check(_lib.tcx_tensor_info_get(info, ctypes.byref(dt), ctypes.byref(n), None, None), "tcx_tensor_info_get")
    ext, st = (ctypes.c_int64 * max(1, n.value))(), (ctypes.c_int64 * max(1, n.value))()
    _check(_lib.tcx_tensor_info_get(info, None, None, ext, st), "tcx_tensor_info_get")
    return dt.value, list(ext)[:n.value], list(st)[:n.value]


def tcx_create_product(handle: int, opA: int, A: int, labelsA, opB: int, B: int, labelsB, opC: int, C: int, labelsC,
                       opD: int, D: int, labelsD, precision: int = TCX_PREC_DEFAULT) -> int:
    p = _h(0)
    _check(_lib.tcx_create_product(handle, opA, A, _arr(labelsA), opB, B, _arr(labelsB), opC, C, _arr(labelsC),
                                   opD, D, _arr(labelsD), precision, ctypes.byref(p)), "tcx_create_product")
    return p.value


def tcx_destroy_product(product: int) -> int:
    p = _h(product)
    _check(_lib.tcx_destroy_product(ctypes.byref(p)), "tcx_destroy_product")
    return p.value


def _get(fn, obj: int, key: int, where: str):
    if key in (TCX_KEY_MODES_M, TCX_KEY_MODES_N, TCX_KEY_MODES_K, TCX_KEY_MODES_H):
        buf = (ctypes.c_int64 * (4 * 64))()
        n = ctypes.c_size_t(ctypes.sizeof(buf))
        _check(fn(obj, key, buf, ctypes.byref(n)), where)
        flat = list(buf)[: n.value // 8]
        return [tuple(flat[i:i + 4]) for i in range(0, len(flat), 4)]
    if key == TCX_KEY_TABLE_ENTRIES:
        buf = (ctypes.c_int64 * 3)()
        n = ctypes.c_size_t(ctypes.sizeof(buf))
        _check(fn(obj, key, buf, ctypes.byref(n)), where)
        return list(buf)
    v = ctypes.c_int64(0)
    n = ctypes.c_size_t(8)
    _check(fn(obj, key, ctypes.byref(v), ctypes.byref(n)), where)
    return v.value


def tcx_product_get(product: int, key: int):
    return _get(_lib.tcx_product_get, product, key, "tcx_product_get")


def tcx_product_set(product: int, key: int, value: int) -> None:
    v = ctypes.c_int64(int(value))
    _check(_lib.tcx_product_set(product, key, ctypes.byref(v), 8), "tcx_product_set")


def _scalar(dtype: int, x):
    if dtype in (TCX_F32, TCX_F16, TCX_BF16):          # 16-bit tensors take their scalars as floats
        return ctypes.c_float(float(x))
    if dtype == TCX_F64:
        return ctypes.c_double(float(x))
    z = complex(x)
    if dtype == TCX_C64:
        return (ctypes.c_float * 2)(z.real, z.imag)
    return (ctypes.c_double * 2)(z.real, z.imag)


def tcx_execute_product(product: int, executor: int, dtype: int, alpha, A: int, B: int, beta, C: int, D: int,
                        want_status: bool = False) -> Optional[int]:
    """A, B, C, D are device addresses (e.g. ``tensor.data_ptr()``) of the element with all
    indices zero; alpha/beta are Python numbers converted to D's dtype.  Returns a status
    handle if ``want_status`` else None."""
    al, be = _scalar(dtype, alpha), _scalar(dtype, beta)
    st = _h(0)
    code = _lib.tcx_execute_product(product, executor, ctypes.byref(st) if want_status else None,
                                    ctypes.cast(ctypes.pointer(al), _vp), _vp(A), _vp(B),
                                    ctypes.cast(ctypes.pointer(be), _vp), _vp(C), _vp(D))
    if code != TCX_SUCCESS and st.value:
        s = _h(st.value)
        _lib.tcx_destroy_status(ctypes.byref(s))
    _check(code, "tcx_execute_product")
    return st.value if want_status else None


def tcx_execute_product_noalloc(product: int, executor: int, dtype: int, alpha, A: int, B: int, beta, C: int, D: int) -> None:
    """tcx_execute_product for callers that cannot allocate: no status object, fixed scratch buffer."""
    al, be = _scalar(dtype, alpha), _scalar(dtype, beta)
    _check(_lib.tcx_execute_product_noalloc(product, executor, ctypes.cast(ctypes.pointer(al), _vp), _vp(A), _vp(B),
                                            ctypes.cast(ctypes.pointer(be), _vp), _vp(C), _vp(D)),
           "tcx_execute_product_noalloc")


def tcx_create_binary(handle: int, opA: int, A: int, labelsA, opB: int, B: int, labelsB, opC: int, C: int, labelsC,
                      precision: int = TCX_PREC_DEFAULT) -> int:
    """Plan of C := alpha opA(A) + beta opB(B)."""
    p = _h(0)
    _check(_lib.tcx_create_binary(handle, opA, A, _arr(labelsA), opB, B, _arr(labelsB), opC, C, _arr(labelsC), precision,
                                  ctypes.byref(p)), "tcx_create_binary")
    return p.value


def tcx_execute_binary(plan: int, executor: int, dtype: int, alpha, A: int, beta, B: int, C: int) -> None:
    al, be = _scalar(dtype, alpha), _scalar(dtype, beta)
    _check(_lib.tcx_execute_binary(plan, executor, None, ctypes.cast(ctypes.pointer(al), _vp), _vp(A),
                                   ctypes.cast(ctypes.pointer(be), _vp), _vp(B), _vp(C)), "tcx_execute_binary")


def tcx_create_unary(handle: int, opA: int, A: int, labelsA, opB: int, B: int, labelsB, precision: int = TCX_PREC_DEFAULT) -> int:
    """Plan of B := alpha opA(A)."""
    p = _h(0)
    _check(_lib.tcx_create_unary(handle, opA, A, _arr(labelsA), opB, B, _arr(labelsB), precision, ctypes.byref(p)),
           "tcx_create_unary")
    return p.value


def tcx_execute_unary(plan: int, executor: int, dtype: int, alpha, A: int, B: int) -> None:
    al = _scalar(dtype, alpha)
    _check(_lib.tcx_execute_unary(plan, executor, None, ctypes.cast(ctypes.pointer(al), _vp), _vp(A), _vp(B)), "tcx_execute_unary")


def tcx_status_get(status: int, key: int):
    return _get(_lib.tcx_status_get, status, key, "tcx_status_get")


def tcx_destroy_status(status: int) -> int:
    s = _h(status)
    _check(_lib.tcx_destroy_status(ctypes.byref(s)), "tcx_destroy_status")
    return s.value


def tcx_create_attr(handle: int) -> int:
    a = _h(0)
    _check(_lib.tcx_create_attr(handle, ctypes.byref(a)), "tcx_create_attr")
    return a.value


def tcx_destroy_attr(attr: int) -> int:
    a = _h(attr)
    _check(_lib.tcx_destroy_attr(ctypes.byref(a)), "tcx_destroy_attr")
    return a.value


def tcx_attr_set(obj: int, key: int, value) -> None:
    """value: bytes for a free-form key (>= TCX_KEY_USER), an int for one of the library's keys."""
    if key < TCX_KEY_USER:
        v = ctypes.c_int64(int(value))
        _check(_lib.tcx_attr_set(obj, key, ctypes.byref(v), 8), "tcx_attr_set")
        return
    data = bytes(value)
    buf = ctypes.create_string_buffer(data, len(data)) if data else None
    _check(_lib.tcx_attr_set(obj, key, buf, len(data)), "tcx_attr_set")


def tcx_attr_get(obj: int, key: int):
    """bytes for a free-form key; for the library's keys what tcx_product_get / tcx_status_get return."""
    if key < TCX_KEY_USER:
        return _get(_lib.tcx_attr_get, obj, key, "tcx_attr_get")
    n = ctypes.c_size_t(0)
    err = _lib.tcx_attr_get(obj, key, None, ctypes.byref(n))          # size query
    if err not in (TCX_SUCCESS, TCX_ERR_NULL_ARG):
        _check(err, "tcx_attr_get")
    if n.value == 0:
        return b""
    buf = ctypes.create_string_buffer(n.value)
    _check(_lib.tcx_attr_get(obj, key, buf, ctypes.byref(n)), "tcx_attr_get")
    return buf.raw[: n.value]


def tcx_attr_clear(obj: int, key: int) -> None:
    _check(_lib.tcx_attr_clear(obj, key), "tcx_attr_clear")


def tcx_probe_launch(executor: int, kind: int, buffer: int, nbytes: int, iters: int = 0) -> float:
    """One launch of a measurement kernel; returns the flop or bytes it performs."""
    work = ctypes.c_double(0.0)
    _check(_lib.tcx_probe_launch(executor, kind, _vp(buffer), nbytes, iters, ctypes.byref(work)), "tcx_probe_launch")
    return work.value


def raw():
    """The ctypes library object, for tests that exercise the C calling conventions directly."""
    return _lib
