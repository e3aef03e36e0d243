"""ctypes wrapper around the C oracle (oracle/hif8_oracle.c).

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the CPU-baseline leg
of the benchmark may import this module; the product package never does.  All
arrays are numpy arrays in host memory; bfloat16 travels as raw uint16 patterns.
"""
import ctypes
import os

import numpy as np

from . import build as _build

RM_TA = 0
RM_HR = 1
RM_TE = 2
RM_SSR = 3
RM_SR = 4
SRC_F32, SRC_BF16, SRC_F16 = 0, 1, 2
FLAG_SAT = 0x10
FLAG_NAN2ZERO = 0x20

_lib = ctypes.CDLL(_build.build())

_u8p = ctypes.POINTER(ctypes.c_uint8)
_u16p = ctypes.POINTER(ctypes.c_uint16)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_intp = ctypes.POINTER(ctypes.c_int)

_lib.hif8o_decode_value.restype = ctypes.c_double
_lib.hif8o_decode_value.argtypes = [ctypes.c_uint8]
_lib.hif8o_decode_fields.restype = ctypes.c_double
_lib.hif8o_decode_fields.argtypes = [ctypes.c_uint8, _intp, _intp, _intp, _intp, _intp]
_lib.hif8o_value_table.restype = ctypes.c_int
_lib.hif8o_value_table.argtypes = [_f64p, _u8p]
_lib.hif8o_encode_one.restype = ctypes.c_uint8
_lib.hif8o_encode_one.argtypes = [ctypes.c_float, ctypes.c_uint32, ctypes.c_int]
_lib.hif8o_encode_one_t.restype = ctypes.c_uint8
_lib.hif8o_encode_one_t.argtypes = [ctypes.c_float, ctypes.c_uint32, ctypes.c_int, ctypes.c_uint32]
_lib.hif8o_sr_threshold.restype = ctypes.c_uint32
_lib.hif8o_sr_threshold.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
_lib.hif8o_set_sr_seed.argtypes = [ctypes.c_uint64]
_lib.hif8o_set_sr_index_base.argtypes = [ctypes.c_uint64]
_lib.hif8o_widen_f16.argtypes = [_u16p, _f32p, ctypes.c_size_t]
_lib.hif8o_narrow_f16.argtypes = [_f32p, _u16p, ctypes.c_size_t]
_lib.hif8o_encode_f16.argtypes = [_u16p, _u8p, ctypes.c_size_t, ctypes.c_float, ctypes.c_uint32]
_lib.hif8o_decode_f16.argtypes = [_u8p, _u16p, ctypes.c_size_t, ctypes.c_float]
_lib.hif8o_fake_quant_f16.argtypes = [_u16p, _u16p, _u8p, ctypes.c_size_t, ctypes.c_float, ctypes.c_uint32]
_lib.hif8o_amax_f16.restype = ctypes.c_float
_lib.hif8o_amax_f16.argtypes = [_u16p, ctypes.c_size_t]
_lib.hif8o_set_literal_sr_zero.argtypes = [ctypes.c_int]
_lib.hif8o_threads_used.restype = ctypes.c_int
_lib.hif8o_encode_f32.argtypes = [_f32p, _u8p, ctypes.c_size_t, ctypes.c_float, ctypes.c_uint32]
_lib.hif8o_encode_bf16.argtypes = [_u16p, _u8p, ctypes.c_size_t, ctypes.c_float, ctypes.c_uint32]
_lib.hif8o_decode_f32.argtypes = [_u8p, _f32p, ctypes.c_size_t, ctypes.c_float]
_lib.hif8o_decode_bf16.argtypes = [_u8p, _u16p, ctypes.c_size_t, ctypes.c_float]
_lib.hif8o_fake_quant_f32.argtypes = [_f32p, _f32p, _u8p, ctypes.c_size_t, ctypes.c_float, ctypes.c_uint32]
_lib.hif8o_fake_quant_bf16.argtypes = [_u16p, _u16p, _u8p, ctypes.c_size_t, ctypes.c_float, ctypes.c_uint32]
_lib.hif8o_narrow_bf16.argtypes = [_f32p, _u16p, ctypes.c_size_t]
_lib.hif8o_amax_f32.restype = ctypes.c_float
_lib.hif8o_amax_f32.argtypes = [_f32p, ctypes.c_size_t]
_lib.hif8o_amax_bf16.restype = ctypes.c_float
_lib.hif8o_amax_bf16.argtypes = [_u16p, ctypes.c_size_t]
_vp = ctypes.c_void_p
_lib.hif8o_scale_sweep.argtypes = [_vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_uint32, _f64p]
_lib.hif8o_amax_axis.argtypes = [_vp, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, _f32p]
_lib.hif8o_encode_axis.argtypes = [_vp, _u8p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, _f32p, ctypes.c_uint32]
_lib.hif8o_decode_axis.argtypes = [_u8p, _vp, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, _f32p]
_lib.hif8o_scale_from_amax.restype = ctypes.c_float
_lib.hif8o_scale_from_amax.argtypes = [ctypes.c_float, ctypes.c_float, ctypes.c_int]


def _arr(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, a.dtype))
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def decode_value(code: int) -> float:
    """Real value of one code (Eq. 1 / Eq. 2 / specials) as a Python float."""
    return _lib.hif8o_decode_value(code & 0xFF)


def decode_fields(code: int) -> dict:
    """Parse of one code: kind (zero/nan/inf/dml/nml), D, E, mantissa width, M."""
    k, d, e, w, m = (ctypes.c_int() for _ in range(5))
    v = _lib.hif8o_decode_fields(code & 0xFF, ctypes.byref(k), ctypes.byref(d),
                                 ctypes.byref(e), ctypes.byref(w), ctypes.byref(m))
    kinds = ["zero", "nan", "inf", "dml", "nml"]
    return {"value": v, "kind": kinds[k.value], "D": d.value, "E": e.value,
            "mant_width": w.value, "M": m.value}


def value_table():
    """(values, codes): the finite non-negative magnitudes, ascending."""
    vals = np.zeros(128, np.float64)
    codes = np.zeros(128, np.uint8)
    n = _lib.hif8o_value_table(_ptr(vals, ctypes.c_double), _ptr(codes, ctypes.c_uint8))
    return vals[:n].copy(), codes[:n].copy()


def encode_one(y: float, mode: int = RM_TA, src_bf16=False, t32: int = 0) -> int:
    """src_bf16: False / SRC_F32, True / SRC_BF16, or SRC_F16; t32: threshold for RM_SR."""
    return _lib.hif8o_encode_one_t(np.float32(y), mode, int(src_bf16), t32)


def sr_threshold(seed: int, index: int) -> int:
    return _lib.hif8o_sr_threshold(seed, index)


def set_sr_seed(seed: int) -> None:
    """Seed of the standard-SR threshold generator used by the array functions."""
    _lib.hif8o_set_sr_seed(seed)


def set_sr_index_base(base: int) -> None:
    """Index that element 0 of the arrays passed to the array functions has (default 0)."""
    _lib.hif8o_set_sr_index_base(base)


def widen_f16(src):
    src = _arr(src, np.uint16)
    dst = np.empty(src.shape, np.float32)
    _lib.hif8o_widen_f16(_ptr(src, ctypes.c_uint16), _ptr(dst, ctypes.c_float), src.size)
    return dst


def narrow_f16(src):
    src = _arr(src, np.float32)
    dst = np.empty(src.shape, np.uint16)
    _lib.hif8o_narrow_f16(_ptr(src, ctypes.c_float), _ptr(dst, ctypes.c_uint16), src.size)
    return dst


def encode_f16(src, scale=1.0, mode=RM_TA):
    src = _arr(src, np.uint16)
    dst = np.empty(src.shape, np.uint8)
    _lib.hif8o_encode_f16(_ptr(src, ctypes.c_uint16), _ptr(dst, ctypes.c_uint8), src.size,
                          np.float32(scale), mode)
    return dst


def decode_f16(codes, scale=1.0):
    codes = _arr(codes, np.uint8)
    dst = np.empty(codes.shape, np.uint16)
    _lib.hif8o_decode_f16(_ptr(codes, ctypes.c_uint8), _ptr(dst, ctypes.c_uint16), codes.size,
                          np.float32(scale))
    return dst


def fake_quant_f16(src, scale=1.0, mode=RM_TA):
    src = _arr(src, np.uint16)
    dst = np.empty(src.shape, np.uint16)
    codes = np.empty(src.shape, np.uint8)
    _lib.hif8o_fake_quant_f16(_ptr(src, ctypes.c_uint16), _ptr(dst, ctypes.c_uint16),
                              _ptr(codes, ctypes.c_uint8), src.size, np.float32(scale), mode)
    return dst, codes


def amax_f16(src) -> np.float32:
    src = _arr(src, np.uint16)
    return np.float32(_lib.hif8o_amax_f16(_ptr(src, ctypes.c_uint16), src.size))


def set_literal_sr_zero(on: bool) -> None:
    _lib.hif8o_set_literal_sr_zero(int(on))


def threads_used() -> int:
    return _lib.hif8o_threads_used()


def encode_f32(src, scale=1.0, mode=RM_TA):
    src = _arr(src, np.float32)
    dst = np.empty(src.shape, np.uint8)
    _lib.hif8o_encode_f32(_ptr(src, ctypes.c_float), _ptr(dst, ctypes.c_uint8), src.size,
                          np.float32(scale), mode)
    return dst


def encode_bf16(src, scale=1.0, mode=RM_TA):
    src = _arr(src, np.uint16)
    dst = np.empty(src.shape, np.uint8)
    _lib.hif8o_encode_bf16(_ptr(src, ctypes.c_uint16), _ptr(dst, ctypes.c_uint8), src.size,
                           np.float32(scale), mode)
    return dst


def decode_f32(codes, scale=1.0):
    codes = _arr(codes, np.uint8)
    dst = np.empty(codes.shape, np.float32)
    _lib.hif8o_decode_f32(_ptr(codes, ctypes.c_uint8), _ptr(dst, ctypes.c_float), codes.size,
                          np.float32(scale))
    return dst


def decode_bf16(codes, scale=1.0):
    codes = _arr(codes, np.uint8)
    dst = np.empty(codes.shape, np.uint16)
    _lib.hif8o_decode_bf16(_ptr(codes, ctypes.c_uint8), _ptr(dst, ctypes.c_uint16), codes.size,
                           np.float32(scale))
    return dst


def fake_quant_f32(src, scale=1.0, mode=RM_TA):
    src = _arr(src, np.float32)
    dst = np.empty(src.shape, np.float32)
    codes = np.empty(src.shape, np.uint8)
    _lib.hif8o_fake_quant_f32(_ptr(src, ctypes.c_float), _ptr(dst, ctypes.c_float),
                              _ptr(codes, ctypes.c_uint8), src.size, np.float32(scale), mode)
    return dst, codes


def fake_quant_bf16(src, scale=1.0, mode=RM_TA):
    src = _arr(src, np.uint16)
    dst = np.empty(src.shape, np.uint16)
    codes = np.empty(src.shape, np.uint8)
    _lib.hif8o_fake_quant_bf16(_ptr(src, ctypes.c_uint16), _ptr(dst, ctypes.c_uint16),
                               _ptr(codes, ctypes.c_uint8), src.size, np.float32(scale), mode)
    return dst, codes


def narrow_bf16(src):
    """binary32 -> bfloat16 patterns, round to nearest even (the narrowing used by decode)."""
    src = _arr(src, np.float32)
    dst = np.empty(src.shape, np.uint16)
    _lib.hif8o_narrow_bf16(_ptr(src, ctypes.c_float), _ptr(dst, ctypes.c_uint16), src.size)
    return dst


def amax_f32(src) -> np.float32:
    src = _arr(src, np.float32)
    return np.float32(_lib.hif8o_amax_f32(_ptr(src, ctypes.c_float), src.size))


def amax_bf16(src) -> np.float32:
    src = _arr(src, np.uint16)
    return np.float32(_lib.hif8o_amax_bf16(_ptr(src, ctypes.c_uint16), src.size))


def scale_from_amax(amax, target=32768.0, pow2=False) -> np.float32:
    return np.float32(_lib.hif8o_scale_from_amax(np.float32(amax), np.float32(target), int(pow2)))


def _kind_dtype(kind):
    return np.float32 if kind == SRC_F32 else np.uint16


def scale_sweep(src, kind=SRC_F32, e_lo=-4, count=10, mode=RM_TA):
    """Sum of squared cast errors of one tensor at the scales 2^e_lo .. 2^(e_lo+count-1)
    (fp64 array of `count` sums; divide by the element count for the MSE)."""
    src = _arr(src, _kind_dtype(kind))
    err = np.zeros(count, np.float64)
    _lib.hif8o_scale_sweep(src.ctypes.data_as(ctypes.c_void_p), src.size, kind, e_lo, count, mode,
                           _ptr(err, ctypes.c_double))
    return err


def amax_axis(src, kind=SRC_F32, axis=0):
    src = _arr(src, _kind_dtype(kind))
    rows, cols = src.shape
    out = np.zeros(rows if axis == 0 else cols, np.float32)
    _lib.hif8o_amax_axis(src.ctypes.data_as(ctypes.c_void_p), rows, cols, kind, axis, _ptr(out, ctypes.c_float))
    return out


def encode_axis(src, scale, kind=SRC_F32, axis=0, mode=RM_TA):
    src = _arr(src, _kind_dtype(kind))
    scale = _arr(scale, np.float32)
    rows, cols = src.shape
    assert scale.size == (rows if axis == 0 else cols)
    dst = np.empty(src.shape, np.uint8)
    _lib.hif8o_encode_axis(src.ctypes.data_as(ctypes.c_void_p), _ptr(dst, ctypes.c_uint8), rows, cols, kind, axis,
                           _ptr(scale, ctypes.c_float), mode)
    return dst


def decode_axis(codes, scale, kind=SRC_F32, axis=0):
    codes = _arr(codes, np.uint8)
    scale = _arr(scale, np.float32)
    rows, cols = codes.shape
    assert scale.size == (rows if axis == 0 else cols)
    dst = np.empty(codes.shape, _kind_dtype(kind))
    _lib.hif8o_decode_axis(_ptr(codes, ctypes.c_uint8), dst.ctypes.data_as(ctypes.c_void_p), rows, cols, kind, axis,
                           _ptr(scale, ctypes.c_float))
    return dst
