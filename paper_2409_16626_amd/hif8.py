"""Thin ctypes binding over libhif8.so: same names as the C ABI in include/hif8.h.

Argument marshalling only -- every step of the conversion runs in the HIP kernels.
Data arguments are torch tensors living on the GPU (or raw integer device pointers);
bfloat16 / float16 tensors may be passed as such or as int16/uint16 views.  The HIP
stream defaults to torch's current stream.  There is no CPU fallback: if the library
is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

from . import build as _build

RM_TA = 0
RM_HR = 1
RM_TE = 2    # comparison modes (described by the paper, not adopted by the format)
RM_SSR = 3
RM_SR = 4
FLAG_SAT = 0x10
FLAG_NAN2ZERO = 0x20
MAX_FINITE = 32768.0

TUNE_BLOCK, TUNE_WG_PER_CU, TUNE_UNROLL, TUNE_TA_IMPL, TUNE_TILES_PER_WG, TUNE_AMAX_NT, TUNE_GROUP_MIB, TUNE_FAMILY, TUNE_STAGE_OVERLAP = 0, 1, 2, 3, 4, 5, 6, 7, 8
N_TUNE_KEYS = 9
(FAM_ENC32_TA, FAM_ENC32_HR, FAM_ENC16, FAM_FQ, FAM_DEC, FAM_AMAX, FAM_DIAG, FAM_CALIB, FAM_AMAX_PARTS, FAM_MULTI_STAGE) = range(10)

_STATUS = {0: "HIF8_OK", -1: "HIF8_ERR_NULL", -2: "HIF8_ERR_MODE", -3: "HIF8_ERR_SCALE",
           -4: "HIF8_ERR_HIP", -5: "HIF8_ERR_ARG"}


class Hif8Error(RuntimeError):
    def __init__(self, status, hip_error=0):
        self.status = status
        self.hip_error = hip_error
        super().__init__("%s (status %d, hipError %d)" % (_STATUS.get(status, "?"), status, hip_error))


def _load():
    path = _build.LIB
    if not os.path.exists(path):
        # nothing built yet: build once (hipcc cross-compiles without a GPU); never fall back
        _build.build(force=True)
    return ctypes.CDLL(path)


lib = _load()

_vp, _sz, _f, _u32, _i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float, ctypes.c_uint32, ctypes.c_int
_u64 = ctypes.c_uint64

_SIGS = {
    "hif8_version": ([], _i),
    "hif8_last_hip_error": ([], _i),
    "hif8_init": ([], _i),
    "hif8_set_sr_seed": ([_u64], _i),
    "hif8_get_sr_seed": ([], _u64),
    "hif8_sr_threshold": ([_u64, _u64], _u32),
    "hif8_amax_f16": ([_vp, _sz, _vp, _vp], _i),
    "hif8_encode_f16": ([_vp, _vp, _sz, _f, _u32, _vp], _i),
    "hif8_decode_f16": ([_vp, _vp, _sz, _f, _vp], _i),
    "hif8_fake_quant_f16": ([_vp, _vp, _vp, _sz, _f, _u32, _vp], _i),
    "hif8_encode_f16_ds": ([_vp, _vp, _sz, _vp, _vp, _u32, _vp], _i),
    "hif8_decode_f16_ds": ([_vp, _vp, _sz, _vp, _vp], _i),
    "hif8_fake_quant_f16_ds": ([_vp, _vp, _vp, _sz, _vp, _vp, _u32, _vp], _i),
    "hif8_multi_cast_f16": ([_vp, _vp, _sz, ctypes.c_uint64, _vp, _vp, _f, _i, _u32, _vp], _i),
    "hif8_encode_f16_sr": ([_vp, _vp, _sz, _f, _u32, _u64, _u64, _vp], _i),
    "hif8_fake_quant_f16_sr": ([_vp, _vp, _vp, _sz, _f, _u32, _u64, _u64, _vp], _i),
    "hif8_quantize_tensor_f16": ([_vp, _vp, _vp, _sz, _f, _i, _u32, _vp, _vp, _vp, _sz, _vp], _i),
    "hif8_amax_f32": ([_vp, _sz, _vp, _vp], _i),
    "hif8_amax_bf16": ([_vp, _sz, _vp, _vp], _i),
    "hif8_scale_from_amax": ([_vp, _vp, _f, _i, _vp], _i),
    "hif8_encode_f32": ([_vp, _vp, _sz, _f, _u32, _vp], _i),
    "hif8_encode_bf16": ([_vp, _vp, _sz, _f, _u32, _vp], _i),
    "hif8_decode_f32": ([_vp, _vp, _sz, _f, _vp], _i),
    "hif8_decode_bf16": ([_vp, _vp, _sz, _f, _vp], _i),
    "hif8_fake_quant_f32": ([_vp, _vp, _vp, _sz, _f, _u32, _vp], _i),
    "hif8_fake_quant_bf16": ([_vp, _vp, _vp, _sz, _f, _u32, _vp], _i),
    "hif8_encode_f32_ds": ([_vp, _vp, _sz, _vp, _vp, _u32, _vp], _i),
    "hif8_encode_bf16_ds": ([_vp, _vp, _sz, _vp, _vp, _u32, _vp], _i),
    "hif8_decode_f32_ds": ([_vp, _vp, _sz, _vp, _vp], _i),
    "hif8_decode_bf16_ds": ([_vp, _vp, _sz, _vp, _vp], _i),
    "hif8_fake_quant_f32_ds": ([_vp, _vp, _vp, _sz, _vp, _vp, _u32, _vp], _i),
    "hif8_fake_quant_bf16_ds": ([_vp, _vp, _vp, _sz, _vp, _vp, _u32, _vp], _i),
    "hif8_multi_plan": ([_vp, _sz, _i, _vp], _i),
    "hif8_quantize_workspace_bytes": ([], _sz),
    "hif8_quantize_tensor_static": ([_vp, _vp, _vp, _sz, _i, _f, _i, _u32, _vp, _vp, _vp], _i),
    "hif8_multi_cast_bf16": ([_vp, _vp, _sz, ctypes.c_uint64, _vp, _vp, _f, _i, _u32, _vp], _i),
    "hif8_encode_bf16_sr": ([_vp, _vp, _sz, _f, _u32, _u64, _u64, _vp], _i),
    "hif8_fake_quant_bf16_sr": ([_vp, _vp, _vp, _sz, _f, _u32, _u64, _u64, _vp], _i),
    "hif8_quantize_tensor_bf16": ([_vp, _vp, _vp, _sz, _f, _i, _u32, _vp, _vp, _vp, _sz, _vp], _i),
    "hif8_multi_encode_bf16_ds": ([_vp, _sz, ctypes.c_uint64, _vp, _vp, _u32, _vp], _i),
    "hif8_multi_encode_f32_ds": ([_vp, _sz, ctypes.c_uint64, _vp, _vp, _u32, _vp], _i),
    "hif8_multi_encode_f16_ds": ([_vp, _sz, ctypes.c_uint64, _vp, _vp, _u32, _vp], _i),
    "hif8_multi_cast_f32": ([_vp, _vp, _sz, ctypes.c_uint64, _vp, _vp, _f, _i, _u32, _vp], _i),
    "hif8_encode_f32_sr": ([_vp, _vp, _sz, _f, _u32, _u64, _u64, _vp], _i),
    "hif8_fake_quant_f32_sr": ([_vp, _vp, _vp, _sz, _f, _u32, _u64, _u64, _vp], _i),
    "hif8_quantize_tensor_f32": ([_vp, _vp, _vp, _sz, _f, _i, _u32, _vp, _vp, _vp, _sz, _vp], _i),
    "hif8_scale_from_amax_n": ([_vp, _vp, _sz, _f, _i, _vp], _i),
    "hif8_scale_sweep_f32": ([_vp, _sz, _i, _i, _u32, _vp, _vp], _i),
    "hif8_scale_sweep_bf16": ([_vp, _sz, _i, _i, _u32, _vp, _vp], _i),
    "hif8_scale_sweep_f16": ([_vp, _sz, _i, _i, _u32, _vp, _vp], _i),
    "hif8_amax_axis_f32": ([_vp, _sz, _sz, _i, _vp, _vp], _i),
    "hif8_amax_axis_bf16": ([_vp, _sz, _sz, _i, _vp, _vp], _i),
    "hif8_amax_axis_f16": ([_vp, _sz, _sz, _i, _vp, _vp], _i),
    "hif8_encode_axis_f32": ([_vp, _vp, _sz, _sz, _i, _vp, _u32, _vp], _i),
    "hif8_encode_axis_bf16": ([_vp, _vp, _sz, _sz, _i, _vp, _u32, _vp], _i),
    "hif8_encode_axis_f16": ([_vp, _vp, _sz, _sz, _i, _vp, _u32, _vp], _i),
    "hif8_decode_axis_f32": ([_vp, _vp, _sz, _sz, _i, _vp, _vp], _i),
    "hif8_decode_axis_bf16": ([_vp, _vp, _sz, _sz, _i, _vp, _vp], _i),
    "hif8_decode_axis_f16": ([_vp, _vp, _sz, _sz, _i, _vp, _vp], _i),
    "hif8_quantize_rows_f32": ([_vp, _vp, _sz, _sz, _f, _i, _u32, _vp, _vp, _vp], _i),
    "hif8_quantize_rows_bf16": ([_vp, _vp, _sz, _sz, _f, _i, _u32, _vp, _vp, _vp], _i),
    "hif8_quantize_rows_f16": ([_vp, _vp, _sz, _sz, _f, _i, _u32, _vp, _vp, _vp], _i),
    "hif8_pts_init": ([_vp, _vp, _vp, _sz, _u32, _f, _vp], _i),
    "hif8_pts_collects": ([_vp], _i),
    "hif8_pts_end_iteration": ([_vp, _vp], _i),
    "hif8_als_init": ([_vp], None),
    "hif8_als_window": ([_vp], _i),
    "hif8_als_update": ([_vp, _i], _i),
    "hif8_gemm_f32": ([_vp, _vp, _vp, _sz, _sz, _sz, _f, _f, _vp], _i),
    "hif8_gemm_bf16": ([_vp, _vp, _vp, _sz, _sz, _sz, _f, _f, _vp], _i),
    "hif8_gemm_f16": ([_vp, _vp, _vp, _sz, _sz, _sz, _f, _f, _vp], _i),
    "hif8_gemm_sqerr": ([_vp, _vp, _vp, _sz, _sz, _sz, _f, _f, _vp, _vp], _i),
    "hif8_gemm_workspace_bytes": ([_sz, _sz, _sz], _sz),
    "hif8_gemm_ws_f32": ([_vp, _vp, _vp, _sz, _sz, _sz, _f, _f, _vp, _sz, _vp], _i),
    "hif8_gemm_ws_bf16": ([_vp, _vp, _vp, _sz, _sz, _sz, _f, _f, _vp, _sz, _vp], _i),
    "hif8_gemm_ws_f16": ([_vp, _vp, _vp, _sz, _sz, _sz, _f, _f, _vp, _sz, _vp], _i),
    "hif8_gemm_ws_sqerr": ([_vp, _vp, _vp, _sz, _sz, _sz, _f, _f, _vp, _vp, _sz, _vp], _i),
    "hif8_gemm_set_variant": ([_i], _i),
    "hif8_calibrate_workspace_bytes": ([_sz, _sz, _sz, _i, _i], _sz),
    "hif8_expanded_ld": ([_sz], _sz),
    "hif8_expand_bf16": ([_vp, _sz, _sz, _vp, _sz, _vp], _i),
    "hif8_expand_bf16_t": ([_vp, _sz, _sz, _vp, _sz, _vp], _i),
    "hif8_gemm_expanded_f32": ([_vp, _vp, _vp, _sz, _sz, _sz, _sz, _f, _f, _vp], _i),
    "hif8_gemm_expanded_bf16": ([_vp, _vp, _vp, _sz, _sz, _sz, _sz, _f, _f, _vp], _i),
    "hif8_gemm_expanded_f16": ([_vp, _vp, _vp, _sz, _sz, _sz, _sz, _f, _f, _vp], _i),
    "hif8_gemm_expanded_sqerr": ([_vp, _vp, _vp, _sz, _sz, _sz, _sz, _f, _f, _vp, _vp], _i),
    "hif8_calibrate_layer_f32": ([_vp, _vp, _vp, _sz, _sz, _sz, _i, _i, _i, _i, _u32, _vp, _sz, _vp, _vp, _vp], _i),
    "hif8_calibrate_layer_bf16": ([_vp, _vp, _vp, _sz, _sz, _sz, _i, _i, _i, _i, _u32, _vp, _sz, _vp, _vp, _vp], _i),
    "hif8_calibrate_layer_f16": ([_vp, _vp, _vp, _sz, _sz, _sz, _i, _i, _i, _i, _u32, _vp, _sz, _vp, _vp, _vp], _i),
    "hif8_set_tuning": ([_i, _i], _i),
    "hif8_get_tuning": ([_i], _i),
    "hif8_diag_stream": ([_vp, _vp, _sz, _i, _vp], _i),
}
for _name, (_args, _res) in _SIGS.items():
    _fn = getattr(lib, _name)
    _fn.argtypes = _args
    _fn.restype = _res

EXPORTED_SYMBOLS = tuple(_SIGS)


def _ptr(t):
    """Device pointer of a tensor (or pass an int / None through)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("libhif8 takes device pointers; got a tensor on %s" % t.device)
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status):
    if status != 0:
        raise Hif8Error(status, lib.hif8_last_hip_error())


def hif8_version():
    return lib.hif8_version()


def hif8_last_hip_error():
    return lib.hif8_last_hip_error()


def hif8_init():
    _check(lib.hif8_init())


def hif8_set_sr_seed(seed):
    _check(lib.hif8_set_sr_seed(seed))


def hif8_get_sr_seed():
    return lib.hif8_get_sr_seed()


def hif8_sr_threshold(seed, index):
    return lib.hif8_sr_threshold(seed, index)


def hif8_amax_f16(src, n, d_amax, stream=None):
    _check(lib.hif8_amax_f16(_ptr(src), n, _ptr(d_amax), _stream(stream)))


def hif8_encode_f16(src, dst, n, scale=1.0, rounding_mode=RM_TA, stream=None):
    _check(lib.hif8_encode_f16(_ptr(src), _ptr(dst), n, scale, rounding_mode, _stream(stream)))


def hif8_decode_f16(src, dst, n, scale=1.0, stream=None):
    _check(lib.hif8_decode_f16(_ptr(src), _ptr(dst), n, scale, _stream(stream)))


def hif8_fake_quant_f16(src, dst, codes_or_none, n, scale=1.0, rounding_mode=RM_TA, stream=None):
    _check(lib.hif8_fake_quant_f16(_ptr(src), _ptr(dst), _ptr(codes_or_none), n, scale, rounding_mode,
                                   _stream(stream)))


def hif8_encode_f16_ds(src, dst, n, d_scale2, rounding_mode=RM_TA, stream=None, d_amax_accum=None):
    _check(lib.hif8_encode_f16_ds(_ptr(src), _ptr(dst), n, _ptr(d_scale2), _ptr(d_amax_accum), rounding_mode,
                                  _stream(stream)))


def hif8_decode_f16_ds(src, dst, n, d_scale2, stream=None):
    _check(lib.hif8_decode_f16_ds(_ptr(src), _ptr(dst), n, _ptr(d_scale2), _stream(stream)))


def hif8_fake_quant_f16_ds(src, dst, codes_or_none, n, d_scale2, rounding_mode=RM_TA, stream=None,
                           d_amax_accum=None):
    _check(lib.hif8_fake_quant_f16_ds(_ptr(src), _ptr(dst), _ptr(codes_or_none), n, _ptr(d_scale2),
                                      _ptr(d_amax_accum), rounding_mode, _stream(stream)))


def hif8_amax_f32(src, n, d_amax, stream=None):
    _check(lib.hif8_amax_f32(_ptr(src), n, _ptr(d_amax), _stream(stream)))


def hif8_amax_bf16(src, n, d_amax, stream=None):
    _check(lib.hif8_amax_bf16(_ptr(src), n, _ptr(d_amax), _stream(stream)))


def hif8_scale_from_amax(d_amax, d_scale2, target=MAX_FINITE, pow2=0, stream=None):
    _check(lib.hif8_scale_from_amax(_ptr(d_amax), _ptr(d_scale2), target, int(pow2), _stream(stream)))


def hif8_encode_f32(src, dst, n, scale=1.0, rounding_mode=RM_TA, stream=None):
    _check(lib.hif8_encode_f32(_ptr(src), _ptr(dst), n, scale, rounding_mode, _stream(stream)))


def hif8_encode_bf16(src, dst, n, scale=1.0, rounding_mode=RM_TA, stream=None):
    _check(lib.hif8_encode_bf16(_ptr(src), _ptr(dst), n, scale, rounding_mode, _stream(stream)))


def hif8_decode_f32(src, dst, n, scale=1.0, stream=None):
    _check(lib.hif8_decode_f32(_ptr(src), _ptr(dst), n, scale, _stream(stream)))


def hif8_decode_bf16(src, dst, n, scale=1.0, stream=None):
    _check(lib.hif8_decode_bf16(_ptr(src), _ptr(dst), n, scale, _stream(stream)))


def hif8_fake_quant_f32(src, dst, codes_or_none, n, scale=1.0, rounding_mode=RM_TA, stream=None):
    _check(lib.hif8_fake_quant_f32(_ptr(src), _ptr(dst), _ptr(codes_or_none), n, scale, rounding_mode,
                                   _stream(stream)))


def hif8_fake_quant_bf16(src, dst, codes_or_none, n, scale=1.0, rounding_mode=RM_TA, stream=None):
    _check(lib.hif8_fake_quant_bf16(_ptr(src), _ptr(dst), _ptr(codes_or_none), n, scale, rounding_mode,
                                    _stream(stream)))


def hif8_encode_f32_ds(src, dst, n, d_scale2, rounding_mode=RM_TA, stream=None, d_amax_accum=None):
    _check(lib.hif8_encode_f32_ds(_ptr(src), _ptr(dst), n, _ptr(d_scale2), _ptr(d_amax_accum), rounding_mode,
                                  _stream(stream)))


def hif8_encode_bf16_ds(src, dst, n, d_scale2, rounding_mode=RM_TA, stream=None, d_amax_accum=None):
    _check(lib.hif8_encode_bf16_ds(_ptr(src), _ptr(dst), n, _ptr(d_scale2), _ptr(d_amax_accum), rounding_mode,
                                   _stream(stream)))


def hif8_decode_f32_ds(src, dst, n, d_scale2, stream=None):
    _check(lib.hif8_decode_f32_ds(_ptr(src), _ptr(dst), n, _ptr(d_scale2), _stream(stream)))


def hif8_decode_bf16_ds(src, dst, n, d_scale2, stream=None):
    _check(lib.hif8_decode_bf16_ds(_ptr(src), _ptr(dst), n, _ptr(d_scale2), _stream(stream)))


def hif8_fake_quant_f32_ds(src, dst, codes_or_none, n, d_scale2, rounding_mode=RM_TA, stream=None,
                           d_amax_accum=None):
    _check(lib.hif8_fake_quant_f32_ds(_ptr(src), _ptr(dst), _ptr(codes_or_none), n, _ptr(d_scale2),
                                      _ptr(d_amax_accum), rounding_mode, _stream(stream)))


def hif8_fake_quant_bf16_ds(src, dst, codes_or_none, n, d_scale2, rounding_mode=RM_TA, stream=None,
                            d_amax_accum=None):
    _check(lib.hif8_fake_quant_bf16_ds(_ptr(src), _ptr(dst), _ptr(codes_or_none), n, _ptr(d_scale2),
                                       _ptr(d_amax_accum), rounding_mode, _stream(stream)))


class CastItem(ctypes.Structure):
    """Mirror of hif8_cast_item."""
    _fields_ = [("src", ctypes.c_void_p), ("dst", ctypes.c_void_p), ("n", ctypes.c_uint64),
                ("first_tile", ctypes.c_uint64)]


class MultiPlan:
    """A planned list of tensors: the hif8_cast_item array on the host (ctypes) and its device copy."""

    def __init__(self, host_items, d_items, count, total_tiles):
        self.host_items, self.d_items, self.count, self.total_tiles = host_items, d_items, count, total_tiles

    def __iter__(self):   # (d_items, count, total_tiles), the arguments the launches take
        return iter((self.d_items, self.count, self.total_tiles))


def hif8_multi_plan(items, src_is_16bit=True):
    """items: list of (src_ptr_or_tensor, dst_ptr_or_tensor, n).  Returns a MultiPlan (it unpacks into
    (device uint8 tensor holding the planned hif8_cast_item array, count, total_tiles))."""
    count = len(items)
    arr = (CastItem * max(count, 1))()
    for i, (src, dst, n) in enumerate(items):
        arr[i].src = _ptr(src)
        arr[i].dst = _ptr(dst)
        arr[i].n = n
    total = ctypes.c_uint64(0)
    _check(lib.hif8_multi_plan(ctypes.cast(arr, ctypes.c_void_p), count, int(src_is_16bit),
                               ctypes.cast(ctypes.byref(total), ctypes.c_void_p)))
    raw = bytes(arr)[:count * ctypes.sizeof(CastItem)]
    d_items = torch.frombuffer(bytearray(raw), dtype=torch.uint8).cuda() if count else torch.empty(0, dtype=torch.uint8, device="cuda")
    return MultiPlan(arr, d_items, count, total.value)


def _def_multi_cast(sfx):
    fn = getattr(lib, "hif8_multi_cast_" + sfx)

    def multi_cast(d_items, count, total_tiles, d_amax, d_scale2, target=MAX_FINITE, pow2=0, rounding_mode=RM_TA,
                   stream=None, host_items=None):
        """host_items: the planned array on the host (MultiPlan.host_items) -> group-wise schedule."""
        hp = ctypes.cast(host_items, ctypes.c_void_p) if host_items is not None else None
        _check(fn(hp, _ptr(d_items), count, total_tiles, _ptr(d_amax), _ptr(d_scale2), target, int(pow2), rounding_mode,
                  _stream(stream)))

    return multi_cast


hif8_multi_cast_bf16 = _def_multi_cast("bf16")
hif8_multi_cast_f32 = _def_multi_cast("f32")
hif8_multi_cast_f16 = _def_multi_cast("f16")


def hif8_quantize_workspace_bytes():
    return lib.hif8_quantize_workspace_bytes()


KIND_F32, KIND_BF16, KIND_F16 = 0, 1, 2
STATIC_MAX_ELEMENTS = 1 << 32


def hif8_quantize_tensor_static(src, dst_or_none, codes_or_none, n, src_kind, d_amax, d_scale2, target=MAX_FINITE, pow2=0,
                                rounding_mode=RM_TA, stream=None):
    _check(lib.hif8_quantize_tensor_static(_ptr(src), _ptr(dst_or_none), _ptr(codes_or_none), n, src_kind, target, int(pow2),
                                           rounding_mode, _ptr(d_amax), _ptr(d_scale2), _stream(stream)))


def _def_tensor_calls(sfx):
    enc_sr, fq_sr = getattr(lib, "hif8_encode_%s_sr" % sfx), getattr(lib, "hif8_fake_quant_%s_sr" % sfx)
    qt = getattr(lib, "hif8_quantize_tensor_" + sfx)

    def encode_sr(src, dst, n, scale, rounding_mode, seed, index_base=0, stream=None):
        _check(enc_sr(_ptr(src), _ptr(dst), n, scale, rounding_mode, seed, index_base, _stream(stream)))

    def fake_quant_sr(src, dst, codes_or_none, n, scale, rounding_mode, seed, index_base=0, stream=None):
        _check(fq_sr(_ptr(src), _ptr(dst), _ptr(codes_or_none), n, scale, rounding_mode, seed, index_base, _stream(stream)))

    def quantize_tensor(src, dst_or_none, codes_or_none, n, d_amax, d_scale2, workspace, target=MAX_FINITE, pow2=0,
                        rounding_mode=RM_TA, stream=None, workspace_bytes=None):
        if workspace_bytes is None:
            workspace_bytes = 0 if workspace is None or isinstance(workspace, int) else workspace.numel() * workspace.element_size()
        _check(qt(_ptr(src), _ptr(dst_or_none), _ptr(codes_or_none), n, target, int(pow2), rounding_mode, _ptr(d_amax),
                  _ptr(d_scale2), _ptr(workspace), workspace_bytes, _stream(stream)))

    return encode_sr, fake_quant_sr, quantize_tensor


hif8_encode_f32_sr, hif8_fake_quant_f32_sr, hif8_quantize_tensor_f32 = _def_tensor_calls("f32")
hif8_encode_bf16_sr, hif8_fake_quant_bf16_sr, hif8_quantize_tensor_bf16 = _def_tensor_calls("bf16")
hif8_encode_f16_sr, hif8_fake_quant_f16_sr, hif8_quantize_tensor_f16 = _def_tensor_calls("f16")


def _def_multi_encode_ds(sfx):
    fn = getattr(lib, "hif8_multi_encode_%s_ds" % sfx)

    def multi_encode_ds(d_items, count, total_tiles, d_scale2, rounding_mode=RM_TA, stream=None, d_amax_accum=None):
        _check(fn(_ptr(d_items), count, total_tiles, _ptr(d_scale2), _ptr(d_amax_accum), rounding_mode, _stream(stream)))

    return multi_encode_ds


hif8_multi_encode_bf16_ds = _def_multi_encode_ds("bf16")
hif8_multi_encode_f32_ds = _def_multi_encode_ds("f32")
hif8_multi_encode_f16_ds = _def_multi_encode_ds("f16")


def hif8_scale_from_amax_n(d_amax, d_scale2, count, target=MAX_FINITE, pow2=0, stream=None):
    _check(lib.hif8_scale_from_amax_n(_ptr(d_amax), _ptr(d_scale2), count, target, int(pow2), _stream(stream)))


def _def_calib(sfx):
    sweep, amax = getattr(lib, "hif8_scale_sweep_" + sfx), getattr(lib, "hif8_amax_axis_" + sfx)
    enc, dec = getattr(lib, "hif8_encode_axis_" + sfx), getattr(lib, "hif8_decode_axis_" + sfx)

    def scale_sweep(src, n, e_lo, count, rounding_mode, d_err, stream=None):
        _check(sweep(_ptr(src), n, e_lo, count, rounding_mode, _ptr(d_err), _stream(stream)))

    def amax_axis(src, rows, cols, axis, d_amax, stream=None):
        _check(amax(_ptr(src), rows, cols, axis, _ptr(d_amax), _stream(stream)))

    def encode_axis(src, dst, rows, cols, axis, d_scale2, rounding_mode=RM_TA, stream=None):
        _check(enc(_ptr(src), _ptr(dst), rows, cols, axis, _ptr(d_scale2), rounding_mode, _stream(stream)))

    def decode_axis(src, dst, rows, cols, axis, d_scale2, stream=None):
        _check(dec(_ptr(src), _ptr(dst), rows, cols, axis, _ptr(d_scale2), _stream(stream)))

    return scale_sweep, amax_axis, encode_axis, decode_axis


hif8_scale_sweep_f32, hif8_amax_axis_f32, hif8_encode_axis_f32, hif8_decode_axis_f32 = _def_calib("f32")
hif8_scale_sweep_bf16, hif8_amax_axis_bf16, hif8_encode_axis_bf16, hif8_decode_axis_bf16 = _def_calib("bf16")
hif8_scale_sweep_f16, hif8_amax_axis_f16, hif8_encode_axis_f16, hif8_decode_axis_f16 = _def_calib("f16")


def _def_quantize_rows(sfx):
    fn = getattr(lib, "hif8_quantize_rows_" + sfx)

    def quantize_rows(src, dst, rows, cols, d_amax, d_scale2, target=MAX_FINITE, pow2=0, rounding_mode=RM_TA, stream=None):
        _check(fn(_ptr(src), _ptr(dst), rows, cols, target, int(pow2), rounding_mode, _ptr(d_amax), _ptr(d_scale2),
                  _stream(stream)))

    return quantize_rows


hif8_quantize_rows_f32 = _def_quantize_rows("f32")
hif8_quantize_rows_bf16 = _def_quantize_rows("bf16")
hif8_quantize_rows_f16 = _def_quantize_rows("f16")


class PtsState(ctypes.Structure):
    """Mirror of hif8_pts_state."""
    _fields_ = [("d_amax", ctypes.c_void_p), ("d_scale2", ctypes.c_void_p), ("count", ctypes.c_uint32),
                ("interval", ctypes.c_uint32), ("target", ctypes.c_float), ("iteration", ctypes.c_uint64)]


class AlsState(ctypes.Structure):
    """Mirror of hif8_als_state."""
    _fields_ = [("scale", ctypes.c_float), ("window_index", ctypes.c_int32), ("good_steps", ctypes.c_int32),
                ("increases", ctypes.c_int32), ("decrease_streak", ctypes.c_int32)]


def hif8_pts_init(state, d_amax, d_scale2, count, interval=10, target=MAX_FINITE, stream=None):
    _check(lib.hif8_pts_init(ctypes.addressof(state), _ptr(d_amax), _ptr(d_scale2), count, interval, target,
                             _stream(stream)))


def hif8_pts_collects(state):
    return lib.hif8_pts_collects(ctypes.addressof(state))


def hif8_pts_end_iteration(state, stream=None):
    _check(lib.hif8_pts_end_iteration(ctypes.addressof(state), _stream(stream)))


def hif8_als_init(state):
    lib.hif8_als_init(ctypes.addressof(state))


def hif8_als_window(state):
    return lib.hif8_als_window(ctypes.addressof(state))


def hif8_als_update(state, found_overflow):
    _check(lib.hif8_als_update(ctypes.addressof(state), int(bool(found_overflow))))


def hif8_gemm_f32(a_codes, b_codes, out, M, N, K, scale_a=1.0, scale_b=1.0, stream=None):
    _check(lib.hif8_gemm_f32(_ptr(a_codes), _ptr(b_codes), _ptr(out), M, N, K, scale_a, scale_b, _stream(stream)))


def hif8_gemm_bf16(a_codes, b_codes, out, M, N, K, scale_a=1.0, scale_b=1.0, stream=None):
    _check(lib.hif8_gemm_bf16(_ptr(a_codes), _ptr(b_codes), _ptr(out), M, N, K, scale_a, scale_b, _stream(stream)))


def hif8_gemm_f16(a_codes, b_codes, out, M, N, K, scale_a=1.0, scale_b=1.0, stream=None):
    _check(lib.hif8_gemm_f16(_ptr(a_codes), _ptr(b_codes), _ptr(out), M, N, K, scale_a, scale_b, _stream(stream)))


def hif8_gemm_workspace_bytes(M, N, K):
    return lib.hif8_gemm_workspace_bytes(M, N, K)


def _ws_bytes(workspace, workspace_bytes):
    if workspace_bytes is not None:
        return workspace_bytes
    return 0 if workspace is None or isinstance(workspace, int) else workspace.numel() * workspace.element_size()


def _def_gemm_ws(sfx):
    fn = getattr(lib, "hif8_gemm_ws_" + sfx)

    def gemm_ws(a_codes, b_codes, out, M, N, K, workspace, scale_a=1.0, scale_b=1.0, stream=None, workspace_bytes=None):
        _check(fn(_ptr(a_codes), _ptr(b_codes), _ptr(out), M, N, K, scale_a, scale_b, _ptr(workspace),
                  _ws_bytes(workspace, workspace_bytes), _stream(stream)))

    return gemm_ws


hif8_gemm_ws_f32, hif8_gemm_ws_bf16, hif8_gemm_ws_f16 = _def_gemm_ws("f32"), _def_gemm_ws("bf16"), _def_gemm_ws("f16")


def hif8_gemm_ws_sqerr(a_codes, b_codes, ref, M, N, K, scale_a, scale_b, d_err, workspace, stream=None, workspace_bytes=None):
    _check(lib.hif8_gemm_ws_sqerr(_ptr(a_codes), _ptr(b_codes), _ptr(ref), M, N, K, scale_a, scale_b, _ptr(d_err),
                                  _ptr(workspace), _ws_bytes(workspace, workspace_bytes), _stream(stream)))


def hif8_gemm_sqerr(a_codes, b_codes, ref, M, N, K, scale_a, scale_b, d_err, stream=None):
    _check(lib.hif8_gemm_sqerr(_ptr(a_codes), _ptr(b_codes), _ptr(ref), M, N, K, scale_a, scale_b, _ptr(d_err),
                               _stream(stream)))


def hif8_gemm_set_variant(variant):
    _check(lib.hif8_gemm_set_variant(variant))


def hif8_expanded_ld(K):
    return lib.hif8_expanded_ld(K)


def hif8_expand_bf16(codes, rows, K, dst, ld, stream=None):
    _check(lib.hif8_expand_bf16(_ptr(codes), rows, K, _ptr(dst), ld, _stream(stream)))


def hif8_expand_bf16_t(codes, rows, cols, dst, ld, stream=None):
    _check(lib.hif8_expand_bf16_t(_ptr(codes), rows, cols, _ptr(dst), ld, _stream(stream)))


def hif8_gemm_expanded_f32(a, b, out, M, N, K, ld, scale_a=1.0, scale_b=1.0, stream=None):
    _check(lib.hif8_gemm_expanded_f32(_ptr(a), _ptr(b), _ptr(out), M, N, K, ld, scale_a, scale_b, _stream(stream)))


def hif8_gemm_expanded_bf16(a, b, out, M, N, K, ld, scale_a=1.0, scale_b=1.0, stream=None):
    _check(lib.hif8_gemm_expanded_bf16(_ptr(a), _ptr(b), _ptr(out), M, N, K, ld, scale_a, scale_b, _stream(stream)))


def hif8_gemm_expanded_f16(a, b, out, M, N, K, ld, scale_a=1.0, scale_b=1.0, stream=None):
    _check(lib.hif8_gemm_expanded_f16(_ptr(a), _ptr(b), _ptr(out), M, N, K, ld, scale_a, scale_b, _stream(stream)))


def hif8_gemm_expanded_sqerr(a, b, ref, M, N, K, ld, scale_a, scale_b, d_err, stream=None):
    _check(lib.hif8_gemm_expanded_sqerr(_ptr(a), _ptr(b), _ptr(ref), M, N, K, ld, scale_a, scale_b, _ptr(d_err),
                                        _stream(stream)))


def hif8_calibrate_workspace_bytes(M, N, K, ea_count=10, ew_count=10):
    return lib.hif8_calibrate_workspace_bytes(M, N, K, ea_count, ew_count)


def _def_calibrate(sfx):
    fn = getattr(lib, "hif8_calibrate_layer_" + sfx)

    def calibrate_layer(a, w, o_ref, M, N, K, ea_lo, ea_count, ew_lo, ew_count, rounding_mode, workspace,
                        workspace_bytes, d_err, d_best=None, stream=None):
        _check(fn(_ptr(a), _ptr(w), _ptr(o_ref), M, N, K, ea_lo, ea_count, ew_lo, ew_count, rounding_mode,
                  _ptr(workspace), workspace_bytes, _ptr(d_err), _ptr(d_best), _stream(stream)))

    return calibrate_layer


hif8_calibrate_layer_f32 = _def_calibrate("f32")
hif8_calibrate_layer_bf16 = _def_calibrate("bf16")
hif8_calibrate_layer_f16 = _def_calibrate("f16")


def hif8_set_tuning(key, value):
    _check(lib.hif8_set_tuning(key, value))


def hif8_get_tuning(key):
    return lib.hif8_get_tuning(key)


def hif8_diag_stream(src, dst, n_groups, out_bytes_per_lane, stream=None):
    _check(lib.hif8_diag_stream(_ptr(src), _ptr(dst), n_groups, out_bytes_per_lane, _stream(stream)))
