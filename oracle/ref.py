"""ctypes front end of the C++ oracle (test infrastructure, not product code).

Every function takes and returns numpy arrays on the host.  The arithmetic
lives in mqgrad_oracle.cpp; this file only marshals arguments.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        # MQGRAD_ORACLE_LIB: load another build of the oracle (used to check that planted mistakes fail the pins)
        path = os.environ.get("MQGRAD_ORACLE_LIB") or _build.build(force=False)
        L = C.CDLL(path)
        u8p, u32p, f32p, f64p = (C.POINTER(C.c_uint8), C.POINTER(C.c_uint32),
                                 C.POINTER(C.c_float), C.POINTER(C.c_double))
        L.orc_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.orc_philox4x32_10.restype = None
        L.orc_uniform16.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64]
        L.orc_uniform16.restype = C.c_uint32
        L.orc_num_buckets.argtypes = [C.c_uint64, C.c_uint32]
        L.orc_num_buckets.restype = C.c_uint64
        L.orc_packed_words.argtypes = [C.c_uint64, C.c_uint32]
        L.orc_packed_words.restype = C.c_uint64
        L.orc_bucket_scales.argtypes = [f32p, C.c_uint64, C.c_uint32, C.c_int, f32p]
        L.orc_bucket_scales.restype = None
        L.orc_round_code.argtypes = [C.c_float, C.c_float, C.c_uint32, C.c_uint32]
        L.orc_round_code.restype = C.c_uint32
        L.orc_level_value.argtypes = [C.c_uint32, C.c_float, C.c_uint32]
        L.orc_level_value.restype = C.c_float
        L.orc_quantize_codes.argtypes = [f32p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64,
                                         C.c_uint32, C.c_uint32, C.c_uint64, f32p, u8p]
        L.orc_quantize_codes.restype = None
        L.orc_pack.argtypes = [u8p, C.c_uint64, C.c_uint32, u32p]
        L.orc_pack.restype = None
        L.orc_unpack.argtypes = [u32p, C.c_uint64, C.c_uint32, u8p]
        L.orc_unpack.restype = None
        L.orc_quantize.argtypes = [f32p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int, C.c_uint64,
                                   C.c_uint32, C.c_uint32, C.c_uint64, f32p, u32p, f32p, u8p]
        L.orc_quantize.restype = None
        L.orc_dequantize.argtypes = [u32p, f32p, C.c_uint64, C.c_uint32, C.c_uint32, f32p, u8p]
        L.orc_dequantize.restype = None
        pp_u32, pp_f32 = C.POINTER(u32p), C.POINTER(f32p)
        L.orc_aggregate_update.argtypes = [pp_u32, pp_f32, C.c_uint32, C.c_uint64, C.c_uint32,
                                           C.c_uint32, C.c_float, f32p]
        L.orc_aggregate_update.restype = None
        L.orc_aggregate_update_f64.argtypes = [pp_u32, pp_f32, C.c_uint32, C.c_uint64, C.c_uint32,
                                               C.c_uint32, C.c_double, f32p, f64p]
        L.orc_aggregate_update_f64.restype = None
        L.orc_aggregate_sum.argtypes = [pp_u32, pp_f32, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, f32p]
        L.orc_aggregate_sum.restype = None
        L.orc_aggregate_requantize.argtypes = [pp_u32, pp_f32, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32,
                                               C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64, u32p, f32p, f32p, u8p]
        L.orc_aggregate_requantize.restype = None
        L.orc_dequantize_update.argtypes = [u32p, f32p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_float, f32p]
        L.orc_dequantize_update.restype = None
        L.orc_aggregate_mean.argtypes = [pp_u32, pp_f32, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, f32p]
        L.orc_aggregate_mean.restype = None
        L.orc_average_update_raw.argtypes = [pp_f32, C.c_uint32, C.c_uint64, C.c_float, f32p]
        L.orc_average_update_raw.restype = None
        L.orc_minmax_ranges.argtypes = [f32p, C.c_uint64, C.c_uint32, f32p]
        L.orc_minmax_ranges.restype = None
        L.orc_nearest_code.argtypes = [C.c_float, C.c_float, C.c_float, C.c_uint32]
        L.orc_nearest_code.restype = C.c_uint32
        L.orc_minmax_level_value.argtypes = [C.c_uint32, C.c_float, C.c_float, C.c_uint32]
        L.orc_minmax_level_value.restype = C.c_float
        L.orc_quantize_minmax.argtypes = [f32p, C.c_uint64, C.c_uint32, C.c_uint32, u32p, f32p, u8p]
        L.orc_quantize_minmax.restype = None
        L.orc_dequantize_minmax.argtypes = [u32p, f32p, C.c_uint64, C.c_uint32, C.c_uint32, f32p]
        L.orc_dequantize_minmax.restype = None
        L.orc_aggregate_update_minmax.argtypes = [pp_u32, pp_f32, C.c_uint32, C.c_uint64, C.c_uint32,
                                                  C.c_uint32, C.c_float, f32p]
        L.orc_aggregate_update_minmax.restype = None
        L.orc_aggregate_sum_minmax.argtypes = [pp_u32, pp_f32, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, f32p]
        L.orc_aggregate_sum_minmax.restype = None
        L.orc_aggregate_requantize_minmax.argtypes = [pp_u32, pp_f32, C.c_uint32, C.c_uint64, C.c_uint32,
                                                      C.c_uint32, u32p, f32p]
        L.orc_aggregate_requantize_minmax.restype = None
        _lib = L
    return _lib


SCALE_MAXABS = 0
SCALE_L2 = 1


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    assert ctr.shape == (4,) and key.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(ctr, C.c_uint32), _p(key, C.c_uint32), _p(out, C.c_uint32))
    return out


def uniform16(seed, iteration, worker, e):
    return int(lib().orc_uniform16(seed, iteration, worker, e))


def num_buckets(n, bucket):
    return int(lib().orc_num_buckets(n, bucket))


def packed_words(n, bits):
    return int(lib().orc_packed_words(n, bits))


def bucket_scales(g, bucket, scale_mode=SCALE_MAXABS):
    g = _f32(g)
    out = np.empty(num_buckets(g.size, bucket), dtype=np.float32)
    lib().orc_bucket_scales(_p(g, C.c_float), g.size, bucket, scale_mode, _p(out, C.c_float))
    return out


def round_code(x, s, bits, h):
    return int(lib().orc_round_code(float(np.float32(x)), float(np.float32(s)), bits, h))


def level_value(k, s, bits):
    return np.float32(lib().orc_level_value(k, float(np.float32(s)), bits))


def quantize_codes(g, bits, bucket, seed, iteration, worker, elem_base, scales):
    g = _f32(g)
    scales = _f32(scales)
    assert scales.size == num_buckets(g.size, bucket)
    codes = np.empty(g.size, dtype=np.uint8)
    lib().orc_quantize_codes(_p(g, C.c_float), g.size, bits, bucket, seed, iteration, worker,
                             elem_base, _p(scales, C.c_float), _p(codes, C.c_uint8))
    return codes


def pack(codes, bits):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    words = np.empty(packed_words(codes.size, bits), dtype=np.uint32)
    lib().orc_pack(_p(codes, C.c_uint8), codes.size, bits, _p(words, C.c_uint32))
    return words


def unpack(words, n, bits):
    words = np.ascontiguousarray(words, dtype=np.uint32)
    assert words.size >= packed_words(n, bits)
    codes = np.empty(n, dtype=np.uint8)
    lib().orc_unpack(_p(words, C.c_uint32), n, bits, _p(codes, C.c_uint8))
    return codes


def quantize(g, bits, bucket, seed, iteration=0, worker=0, elem_base=0, scale_mode=SCALE_MAXABS,
             scales_in=None):
    """Worker side, whole.  Returns (packed uint32[words], scales float32[nb])."""
    g = _f32(g)
    n = g.size
    packed = np.empty(packed_words(n, bits), dtype=np.uint32)
    scales = np.empty(num_buckets(n, bucket), dtype=np.float32)
    tmp = np.empty(max(n, 1), dtype=np.uint8)
    sin = None
    if scales_in is not None:
        scales_in = _f32(scales_in)
        assert scales_in.size == scales.size
        sin = _p(scales_in, C.c_float)
    lib().orc_quantize(_p(g, C.c_float), n, bits, bucket, scale_mode, seed, iteration, worker,
                       elem_base, sin, _p(packed, C.c_uint32), _p(scales, C.c_float),
                       _p(tmp, C.c_uint8))
    return packed, scales


def dequantize(packed, scales, n, bits, bucket):
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    scales = _f32(scales)
    out = np.empty(n, dtype=np.float32)
    tmp = np.empty(max(n, 1), dtype=np.uint8)
    lib().orc_dequantize(_p(packed, C.c_uint32), _p(scales, C.c_float), n, bits, bucket,
                         _p(out, C.c_float), _p(tmp, C.c_uint8))
    return out


def _ptr_arrays(packed_list, scales_list):
    W = len(packed_list)
    pk = [np.ascontiguousarray(p, dtype=np.uint32) for p in packed_list]
    sc = [_f32(s) for s in scales_list]
    u32p, f32p = C.POINTER(C.c_uint32), C.POINTER(C.c_float)
    pa = (u32p * W)(*[_p(p, C.c_uint32) for p in pk])
    sa = (f32p * W)(*[_p(s, C.c_float) for s in sc])
    return pk, sc, pa, sa


def aggregate_update(packed_list, scales_list, n, bits, bucket, lr, params):
    """Server side: returns the updated copy of `params` (fp32)."""
    W = len(packed_list)
    assert W == len(scales_list) and W >= 1
    pk, sc, pa, sa = _ptr_arrays(packed_list, scales_list)
    out = np.array(params, dtype=np.float32, copy=True).reshape(-1)
    assert out.size == n
    lib().orc_aggregate_update(pa, sa, W, n, bits, bucket, float(np.float32(lr)), _p(out, C.c_float))
    return out


def aggregate_update_f64(packed_list, scales_list, n, bits, bucket, lr, params):
    """The same server step from its plain definition in fp64 (no fp32 rounding)."""
    W = len(packed_list)
    pk, sc, pa, sa = _ptr_arrays(packed_list, scales_list)
    pin = _f32(params).reshape(-1)
    out = np.empty(n, dtype=np.float64)
    lib().orc_aggregate_update_f64(pa, sa, W, n, bits, bucket, float(lr), _p(pin, C.c_float),
                                   _p(out, C.c_double))
    return out


def aggregate_sum(packed_list, scales_list, n, bits, bucket):
    """fp32 sum over workers of the de-quantized gradients (ordered fma chain)."""
    W = len(packed_list)
    pk, sc, pa, sa = _ptr_arrays(packed_list, scales_list)
    out = np.empty(n, dtype=np.float32)
    lib().orc_aggregate_sum(pa, sa, W, n, bits, bucket, _p(out, C.c_float))
    return out


def aggregate_requantize(packed_list, scales_list, n, bits, bucket, seed, iteration=0, worker=0, elem_base=0):
    """Server side of the full exchange: quantized mean.  Returns (packed uint32[words], scales float32[nb])."""
    W = len(packed_list)
    pk, sc, pa, sa = _ptr_arrays(packed_list, scales_list)
    packed = np.empty(packed_words(n, bits), dtype=np.uint32)
    scales = np.empty(num_buckets(n, bucket), dtype=np.float32)
    tmp_f = np.empty(max(n, 1), dtype=np.float32)
    tmp_c = np.empty(max(n, 1), dtype=np.uint8)
    lib().orc_aggregate_requantize(pa, sa, W, n, bits, bucket, seed, iteration, worker, elem_base,
                                   _p(packed, C.c_uint32), _p(scales, C.c_float), _p(tmp_f, C.c_float),
                                   _p(tmp_c, C.c_uint8))
    return packed, scales


def dequantize_update(packed, scales, n, bits, bucket, lr, params):
    """Worker side of the full exchange: returns params - lr * dequantize(packed, scales)."""
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    scales = _f32(scales)
    out = np.array(params, dtype=np.float32, copy=True).reshape(-1)
    assert out.size == n
    lib().orc_dequantize_update(_p(packed, C.c_uint32), _p(scales, C.c_float), n, bits, bucket,
                                float(np.float32(lr)), _p(out, C.c_float))
    return out


def average_update_raw(grads, lr, params):
    """Uncompressed layers: params - (lr / W) * sum_w grads[w], summed in worker order in fp32."""
    W = len(grads)
    gs = [_f32(g).reshape(-1) for g in grads]
    n = gs[0].size
    f32p = C.POINTER(C.c_float)
    ga = (f32p * W)(*[_p(g, C.c_float) for g in gs])
    out = np.array(params, dtype=np.float32, copy=True).reshape(-1)
    assert out.size == n and all(g.size == n for g in gs)
    lib().orc_average_update_raw(ga, W, n, float(np.float32(lr)), _p(out, C.c_float))
    return out


# ---- the footnote read literally: deterministic min/max range-linear encode ---------------------------

def minmax_ranges(g, bucket):
    """Per-bucket [min, max], interleaved: ranges[2k], ranges[2k+1]."""
    g = _f32(g).reshape(-1)
    out = np.zeros(2 * num_buckets(g.size, bucket), dtype=np.float32)
    if g.size:
        lib().orc_minmax_ranges(_p(g, C.c_float), g.size, bucket, _p(out, C.c_float))
    return out


def nearest_code(x, mn, mx, bits):
    return int(lib().orc_nearest_code(float(np.float32(x)), float(np.float32(mn)), float(np.float32(mx)), bits))


def encode_minmax_given_range(values, bits, mn, mx):
    """Packed words of `values` encoded over the given [mn, mx] (one nearest-level call per element)."""
    v = _f32(values).reshape(-1)
    codes = np.array([nearest_code(x, mn, mx, bits) for x in v], dtype=np.uint8)
    return pack(codes, bits)


def minmax_level_value(k, mn, mx, bits):
    return np.float32(lib().orc_minmax_level_value(int(k), float(np.float32(mn)), float(np.float32(mx)), bits))


def quantize_minmax(g, bits, bucket, return_codes=False):
    g = _f32(g).reshape(-1)
    n = g.size
    packed = np.zeros(packed_words(n, bits), dtype=np.uint32)
    ranges = np.zeros(2 * num_buckets(n, bucket), dtype=np.float32)
    codes = np.zeros(max(n, 1), dtype=np.uint8)
    if n:
        lib().orc_quantize_minmax(_p(g, C.c_float), n, bits, bucket, _p(packed, C.c_uint32), _p(ranges, C.c_float),
                                  _p(codes, C.c_uint8))
    if return_codes:
        return packed, ranges, codes[:n]
    return packed, ranges


def dequantize_minmax(packed, ranges, n, bits, bucket):
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    ranges = _f32(ranges)
    out = np.zeros(n, dtype=np.float32)
    if n:
        lib().orc_dequantize_minmax(_p(packed, C.c_uint32), _p(ranges, C.c_float), n, bits, bucket, _p(out, C.c_float))
    return out


def aggregate_update_minmax(packed_list, ranges_list, n, bits, bucket, lr, params):
    pk, rg, pa, sa = _ptr_arrays(packed_list, ranges_list)
    out = np.array(params, dtype=np.float32, copy=True).reshape(-1)
    assert out.size == n
    lib().orc_aggregate_update_minmax(pa, sa, len(packed_list), n, bits, bucket, float(np.float32(lr)),
                                      _p(out, C.c_float))
    return out


def aggregate_sum_minmax(packed_list, ranges_list, n, bits, bucket):
    """fp32 sum, in worker order, of the workers' de-quantized gradients ([min, max] encoding)."""
    pk, rg, pa, sa = _ptr_arrays(packed_list, ranges_list)
    out = np.zeros(n, dtype=np.float32)
    if n:
        lib().orc_aggregate_sum_minmax(pa, sa, len(packed_list), n, bits, bucket, _p(out, C.c_float))
    return out


def aggregate_requantize_minmax(packed_list, ranges_list, n, bits, bucket):
    """Server side of the full exchange with the [min, max] encoding: (packed, ranges) of the mean."""
    pk, rg, pa, sa = _ptr_arrays(packed_list, ranges_list)
    packed = np.zeros(packed_words(n, bits), dtype=np.uint32)
    ranges = np.zeros(2 * num_buckets(n, bucket), dtype=np.float32)
    if n:
        lib().orc_aggregate_requantize_minmax(pa, sa, len(packed_list), n, bits, bucket, _p(packed, C.c_uint32),
                                              _p(ranges, C.c_float))
    return packed, ranges


def aggregate_mean(packed_list, scales_list, n, bits, bucket):
    """Mean over the workers of their de-quantized gradients (fp32 chain in worker order, one division)."""
    pk, sc, pa, sa = _ptr_arrays(packed_list, scales_list)
    out = np.zeros(n, dtype=np.float32)
    if n:
        lib().orc_aggregate_mean(pa, sa, len(packed_list), n, bits, bucket, _p(out, C.c_float))
    return out
